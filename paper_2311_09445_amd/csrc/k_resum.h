// Re-summation of node ranges after inserts and of the top heights an update left stale.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// re-summation
// ---------------------------------------------------------------------------------
// Recompute nodes [a, a+count) of height h from their children.  grid (x, T).
template <int LOGK>
__global__ void k_resum_dense(Geom g, uint32_t h, uint32_t a, uint32_t count) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t t = blockIdx.y;
  const uint32_t gt = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t e = gt / LPS;
  const unsigned q = gt % LPS;
  const bool active = e < count;
  const uint32_t node = a + (active ? e : 0u);
  const float sum = group_sum<LOGK>(g.level[h - 1] + (size_t)t * g.stride[h - 1] + (size_t)node * K, q);
  if (active && q == 0) g.level[h][(size_t)t * g.stride[h] + node] = sum;
}

// One workgroup per tree finishes heights h_start .. H over the node ranges in r (given at
// height h_start and narrowed by K per height).
// The workgroup recomputes the nodes of height h in the two ranges of r from their children.
template <int LOGK>
__device__ __forceinline__ void resum_level(const Geom& g, uint32_t t, uint32_t h, const Range2& r) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const unsigned q = threadIdx.x % LPS;
  const uint32_t grp = threadIdx.x / LPS;
  const uint32_t ngrp = blockDim.x / LPS;
  const float* child = g.level[h - 1] + (size_t)t * g.stride[h - 1];
  float* par = g.level[h] + (size_t)t * g.stride[h];
  for (int part = 0; part < 2; ++part) {
    const uint32_t a = part ? r.a1 : r.a0, b = part ? r.b1 : r.b0;
    for (uint32_t base = a; base < b; base += ngrp) {
      const uint32_t e = base + grp;
      const bool ok = e < b;
      const uint32_t node = ok ? e : a;
      const float sum = group_sum<LOGK>(child + (size_t)node * K, q);
      if (ok && q == 0) par[node] = sum;
    }
  }
}

template <int LOGK>
__global__ void k_resum_tail(Geom g, uint32_t h_start, Range2 r) {
  const uint32_t t = blockIdx.x;
  for (uint32_t h = h_start; h <= g.H; ++h) {
    resum_level<LOGK>(g, t, h, r);
    __syncthreads();
    if (r.b0 > r.a0) { r.a0 >>= LOGK; r.b0 = ((r.b0 - 1) >> LOGK) + 1; }
    if (r.b1 > r.a1) { r.a1 >>= LOGK; r.b1 = ((r.b1 - 1) >> LOGK) + 1; }
  }
}

// A single workgroup handles a height while the groups it must read stay below this many floats.
constexpr uint64_t kTailFloats = 16384;

template <int LOGK>
static hipError_t launch_resum_ranges_k(const Geom& g, const Tuning& tn, Range2 r, hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t block = tn.update_block;
  // r holds touched leaf slots; move to height 1
  uint32_t h = 1;
  for (; h <= g.H; ++h) {
    if (r.b0 > r.a0) { r.a0 >>= LOGK; r.b0 = ((r.b0 - 1) >> LOGK) + 1; }
    if (r.b1 > r.a1) { r.a1 >>= LOGK; r.b1 = ((r.b1 - 1) >> LOGK) + 1; }
    const uint64_t nodes = (uint64_t)(r.b0 - r.a0) + (r.b1 - r.a1);
    if (nodes * K <= kTailFloats) break;
    for (int part = 0; part < 2; ++part) {
      const uint32_t a = part ? r.a1 : r.a0, b = part ? r.b1 : r.b0;
      if (b <= a) continue;
      const uint64_t threads = (uint64_t)(b - a) * LPS;
      PER_LAUNCH(KID_RESUM_DENSE, k_resum_dense<LOGK>, dim3((uint32_t)((threads + block - 1) / block), g.T),
                 dim3(block), 0, s, g, h, a, b - a);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  if (h <= g.H) {
    PER_LAUNCH(KID_RESUM_TAIL, k_resum_tail<LOGK>, dim3(g.T), dim3(1024), 0, s, g, h, r);
    return hipGetLastError();
  }
  return hipSuccess;
}

// Recompute every node above height hb (after an update that left them stale).
template <int LOGK>
static hipError_t launch_resum_top_k(const Geom& g, const Tuning& tn, uint32_t hb, hipStream_t s) {
  if (hb >= g.H) return hipSuccess;
  Range2 r{0, g.n[hb + 1], 0, 0};
  PER_LAUNCH(KID_RESUM_TAIL, k_resum_tail<LOGK>, dim3(g.T), dim3(1024), 0, s, g, hb + 1, r);
  return hipGetLastError();
}

hipError_t launch_resum_top(const Geom& g, const Tuning& tn, uint32_t hb, hipStream_t s) {
#define CALL(L) launch_resum_top_k<L>(g, tn, hb, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

hipError_t launch_resum_ranges(const Geom& g, const Tuning& tn, Range2 r0, hipStream_t s) {
#define CALL(L) launch_resum_ranges_k<L>(g, tn, r0, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}
