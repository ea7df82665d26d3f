// Priority update in the paper's own form: a change added along every path.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// priority update in the paper's form: add a change to every node of the path (Section V-A)
// ---------------------------------------------------------------------------------
// One lane per element; the node of every height on the element's path gets the change added with
// a hardware float atomic, root first and leaf last as the paper orders it.  The few topmost heights
// (all heights >= h_lds, acc_floats nodes in total) would take thousands of atomics on the same
// address, so a workgroup first adds its elements' changes up in LDS (the root even per wave in
// registers) and then issues one atomic per node it touched.  The order in which changes meet in a
// node is not fixed, so results agree with a sequential pass only up to fp32 rounding.
__global__ void k_update_delta(Geom g, uint32_t B, uint32_t size, const uint32_t* __restrict__ idx,
                               const float* __restrict__ delta, uint32_t h_lds, uint32_t acc_floats) {
  extern __shared__ __attribute__((aligned(16))) float acc[];
  const uint32_t t = blockIdx.y;
  const uint32_t H = g.H;
  for (uint32_t e = threadIdx.x; e < acc_floats; e += blockDim.x) acc[e] = 0.0f;
  __syncthreads();
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t flags = 0;
  float d = 0.0f;
  uint32_t i = 0;
  bool ok = false;
  if (j < B) {
    i = idx[(size_t)t * B + j];
    d = delta[(size_t)t * B + j];
    if (!(i < size)) flags |= 1u;
    else if (!__builtin_isfinite(d)) flags |= 2u;
    else ok = true;
  }
  if (!ok) d = 0.0f;
  // the root: one LDS add per wave
  float wave_sum = d;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) wave_sum += __shfl_xor(wave_sum, m);
  uint32_t off_root = 0;   // the LDS copy holds heights h_lds .. H in that order
  for (uint32_t h = h_lds; h < H; ++h) off_root += g.n[h];
  if (h_lds <= H && (threadIdx.x & 63u) == 0 && wave_sum != 0.0f) atomicAdd(&acc[off_root], wave_sum);
  if (ok) {
    uint32_t off = off_root;
    for (uint32_t h = H; h-- > 0;) {   // heights H-1 .. 0 (the root is done above, or here when it is not in LDS)
      const uint32_t node = i >> (h * g.logK);
      if (h >= h_lds) {
        off -= g.n[h];
        atomicAdd(&acc[off + node], d);
      } else {
        unsafeAtomicAdd(g.level[h] + (size_t)t * g.stride[h] + node, d);
      }
    }
    if (h_lds > H) unsafeAtomicAdd(g.level[H] + (size_t)t * g.stride[H], d);
  }
  if (flags) atomicOr(&g.status[t], flags);
  __syncthreads();
  uint32_t off = 0;
  for (uint32_t h = h_lds; h <= H; ++h) {
    float* lvl = g.level[h] + (size_t)t * g.stride[h];
    for (uint32_t e = threadIdx.x; e < g.n[h]; e += blockDim.x) {
      const float v = acc[off + e];
      if (v != 0.0f) unsafeAtomicAdd(lvl + e, v);
    }
    off += g.n[h];
  }
}

constexpr uint32_t kDeltaLdsFloats = 4096;

hipError_t launch_update_delta(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, const uint32_t* idx,
                               const float* delta, hipStream_t s) {
  // heights h_lds .. H go through LDS: as many of the topmost heights as fit
  uint32_t h_lds = g.H + 1, floats = 0;
  while (h_lds > 1 && floats + g.n[h_lds - 1] <= kDeltaLdsFloats) {
    --h_lds;
    floats += g.n[h_lds];
  }
  const uint32_t block = tn.update_block;
  PER_LAUNCH(KID_UPDATE_DELTA, k_update_delta, dim3((B + block - 1) / block, g.T), dim3(block), (size_t)floats * 4, s, g,
             B, size, idx, delta, h_lds, floats);
  return hipGetLastError();
}
