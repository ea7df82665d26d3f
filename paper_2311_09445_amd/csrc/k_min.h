// Companion minimum of the sum tree: rebuild from the leaves, reduction to one value per tree.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// smallest positive priority of the whole buffer
// ---------------------------------------------------------------------------------
// Importance weights scaled by the largest weight of the WHOLE buffer (prioritized experience replay,
// cited in Section II-A, scales by 1 / max w; implementations keep a min tree beside the sum tree for
// it) need the smallest positive leaf of the tree.  A minimum does not depend on the order or shape
// of its reduction, so the companion structure need not mirror the sum tree: min1 holds the
// minimum under every height-1 node, kept current by the kernels that rewrite leaves of few nodes (the
// update's tree pass, small inserts); everything else marks it stale on the host and k_min_rebuild
// recomputes it from the leaves when it is next needed.  k_min_reduce folds min1 into a few partial
// minima per tree before a sampling call that wants it.

// min1 of every height-1 node from its K leaves; LPS lanes per node.
template <int LOGK>
__global__ void __launch_bounds__(256)
k_min_rebuild(Geom g) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t t = blockIdx.y;
  const unsigned q = threadIdx.x % LPS;
  const uint64_t ngrp = (uint64_t)gridDim.x * blockDim.x / LPS;
  const float* leaves = g.level[0] + (size_t)t * g.stride[0];
  uint32_t* min1 = g.min1 + (size_t)t * g.min1_stride;
  const uint32_t n1 = g.n[1];
  for (uint64_t node = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) / LPS; node < n1; node += ngrp) {
    const uint32_t m = group_min_positive<LOGK>(leaves + node * K, q);   // (the lanes of a group share their node)
    if (q == 0) min1[node] = m;
  }
}

// vmin_buf[t][b] = minimum of the part of min1 of tree t that workgroup b has swept.  Plain stores, one
// per workgroup, so nothing has to be armed beforehand; the readers fold the gridDim.x partial minima.
__global__ void __launch_bounds__(256)
k_min_reduce(Geom g) {
  __shared__ uint32_t s_m[4];
  const uint32_t t = blockIdx.y;
  const uint32_t* min1 = g.min1 + (size_t)t * g.min1_stride;
  const uint32_t n1 = g.n[1];
  uint32_t m = kNoMin;
  // four entries per lane and load (the launch gives every lane one load for all but huge trees); the
  // entries beyond n1 up to the stride are not minima and are not read
  const uint64_t lanes = (uint64_t)gridDim.x * blockDim.x, lane0 = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t n4 = n1 / 4;
  const uint4* min4 = reinterpret_cast<const uint4*>(min1);
  for (uint64_t i = lane0; i < n4; i += lanes) {
    const uint4 v = min4[i];
    m = min_u32(min_u32(m, min_u32(v.x, v.y)), min_u32(v.z, v.w));
  }
  for (uint64_t i = (uint64_t)n4 * 4 + lane0; i < n1; i += lanes) m = min_u32(m, min1[i]);
  m = wave_min_u32(m);
  if ((threadIdx.x & 63u) == 0) s_m[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0)
    g.vmin_buf[(size_t)t * kMinParts + blockIdx.x] = min_u32(min_u32(s_m[0], s_m[1]), min_u32(s_m[2], s_m[3]));
}

template <int LOGK>
static hipError_t launch_min_rebuild_k(const Geom& g, const Tuning& tn, hipStream_t s) {
  const uint64_t lanes = (uint64_t)g.n[1] * Fan<LOGK>::LPS;
  uint64_t blocks = (lanes + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  PER_LAUNCH(KID_MIN_REBUILD, k_min_rebuild<LOGK>, dim3((unsigned)blocks, g.T), dim3(256), 0, s, g);
  return hipGetLastError();
}

hipError_t launch_min_rebuild(const Geom& g, const Tuning& tn, hipStream_t s) {
#define CALL(L) launch_min_rebuild_k<L>(g, tn, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

hipError_t launch_min_reduce(const Geom& g, const Tuning& tn, uint32_t* weight_mode, hipStream_t s) {
  uint64_t blocks = ((uint64_t)g.n[1] + 1023) / 1024;   // four entries per lane
  if (blocks > kMinParts) blocks = kMinParts;
  PER_LAUNCH(KID_MIN_REDUCE, k_min_reduce, dim3((unsigned)blocks, g.T), dim3(256), 0, s, g);
  *weight_mode = kWeightBufferNorm | ((uint32_t)blocks << kWeightPartsShift);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// the same reduction with its partial minima in a static device array
// ---------------------------------------------------------------------------------
// For callers that may not hand over or allocate scratch memory at all.  The partial minima of k_min_reduce
// ([tree][kMinParts] words) live in this array instead of the caller's arena; every GPU the library runs on
// holds its own copy until the process ends.  In host code the array's name is only a stand-in: its address
// on a device comes from hipGetSymbolAddress, asked once per device with that device current (at per_create)
// and kept; the kernels take that address as an argument, as they take the arena's buffer.
static __device__ __align__(256) uint32_t scratch[kStaticMinTrees * kMinParts];
static uint32_t* g_scratch_addr[kMaxDevices];

hipError_t static_scratch_address(int device, uint32_t** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_addr[device]) {
    int current = -1;
    hipError_t e = hipGetDevice(&current);
    if (e != hipSuccess) return e;
    if (current != device) return hipErrorInvalidDevice;   // the symbol's address belongs to the current device
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_addr[device] = static_cast<uint32_t*>(ptr);
  }
  *out = g_scratch_addr[device];
  return hipSuccess;
}
