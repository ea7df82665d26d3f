// HIP kernels (gfx950) for the prioritized replay buffer's K-ary sum tree.
//
// Bit-exactness rule used everywhere: the sum of a K-child group is the balanced
// pairwise sum over child positions, ((c0+c1)+(c2+c3))+..., and the descent
// inside a group is the binary walk over those implicit partial sums.  A group is
// handled by LPS = max(1, K/4) adjacent lanes: each lane loads four children
// (one 16-byte load, so a group is one coalesced 4K-byte access), sums them in
// registers, and an xor-butterfly over the LPS lanes yields every larger block
// sum.  IEEE addition is commutative, so both partners of a butterfly step get
// identical bits.
#include "per_geom.h"

#include <hip/hip_ext.h>

#include <type_traits>

namespace per {

// ---------------------------------------------------------------------------------
// per-kernel timing
// ---------------------------------------------------------------------------------
const char* kernel_name(int kid) {
  static const char* const names[KID_COUNT] = {
      "k_fill_u32", "k_sample", "k_weights", "k_rows_gather", "k_finish", "k_rows_scatter", "k_insert_leaves",
      "k_resum_dense", "k_resum_tail", "k_update_claim", "k_update_tree", "k_tree_finish", "k_update_delta",
      "k_get_priority", "k_insert_small", "k_run_steps"};
  return kid >= 0 && kid < KID_COUNT ? names[kid] : "?";
}

void Profiler::reset() {
  for (Rec& r : recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  recs.clear();
  for (int k = 0; k < KID_COUNT; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
}

hipError_t Profiler::collect() {
  hipError_t first = hipSuccess;
  for (Rec& r : recs) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e == hipSuccess) { total_ms[r.kid] += ms; launches[r.kid] += 1; }
    else if (first == hipSuccess) first = e;
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  recs.clear();
  return first;
}

// When profiling is on, the launch carries its own pair of events (hipExtLaunchKernelGGL stamps
// them at the start and at the end of the kernel's execution, not at enqueue time), so the
// durations are those of the kernels themselves.
bool Profiler::begin(int kid, hipEvent_t* start, hipEvent_t* stop) {
  if (!on) return false;
  Rec r;
  r.kid = kid;
  if (hipEventCreate(&r.start) != hipSuccess) return false;
  if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return false; }
  recs.push_back(r);
  *start = r.start;
  *stop = r.stop;
  return true;
}

#define PER_LAUNCH(KID, KERNEL, GRID, BLOCK, LDS, STREAM, ...)                                     \
  do {                                                                                             \
    hipEvent_t ev_start_, ev_stop_;                                                                \
    if (tn.prof && tn.prof->begin(KID, &ev_start_, &ev_stop_))                                     \
      hipExtLaunchKernelGGL((KERNEL), GRID, BLOCK, LDS, STREAM, ev_start_, ev_stop_, 0, __VA_ARGS__); \
    else                                                                                           \
      KERNEL<<<GRID, BLOCK, LDS, STREAM>>>(__VA_ARGS__);                                           \
  } while (0)

// ---------------------------------------------------------------------------------
// optional in-kernel time stamps (development builds with -DPER_TRACE only)
// ---------------------------------------------------------------------------------
#ifdef PER_TRACE
// Time stamps are kept in registers and stored when the kernel ends, so that taking them does
// not add memory traffic (or waits for it) to the phases being timed.
constexpr int kTraceMarks = 16, kTraceBlocks = 2048;
__device__ unsigned long long g_trace[kTraceBlocks * kTraceMarks];
#define PER_TRACE_DECL unsigned long long tm_[kTraceMarks] = {}
#define PER_MARK(i) do { tm_[(i)] = wall_clock64(); } while (0)
#define PER_MARK_HWID(i) /* XCC id and HW_ID (SE, CU, SIMD, wave slot) of the calling wave */    \
  do {                                                                                         \
    tm_[(i)] = ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |        \
               (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);                            \
  } while (0)
#define PER_MARK_DYN(i)                                                                        \
  do {                                                                                         \
    const unsigned long long now_ = wall_clock64();                                            \
    _Pragma("unroll") for (int k_ = 0; k_ < kTraceMarks; ++k_) if (k_ == (int)(i)) tm_[k_] = now_; \
  } while (0)
#define PER_FLUSH()                                                                            \
  do {                                                                                         \
    if (threadIdx.x == 0 && blockIdx.y == 0 && blockIdx.x < kTraceBlocks) {                    \
      _Pragma("unroll") for (int k_ = 0; k_ < kTraceMarks; ++k_)                               \
        g_trace[blockIdx.x * kTraceMarks + k_] = tm_[k_];                                      \
    }                                                                                          \
  } while (0)
extern "C" int per_trace_read(unsigned long long* host, int clear) {
  if (hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), sizeof(g_trace)) != hipSuccess) return -1;
  if (clear) {
    static unsigned long long zeros[kTraceBlocks * kTraceMarks];
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_trace), zeros, sizeof(zeros)) != hipSuccess) return -1;
  }
  return kTraceBlocks * kTraceMarks;
}
#else
#define PER_TRACE_DECL do { } while (0)
#define PER_MARK(i) do { } while (0)
#define PER_MARK_HWID(i) do { } while (0)
#define PER_MARK_DYN(i) do { } while (0)
#define PER_FLUSH() do { } while (0)
#endif

// ---------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------
template <int LOGK>
struct Fan {
  static constexpr int K = 1 << LOGK;
  static constexpr int LPS = K >= 4 ? K / 4 : 1;          // lanes per child group
  static constexpr int LOGLPS = LOGK >= 2 ? LOGK - 2 : 0;
};

// Workgroup barrier for phases that hand data over through LDS only.  Unlike __syncthreads() it does
// not wait for this wave's outstanding global stores (which nothing in the workgroup reads back).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ bool valid_priority(float v) {
  return v >= 0.0f && v <= 3.402823466e38f;   // finite and >= 0 (false for NaN); -0.0f passes
}

__device__ __forceinline__ uint32_t shr64(uint32_t x, uint32_t sh) { return (uint32_t)((uint64_t)x >> sh); }

// Sum of the K children starting at grp; q = lane position inside the LPS-lane group.
// Every lane of the group returns the same value.
template <int LOGK>
__device__ __forceinline__ float group_sum(const float* grp, unsigned q) {
  if constexpr (LOGK == 1) {
    const float2 c = *reinterpret_cast<const float2*>(grp);
    return c.x + c.y;
  } else {
    const float4 c = *reinterpret_cast<const float4*>(grp + 4 * q);
    float s = (c.x + c.y) + (c.z + c.w);
#pragma unroll
    for (int k = 0; k < Fan<LOGK>::LOGLPS; ++k) s = s + __shfl_xor(s, 1 << k);
    return s;
  }
}

// Per-height facts of one tree, kept in LDS by kernels that loop over heights: indexing the
// kernel arguments by a run-time height costs a dependent scalar load from memory per use.  The
// kernel-argument segment is ordinary read-only memory, so lane h fetches the entries of height h
// from it with a vector load and all heights arrive in one trip.  Only for kernels whose FIRST
// argument is the Geom (it then sits at offset 0 of the segment).
struct LevelTable {
  float* lvl[kMaxHeight + 1];   // level h of this tree
  uint32_t n[kMaxHeight + 1];   // its real nodes
};
template <typename T>
__device__ __forceinline__ const T* kernarg_at(size_t offset) {
  return (const T*)((const char*)__builtin_amdgcn_kernarg_segment_ptr() + offset);
}
__device__ __forceinline__ void fill_level_table(uint32_t H, uint32_t t, LevelTable* tab) {
  const Geom* gk = kernarg_at<Geom>(0);
  const uint32_t h = threadIdx.x;
  if (h <= H) {
    tab->lvl[h] = gk->level[h] + (size_t)t * gk->stride[h];
    tab->n[h] = gk->n[h];
  }
}

// One K-ary level of the prefix-sum traversal (Section V-A "traversing the tree
// performing prefix sum from root to leaf"), done by a single lane as log2(K) binary steps:
//   go right iff the right block is non-zero and not (r < left block); then r -= left.
//
// walk_chunks: s[] holds the 2^M chunk sums of the group (a chunk = 4 adjacent children,
// summed (c0+c1)+(c2+c3)).  The recursion first builds the pairwise sums above the chunks,
// walks those levels from the top, and then decides between the two chunks below the node
// it arrived at.  The pair is picked with a select chain, so everything stays in registers.
template <int M>
__device__ __forceinline__ unsigned walk_chunks(const float (&s)[1 << M], float& r) {
  if constexpr (M == 0) {
    return 0u;
  } else {
    constexpr int HALF = 1 << (M - 1);
    float up[HALF];
#pragma unroll
    for (int i = 0; i < HALF; ++i) up[i] = s[2 * i] + s[2 * i + 1];
    const unsigned pos = walk_chunks<M - 1>(up, r);
    float L = s[0], R = s[1];
#pragma unroll
    for (int i = 1; i < HALF; ++i) {
      const bool here = pos == (unsigned)i;
      L = here ? s[2 * i] : L;
      R = here ? s[2 * i + 1] : R;
    }
    const bool right = (R != 0.0f) && !(r < L);
    r = right ? r - L : r;
    return 2u * pos + (right ? 1u : 0u);
  }
}

// grp points at the K children (LDS or global).  Returns the chosen child, its value and the
// residual.  The chosen chunk is read a second time instead of keeping all K children live.
template <int LOGK>
__device__ __forceinline__ void descend_lane(const float* grp, float& r, unsigned& child, float& val) {
  if constexpr (LOGK == 1) {
    const float2 c = *reinterpret_cast<const float2*>(grp);
    const bool right = (c.y != 0.0f) && !(r < c.x);
    r = right ? r - c.x : r;
    child = right ? 1u : 0u;
    val = right ? c.y : c.x;
  } else {
    constexpr int C = (1 << LOGK) / 4;
    const float4* g4 = reinterpret_cast<const float4*>(grp);
    float s[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const float4 x = g4[c];
      s[c] = (x.x + x.y) + (x.z + x.w);
    }
    const unsigned pos = walk_chunks<LOGK - 2>(s, r);
    const float4 x = g4[pos];
    const float p0 = x.x + x.y, p1 = x.z + x.w;
    const bool r1 = (p1 != 0.0f) && !(r < p0);
    r = r1 ? r - p0 : r;
    const float a = r1 ? x.z : x.x, b = r1 ? x.w : x.y;
    const bool r0 = (b != 0.0f) && !(r < a);
    r = r0 ? r - a : r;
    val = r0 ? b : a;
    child = 4u * pos + (r1 ? 2u : 0u) + (r0 ? 1u : 0u);
  }
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const uint32_t y = (uint32_t)__shfl_xor((int)x, m);
    x = y < x ? y : x;
  }
  return x;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const uint32_t y = (uint32_t)__shfl_xor((int)x, m);
    x = y > x ? y : x;
  }
  return x;
}

// Running maximum priority: mx = fp32 bits of this lane's valid positive value (0: none).  One
// atomic per wave, and only when the wave would actually raise the maximum; the plain read may
// be stale, which can only cause a redundant atomic, never a missed one (the value only grows).
// `seen` is the value read when the kernel started (so the read overlaps the other loads).
__device__ __forceinline__ uint32_t read_max_bits(const Geom& g, uint32_t t) {
  return *reinterpret_cast<volatile uint32_t*>(&g.max_v[t]);
}
__device__ __forceinline__ void raise_max(const Geom& g, uint32_t t, uint32_t mx, uint32_t seen) {
  mx = wave_max_u32(mx);
  if ((threadIdx.x & 63u) == 0 && mx > seen) atomicMax(reinterpret_cast<uint32_t*>(&g.max_v[t]), mx);
}

// Importance weight (prioritized experience replay, cited in Section II-A):
// w = (size * v / total)^-beta / max over the batch, the maximum being reached at the batch
// minimum of v.  fp64, so that the result stays within 1e-6 of an fp64 reference.
__device__ __forceinline__ float importance_weight(float v, float vmin, float total, uint32_t size, float beta) {
  const double nb = -(double)beta;
  const double scale = (double)size / (double)total;
  return (float)(pow(scale * (double)v, nb) / pow(scale * (double)vmin, nb));
}

// ---------------------------------------------------------------------------------
// fills and scalars
// ---------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, uint64_t count, uint32_t value) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  const uint64_t i0 = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t n4 = count / 4;
  uint4* p4 = reinterpret_cast<uint4*>(p);
  const uint4 v4 = make_uint4(value, value, value, value);
  for (uint64_t i = i0; i < n4; i += stride) p4[i] = v4;
  for (uint64_t i = n4 * 4 + i0; i < count; i += stride) p[i] = value;
}

hipError_t launch_fill_u32(const Tuning& tn, uint32_t* p, uint64_t count, uint32_t value, hipStream_t s) {
  if (count == 0) return hipSuccess;
  uint64_t blocks = (count / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 16384) blocks = 16384;
  PER_LAUNCH(KID_FILL, k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, count, value);
  return hipGetLastError();
}

__global__ void k_init_scalars(Geom g, float init_max) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= g.T) return;
  g.max_v[t] = init_max;
  g.status[t] = 0;
  for (uint32_t k = 0; k < 2 * kVminSlots; ++k) g.vmin[(size_t)k * g.T + t] = 0x7F800000u;
}

hipError_t launch_init_scalars(const Geom& g, float init_max, hipStream_t s) {
  k_init_scalars<<<dim3((g.T + 63) / 64), dim3(64), 0, s>>>(g, init_max);
  return hipGetLastError();
}

// which: 0 = root of every tree, 1 = running max priority
__global__ void k_read_scalars(Geom g, int which, float* out) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= g.T) return;
  out[t] = which == 0 ? g.root[(size_t)t * g.root_stride] : g.max_v[t];
}

hipError_t launch_read_scalars(const Geom& g, int which, float* out, hipStream_t s) {
  k_read_scalars<<<dim3((g.T + 63) / 64), dim3(64), 0, s>>>(g, which, out);
  return hipGetLastError();
}

__global__ void k_clear_status(Geom g) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < g.T) g.status[t] = 0;
}

hipError_t launch_clear_status(const Geom& g, hipStream_t s) {
  k_clear_status<<<dim3((g.T + 63) / 64), dim3(64), 0, s>>>(g);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// priority update, first half: claim
// ---------------------------------------------------------------------------------
// Element j raises the 64-bit stamp of its leaf to (stamp_base + j) << 32 | value bits by
// atomic max, and sets the leaf's bit in the dirty mask (one bit per leaf).  The largest j wins
// and carries its value with it.  Stamps grow from call to call, so stale stamps never win
// and the stamp array needs no clearing between calls.
__device__ __forceinline__ void claim_element(const Geom& g, uint32_t t, uint32_t size, uint32_t stamp_base, uint32_t j,
                                              uint32_t i, float v, uint32_t& mx, uint32_t& flags) {
  if (!(i < size)) flags |= 1u;
  else if (!valid_priority(v)) flags |= 2u;
  else {
    const unsigned long long stamp = ((unsigned long long)(stamp_base + j) << 32) | __float_as_uint(v);
    atomicMax(reinterpret_cast<unsigned long long*>(g.owner) + (size_t)t * g.owner_stride + i, stamp);
    atomicOr(&g.dirty[(size_t)t * g.dirty_stride + (i >> 5)], 1u << (i & 31u));
    const uint32_t vb = v > 0.0f ? __float_as_uint(v) : 0u;
    mx = vb > mx ? vb : mx;
  }
}

// Claims elements of the batch, strided over the job's workgroups.  Called by whole workgroups.
// TD: the batch may hold temporal-difference errors to be turned into priorities first (only the
// stand-alone claim kernel carries that code).
template <bool TD = false>
__device__ __forceinline__ void claim_job(const Geom& g, uint32_t t, const ClaimArgs& c, uint32_t job_block,
                                          uint32_t job_blocks) {
  if (job_block * blockDim.x >= c.B) return;   // nothing to do for this workgroup
  const uint32_t max_seen = read_max_bits(g, t);
  uint32_t mx = 0;
  uint32_t flags = 0;
  for (uint32_t base = job_block * blockDim.x; base < c.B; base += job_blocks * blockDim.x) {
    const uint32_t j = base + threadIdx.x;
    if (j < c.B) {
      float v = c.prio[(size_t)t * c.B + j];
      if constexpr (TD) {
        if (c.from_td)   // priority of a temporal-difference error; a non-finite error stays non-finite and is rejected
          v = (float)pow(fabs((double)v) + c.td_eps, c.td_alpha);
      }
      claim_element(g, t, c.size, c.stamp_base, j, c.idx[(size_t)t * c.B + j], v, mx, flags);
    }
  }
  raise_max(g, t, mx, max_seen);
  if (flags) atomicOr(&g.status[t], flags);
}

__global__ void k_update_claim(Geom g, ClaimArgs c) { claim_job<true>(g, blockIdx.y, c, blockIdx.x, gridDim.x); }

// ---------------------------------------------------------------------------------
// priority sampling
// ---------------------------------------------------------------------------------
// The topmost heights below the root are copied to LDS (at most kTopSlots of them, highest
// first).  Their descriptors sit at fixed kernel-argument offsets, so the kernel fetches all of
// them with one batch of scalar loads instead of a chain of dependent ones.
constexpr int kTopSlots = 4;
struct TopCopy {
  const float* ptr[kTopSlots];     // that height of tree 0
  uint32_t stride[kTopSlots];      // floats between trees
  uint32_t cnt[kTopSlots];         // floats copied: whole child groups, n[l+1] * K
  uint32_t nreal[kTopSlots];       // real nodes n[l]
  uint32_t nslots;
  const float* root;               // root of tree 0
  uint32_t root_stride;
};

// One lane per sample; grid (ceil(B / block), T).  Dynamic LDS holds the top copy followed by
// one staging area per wave.  Below the copy each level costs one trip to memory: the wave
// fetches its 64 child groups with fully coalesced 16-byte loads (K/4 adjacent lanes per
// group), parks them in LDS rows of K+4 floats (the pad keeps 16-byte row reads conflict-free),
// and every lane then walks its own row.
//
// Uniform of sample i of tree t when the caller supplies none ("uniformly generated random",
// Section II-A): Philox4x32-10 (Salmon et al., SC 2011), ten rounds of two 32x32->64
// multiplications on the counter (i, call low, call high, t) with the key (seed low, seed high)
// bumped by Weyl constants between rounds; first output word, top 24 bits, scaled by 2^-24.
__device__ __forceinline__ float counter_uniform(const RngArgs& rng, uint32_t i, uint32_t t) {
  uint32_t c0 = i, c1 = rng.call_lo, c2 = rng.call_hi, c3 = t;
  uint32_t k0 = rng.seed_lo, k1 = rng.seed_hi;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  return (float)(c0 >> 8) * (1.0f / 16777216.0f);
}

// Chunk (IT*64 + lane) of the wave's 64*C 16-byte chunks, for IT = 0 .. C-1: fetched from the
// group of the lane that owns it and parked in that lane's staging row.  Written as a recursion over
// IT (not a loop over an array of registers) so that every fetch is issued before the first LDS store
// without the compiler having to promote an array.
template <int LOGK, int IT>
__device__ __forceinline__ void stage_groups(const float* __restrict__ lvl, uint32_t node, unsigned lane, float* stage) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int C = K / 4;
  constexpr int ROW = K + 4;
  if constexpr (IT < C) {
    const unsigned gch = (unsigned)IT * 64u + lane;
    const uint32_t nd = (uint32_t)__shfl((int)node, (int)(gch / C));
    const float4 x = *reinterpret_cast<const float4*>(lvl + (size_t)nd * K + (gch % C) * 4u);
    stage_groups<LOGK, IT + 1>(lvl, node, lane, stage);
    *reinterpret_cast<float4*>(stage + (gch / C) * ROW + (gch % C) * 4u) = x;
  }
}

// stale < 0: the tree in memory is whole.  stale >= 0: the last update left the root and the
// `stale` topmost copied heights to this kernel; they are rebuilt here from the highest fresh
// height (which is in the copy), and the first workgroup of each tree stores them back.
//
// The claim phase of a priority update fused into the call can ride along (it touches stamps, dirty
// bits and the running maximum only, none of which sampling reads).  claim_mode 1: the update targets
// exactly the indices sampled here, element by element, so every lane claims its own sample when it has
// it.  claim_mode 2: the update batch lies in other memory; the first claim_blocks workgroups of the
// grid are claim workgroups.  claim_mode 0: no claim here.
template <int LOGK>
__global__ void __launch_bounds__(1024)
k_sample(Geom g, TopCopy tc, uint32_t B, uint32_t size, float beta, const float* __restrict__ u,
         uint32_t* __restrict__ out_idx, float* __restrict__ out_prio, float* __restrict__ out_w,
         uint32_t parity, int stale, uint32_t claim_blocks, ClaimArgs c, int claim_mode, RngArgs rng) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  constexpr int ROW = K + 4;                  // staging row, floats
  using Vec = typename std::conditional<LOGK == 1, float2, float4>::type;
  constexpr int VF = sizeof(Vec) / 4;
  extern __shared__ __attribute__((aligned(16))) float lds[];   // 16-byte LDS accesses need the alignment
  __shared__ uint32_t s_min[16];
  __shared__ float s_total;
  const uint32_t t = blockIdx.y;
  const uint32_t H = g.H;
  const unsigned lane = threadIdx.x & 63u;
  const unsigned wave = threadIdx.x >> 6;
  const int nslots = (int)tc.nslots;
  if (blockIdx.x < claim_blocks) {   // claim workgroups come first: their atomics are under way before the descent loads start
    claim_job(g, t, c, blockIdx.x, claim_blocks);
    return;
  }
  const uint32_t bx = blockIdx.x - claim_blocks;            // sampling workgroup number
  const uint32_t sample_blocks = gridDim.x - claim_blocks;

  PER_TRACE_DECL;
  PER_MARK(0);
  const uint32_t s_raw = bx * blockDim.x + threadIdx.x;
  const bool active = s_raw < B;
  const uint32_t s = active ? s_raw : B - 1;
  const size_t o = (size_t)t * B + s;
  // the root, this lane's uniform and the top copy are all fetched in the same trip
  float total = tc.root[(size_t)t * tc.root_stride];
  const float u_s = rng.on ? counter_uniform(rng, s, t) : u[o];
  // the new priority of this lane's sample and the running maximum, fetched in that same trip
  float upd_v = 0.0f;
  uint32_t max_seen = 0;
  if (claim_mode == 1) {
    upd_v = c.prio[o];
    max_seen = read_max_bits(g, t);
  }

  uint32_t off[kTopSlots + 1];
  off[0] = 0;
#pragma unroll
  for (int i = 0; i < kTopSlots; ++i) off[i + 1] = off[i] + (i < nslots ? tc.cnt[i] : 0u);
  const uint32_t top_floats = off[kTopSlots];

  if (nslots > 0) {
    // one flat loop over the vectors of all copied heights (stale ones are skipped)
    uint32_t v_lo = 0;   // off[min(stale, kTopSlots)] / VF, without indexing the array by a run-time value
#pragma unroll
    for (int i = 1; i <= kTopSlots; ++i)
      if (stale >= i) v_lo = off[i] / VF;
    for (uint32_t e = v_lo + threadIdx.x; e < top_floats / VF; e += blockDim.x) {
      const uint32_t f = e * VF;
      const float* src = tc.ptr[0] + (size_t)t * tc.stride[0];
      uint32_t base = 0;
#pragma unroll
      for (int i = 1; i < kTopSlots; ++i) {
        const bool here = i < nslots && f >= off[i];
        src = here ? tc.ptr[i] + (size_t)t * tc.stride[i] : src;
        base = here ? off[i] : base;
      }
      *reinterpret_cast<Vec*>(lds + f) = *reinterpret_cast<const Vec*>(src + (f - base));
    }
    __syncthreads();
    PER_MARK(1);
    if (stale >= 0) {   // rebuild slots stale-1 .. 0 and the root, bottom-up
      const unsigned q = threadIdx.x % LPS;
      const uint32_t grp = threadIdx.x / LPS, ngrp = blockDim.x / LPS;
#pragma unroll
      for (int i = kTopSlots - 1; i >= -1; --i) {
        if (i < stale && i + 1 < nslots) {
          const uint32_t nl = i >= 0 ? tc.nreal[i] : 1u;
          const uint32_t cnt = i >= 0 ? tc.cnt[i] : 0u;
          const uint32_t off_l = i >= 0 ? off[i] : 0u;
          for (uint32_t base = 0; base < nl; base += ngrp) {
            const uint32_t j = base + grp;
            const bool real = j < nl;
            const float sum = group_sum<LOGK>(lds + off[i + 1] + (size_t)(real ? j : 0u) * K, q);
            if (q == 0 && real) {
              if (i >= 0) lds[off_l + j] = sum; else s_total = sum;
            }
          }
          for (uint32_t j = nl + threadIdx.x; j < cnt; j += blockDim.x) lds[off_l + j] = 0.0f;   // group padding
          __syncthreads();
        }
      }
      total = s_total;
    }
  }

  if (!(total > 0.0f)) {   // nothing can be sampled from this tree (uniform over the block)
    if (active) {
      out_idx[o] = 0xFFFFFFFFu;
      if (out_prio) out_prio[o] = 0.0f;
      if (out_w) out_w[o] = 0.0f;
    }
    // (a fused update of these samples finds no valid index: every element is out of range)
    if (bx == 0 && threadIdx.x == 0) atomicOr(&g.status[t], claim_mode == 1 ? 5u : 4u);
    return;
  }

  PER_MARK(2);
  const float seg = total / (float)B;
  const float pos = (float)s + u_s;
  float r = pos * seg;

  uint32_t node = 0;
  float val = total;
#pragma unroll
  for (int i = 0; i < kTopSlots; ++i) {
    if (i < nslots) {
      unsigned child;
      descend_lane<LOGK>(lds + off[i] + (size_t)node * K, r, child, val);
      node = node * K + child;
    }
  }

  PER_MARK(3);
  float* stage = lds + top_floats + (size_t)wave * 64 * ROW;
  const int l0 = (int)H - 1 - nslots;     // highest height read from memory
  // the pointer of the next level is fetched while the current one is processed
  const float* lvl_next = l0 >= 0 ? g.level[l0] + (size_t)t * g.stride[l0] : nullptr;
  for (int l = l0; l >= 0; --l) {
    const float* lvl = lvl_next;
    if (l > 0) lvl_next = g.level[l - 1] + (size_t)t * g.stride[l - 1];
    unsigned child;
    if constexpr (LOGK <= 2) {
      descend_lane<LOGK>(lvl + (size_t)node * K, r, child, val);
    } else {
      stage_groups<LOGK, 0>(lvl, node, lane, stage);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      descend_lane<LOGK>(stage + lane * ROW, r, child, val);
      __builtin_amdgcn_wave_barrier();
    }
    node = node * K + child;
    PER_MARK_DYN(4 + (l0 - l));
  }

  if (active) {
    out_idx[o] = node;
    if (out_prio) out_prio[o] = val;
  }
  // Stores come last on purpose: on this hardware a wait for loaded data also waits for every
  // earlier store of the wave.  The first workgroup of each tree puts the rebuilt heights back.
  if (stale >= 0 && bx == 0) {
#pragma unroll
    for (int i = 0; i < kTopSlots; ++i)
      if (i < stale) {
        float* dst = g.level[H - 1 - (uint32_t)i] + (size_t)t * g.stride[H - 1 - (uint32_t)i];
        for (uint32_t j = threadIdx.x; j < tc.nreal[i]; j += blockDim.x) dst[j] = lds[off[i] + j];
      }
    if (threadIdx.x == 0) g.root[(size_t)t * g.root_stride] = total;
  }
  PER_MARK(12);
  PER_FLUSH();
  if (out_w) {
    // Importance weights need the batch minimum of the sampled values.
    const uint32_t m = wave_min_u32(active ? __float_as_uint(val) : 0x7F800000u);
    if (sample_blocks == 1) {   // the whole batch of this tree is in this block: finish here
      if (lane == 0) s_min[wave] = m;
      __syncthreads();
      uint32_t mm = 0x7F800000u;
      for (uint32_t wv = 0; wv < (blockDim.x >> 6); ++wv) mm = s_min[wv] < mm ? s_min[wv] : mm;
      if (active) out_w[o] = importance_weight(val, __uint_as_float(mm), total, size, beta);
    } else {                // partial minima, spread over kVminSlots addresses; the weights job finishes
      if (active) out_w[o] = val;
      if (lane == 0)
        atomicMin(&g.vmin[((size_t)parity * g.T + t) * kVminSlots + ((bx * (blockDim.x >> 6) + wave) % kVminSlots)], m);
    }
  }
  if (claim_mode == 1) {   // element s of the update batch is this lane's own sample
    uint32_t mx = 0, flags = 0;
    if (active) claim_element(g, t, size, c.stamp_base, s, node, upd_v, mx, flags);
    raise_max(g, t, mx, max_seen);
    if (flags) atomicOr(&g.status[t], flags);
  }
}

// Finishes the importance weights of tree t: folds the partial minima of this call, re-arms
// the other buffer for the next call, and turns the sampled values left in w into weights.
// Called by whole workgroups of any size; `first` marks the one that re-arms.
__device__ __forceinline__ void weights_job(const Geom& g, uint32_t t, uint32_t B, uint32_t size, float beta,
                                            float* __restrict__ w, uint32_t parity, uint32_t job_block,
                                            uint32_t job_blocks) {
  __shared__ uint32_t s_wmin[16];
  if (job_block != 0 && job_block * blockDim.x >= B) return;   // nothing to do for this workgroup
  const uint32_t* part = g.vmin + ((size_t)parity * g.T + t) * kVminSlots;
  uint32_t m = 0x7F800000u;
  for (uint32_t j = threadIdx.x; j < kVminSlots; j += blockDim.x) m = part[j] < m ? part[j] : m;
  m = wave_min_u32(m);
  if ((threadIdx.x & 63u) == 0) s_wmin[threadIdx.x >> 6] = m;
  if (job_block == 0)
    for (uint32_t j = threadIdx.x; j < kVminSlots; j += blockDim.x)
      g.vmin[((size_t)(parity ^ 1u) * g.T + t) * kVminSlots + j] = 0x7F800000u;
  __syncthreads();
  uint32_t mm = 0x7F800000u;
  for (uint32_t wv = 0; wv < (blockDim.x >> 6); ++wv) mm = s_wmin[wv] < mm ? s_wmin[wv] : mm;
  const float total = g.root[(size_t)t * g.root_stride];
  for (uint32_t i = job_block * blockDim.x + threadIdx.x; i < B; i += job_blocks * blockDim.x) {
    const size_t o = (size_t)t * B + i;
    w[o] = total > 0.0f ? importance_weight(w[o], __uint_as_float(mm), total, size, beta) : 0.0f;
  }
}

__global__ void k_weights(Geom g, uint32_t B, uint32_t size, float beta, float* __restrict__ w, uint32_t parity) {
  weights_job(g, blockIdx.y, B, size, beta, w, parity, blockIdx.x, gridDim.x);
}

template <int LOGK>
static hipError_t launch_resum_top_k(const Geom& g, const Tuning& tn, uint32_t hb, hipStream_t s);
static hipError_t launch_finish(const Geom& g, const Tuning& tn, const FieldTable* rows, const FinishArgs& a,
                                hipStream_t s);
template <int LOGK>
static hipError_t launch_tree_k(const Geom& g, const Tuning& tn, uint32_t B, hipStream_t s);
template <int LOGK>
static hipError_t launch_tree_finish_k(const Geom& g, const Tuning& tn, uint32_t B, const FieldTable* rows,
                                       const FinishArgs& a, hipStream_t s);

// Sampling call with whatever is fused into it.  rows: gather of the sampled rows.  claim: a priority
// update whose claim phase runs where claim_mode says (CLAIM_INLINE / CLAIM_BLOCKS: in the sampling
// kernel, the tree pass then shares the second kernel with the weights and row jobs; CLAIM_FINISH: in
// the second kernel, the tree pass is a third).
template <int LOGK>
static hipError_t launch_sample_k(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, float beta,
                                  const float* u, const RngArgs& rng, uint32_t* out_idx, float* out_w,
                                  float* out_prio, uint32_t* weight_calls, uint32_t stale_hb, const FieldTable* rows,
                                  const ClaimArgs* claim, int claim_mode, hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  constexpr uint32_t kLdsCap = 128 * 1024;
  const uint32_t wave_bytes = LOGK >= 3 ? 64u * (K + 4) * 4u : 0u;   // staging per wave
  // workgroup size: the whole batch in one workgroup when it is small (the weights are then finished
  // in-kernel), else the configured size; bounded by the LDS the staging rows need
  uint32_t max_waves = wave_bytes ? (uint32_t)(kLdsCap / 2 / wave_bytes) : 16u;
  if (max_waves > 16) max_waves = 16;
  if (max_waves < 1) max_waves = 1;
  uint32_t waves = tn.sample_block / 64;
  const uint32_t need = (B + 63) / 64;
  if (need <= max_waves) waves = need;
  if (waves > max_waves) waves = max_waves;
  const uint32_t block = waves * 64;
  const uint32_t gx = (B + block - 1) / block;
  // topmost heights (below the root) copied to LDS: at most kTopSlots, within the LDS budget, and only
  // while a height is small next to what the workgroup's samples would fetch from it one by one
  TopCopy tc{};
  uint64_t top = 0;
  for (int l = (int)g.H - 1; l >= 0 && tc.nslots < (uint32_t)kTopSlots; --l) {
    const uint64_t cnt = (uint64_t)g.n[l + 1] * K;
    const uint64_t add = cnt * 4;
    if (top + add > tn.lds_budget_bytes || top + add + (uint64_t)waves * wave_bytes > kLdsCap) break;
    const bool needed_for_rebuild = stale_hb && (uint32_t)l >= stale_hb;   // the rebuild of stale heights reads it
    if (cnt > 8ull * block && tn.lds_budget_bytes <= 64 * 1024 && !needed_for_rebuild) break;
    top += add;
    const uint32_t i = tc.nslots++;
    tc.ptr[i] = g.level[l];
    tc.stride[i] = g.stride[l];
    tc.cnt[i] = g.n[l + 1] * K;
    tc.nreal[i] = g.n[l];
  }
  tc.root = g.root;
  tc.root_stride = g.root_stride;
  size_t bytes = (size_t)top + (size_t)waves * wave_bytes;
  if (bytes < tn.sample_min_lds) bytes = tn.sample_min_lds;   // asking for more LDS than needed spreads workgroups over more CUs
  // The two buffers of partial minima alternate between the calls that use them (k_weights of
  // one call re-arms the buffer of the next).
  const uint32_t parity = *weight_calls & 1u;
  if (out_w && gx > 1) ++*weight_calls;
  hipError_t e;
  int stale = -1;
  if (stale_hb) {
    // copied heights above stale_hb are rebuilt in LDS; the copy must reach down to stale_hb
    const int lowest_copied = (int)g.H - (int)tc.nslots;
    if (tc.nslots > 0 && lowest_copied <= (int)stale_hb) {
      stale = (int)g.H - 1 - (int)stale_hb;
    } else {
      e = launch_resum_top_k<LOGK>(g, tn, stale_hb, s);
      if (e != hipSuccess) return e;
    }
  }
  if (bytes > 64 * 1024) {   // more than the default dynamic LDS limit has to be requested per kernel
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_sample<LOGK>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
  }
  if (!claim) claim_mode = CLAIM_NONE;
  const bool claim_here = claim_mode == CLAIM_INLINE || claim_mode == CLAIM_BLOCKS;
  uint32_t claim_blocks = 0;
  if (claim_mode == CLAIM_BLOCKS) {
    claim_blocks = (claim->B + block - 1) / block;
    if (claim_blocks > 4096) claim_blocks = 4096;   // the claim job strides
  }
  PER_LAUNCH(KID_SAMPLE, k_sample<LOGK>, dim3(gx + claim_blocks, g.T), dim3(block), bytes, s, g, tc, B, size, beta, u,
             out_idx, out_prio, out_w, parity, stale, claim_blocks, claim_here ? *claim : ClaimArgs{},
             claim_here ? claim_mode : (int)CLAIM_NONE, rng);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const bool finish_weights = out_w && gx > 1;
  if (rows || claim) {   // fused call
    FinishArgs a{};
    a.B = B;
    a.idx = out_idx;
    a.w = finish_weights ? out_w : nullptr;
    a.size = size;
    a.beta = beta;
    a.parity = parity;
    if (claim_here) {   // second kernel: tree pass beside the weights and the rows
      if (rows || finish_weights) return launch_tree_finish_k<LOGK>(g, tn, claim->B, rows, a, s);
      return launch_tree_k<LOGK>(g, tn, claim->B, s);
    }
    // second kernel: rows, weights and the claim phase; the tree pass follows
    a.has_claim = claim ? 1u : 0u;
    if (claim) a.claim = *claim;
    e = launch_finish(g, tn, rows, a, s);
    if (e != hipSuccess || !claim) return e;
    return launch_tree_k<LOGK>(g, tn, claim->B, s);
  }
  if (!finish_weights) return e;
  PER_LAUNCH(KID_WEIGHTS, k_weights, dim3((B + 255) / 256, g.T), dim3(256), 0, s, g, B, size, beta, out_w, parity);
  return hipGetLastError();
}

#define PER_DISPATCH_LOGK(logK, CALL)            \
  switch (logK) {                                \
    case 1: return CALL(1);                      \
    case 2: return CALL(2);                      \
    case 3: return CALL(3);                      \
    case 4: return CALL(4);                      \
    case 5: return CALL(5);                      \
    case 6: return CALL(6);                      \
    default: return hipErrorInvalidValue;        \
  }

hipError_t launch_sample(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, float beta, const float* u,
                         const RngArgs& rng, uint32_t* out_idx, float* out_w, float* out_prio, uint32_t* weight_calls, uint32_t stale_hb,
                         const FieldTable* rows, const ClaimArgs* claim, int claim_mode, hipStream_t s) {
#define CALL(L) launch_sample_k<L>(g, tn, B, size, beta, u, rng, out_idx, out_w, out_prio, weight_calls, stale_hb, rows, claim, claim_mode, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

// ---------------------------------------------------------------------------------
// Data Storage: row gather and row scatter
// ---------------------------------------------------------------------------------
// grid (x, n_fields, T).  A row of E bytes is moved by E/vec adjacent lanes, vec bytes each,
// so the dense side is fully coalesced and the storage side is coalesced within a row.
template <typename V, bool GATHER>
__device__ __forceinline__ void move_rows(const FieldTable& ft, uint32_t f, uint32_t t, uint32_t B,
                                          const uint32_t* __restrict__ idx, uint32_t cursor, uint32_t N,
                                          uint32_t* status, uint32_t job_block, uint32_t job_blocks) {
  const uint32_t E = ft.bytes[f];
  const uint32_t epr = E / (uint32_t)sizeof(V);
  const uint64_t total = (uint64_t)B * epr;
  uint8_t* col = ft.col[f] + (uint64_t)t * ft.col_stride[f];
  uint8_t* io = ft.io[f] + (uint64_t)t * B * E;
  bool bad = false;
  // Two elements per lane and sweep, both loads issued before the first store: a wait for loaded
  // data also waits for earlier stores, so load -> store -> load would cost two memory trips.
  const uint64_t stride = (uint64_t)job_blocks * blockDim.x;
  for (uint64_t e0 = (uint64_t)job_block * blockDim.x + threadIdx.x; e0 < total; e0 += 2 * stride) {
    const uint64_t e1 = e0 + stride;
    const bool live1 = e1 < total;
    const uint64_t e1c = live1 ? e1 : e0;
    const uint32_t row0 = (uint32_t)(e0 / epr), row1 = (uint32_t)(e1c / epr);
    const uint32_t k0 = (uint32_t)(e0 - (uint64_t)row0 * epr), k1 = (uint32_t)(e1c - (uint64_t)row1 * epr);
    V* dense0 = reinterpret_cast<V*>(io + (uint64_t)row0 * E) + k0;
    V* dense1 = reinterpret_cast<V*>(io + (uint64_t)row1 * E) + k1;
    if constexpr (GATHER) {
      const uint32_t i0 = idx[(size_t)t * B + row0];
      const uint32_t i1 = idx[(size_t)t * B + row1];
      const bool ok0 = i0 < N, ok1 = i1 < N;
      V v0 = *(reinterpret_cast<const V*>(col + (uint64_t)(ok0 ? i0 : 0u) * E) + k0);
      V v1 = *(reinterpret_cast<const V*>(col + (uint64_t)(ok1 ? i1 : 0u) * E) + k1);
      if (!ok0) __builtin_memset(&v0, 0, sizeof(V));
      if (!ok1) __builtin_memset(&v1, 0, sizeof(V));
      bad |= !ok0 || (live1 && !ok1);
      *dense0 = v0;
      if (live1) *dense1 = v1;
    } else {
      uint64_t slot0 = (uint64_t)cursor + row0, slot1 = (uint64_t)cursor + row1;
      if (slot0 >= N) slot0 -= N;
      if (slot1 >= N) slot1 -= N;
      const V v0 = *dense0;
      const V v1 = *dense1;
      *(reinterpret_cast<V*>(col + slot0 * E) + k0) = v0;
      if (live1) *(reinterpret_cast<V*>(col + slot1 * E) + k1) = v1;
    }
  }
  if (bad) atomicOr(&status[t], 1u);
}

// Moves the rows of one payload field; the workgroup is number job_block of job_blocks on that field.
template <bool GATHER>
__device__ __forceinline__ void rows_job(const FieldTable& ft, uint32_t f, uint32_t t, uint32_t B,
                                         const uint32_t* __restrict__ idx, uint32_t cursor, uint32_t N,
                                         uint32_t* status, uint32_t job_block, uint32_t job_blocks) {
  switch (ft.vec[f]) {
    case 16: move_rows<uint4, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks); break;
    case 8: move_rows<uint2, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks); break;
    case 4: move_rows<uint32_t, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks); break;
    case 2: move_rows<uint16_t, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks); break;
    default: move_rows<uint8_t, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks); break;
  }
}

// Rows moved by one workgroup (small inserts, and the workgroup-per-tree step kernel): the elements
// of all fields form one flat index space shared out over the lanes.  Addresses are worked out
// first (the part that differs by field), then every lane issues its one load and, after it, its
// one store: the lanes of a wave that serve different fields do not wait for each other's trips
// to memory.  The caller's dense rows start at row dense_row0 of each field's array.
// GATHER: row j comes from slot idx[j] (idx may live in LDS); slots >= N give zero bytes and the
// return value true.  Otherwise row j goes to ring slot cursor + j.
template <bool GATHER>
__device__ __forceinline__ bool move_rows_one_workgroup(const FieldTable& ft, uint32_t t, uint64_t dense_row0, uint32_t n,
                                                        uint32_t cursor, uint32_t N, const uint32_t* idx) {
  uint32_t first[kMaxFields + 1];
  first[0] = 0;
#pragma unroll
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f)
    first[f + 1] = first[f] + (f < ft.n_fields && ft.io[f] ? n * (ft.bytes[f] / ft.vec[f]) : 0u);
  bool bad = false;
  for (uint32_t e = threadIdx.x; e < first[kMaxFields]; e += blockDim.x) {
    // the field of this element, picked with selects; the divisions are done once, after the choice
    uint8_t* io = nullptr;
    uint8_t* col = nullptr;
    uint32_t E = 1, w = 1, base = 0;
#pragma unroll
    for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f) {
      const bool here = e >= first[f] && e < first[f + 1];
      io = here ? ft.io[f] : io;
      col = here ? ft.col[f] + (uint64_t)t * ft.col_stride[f] : col;
      E = here ? ft.bytes[f] : E;
      w = here ? ft.vec[f] : w;
      base = here ? first[f] : base;
    }
    const uint32_t epr = E / w;
    const uint32_t el = e - base;
    const uint32_t row = el / epr, k = el - row * epr;
    uint64_t slot;
    bool live = true;
    if constexpr (GATHER) {
      slot = idx[row];
      live = slot < N;
      bad = bad || !live;
      if (!live) slot = 0;
    } else {
      slot = (uint64_t)cursor + row;
      if (slot >= N) slot -= N;
    }
    uint8_t* dense = io + (dense_row0 + row) * E + (uint64_t)k * w;
    uint8_t* stored = col + slot * E + (uint64_t)k * w;
    const uint8_t* src = GATHER ? stored : dense;
    uint8_t* dst = GATHER ? dense : stored;
    uint4 v = make_uint4(0, 0, 0, 0);
    switch (w) {
      case 16: v = *reinterpret_cast<const uint4*>(src); break;
      case 8: { const uint2 x = *reinterpret_cast<const uint2*>(src); v.x = x.x; v.y = x.y; } break;
      case 4: v.x = *reinterpret_cast<const uint32_t*>(src); break;
      case 2: v.x = *reinterpret_cast<const uint16_t*>(src); break;
      default: v.x = *src; break;
    }
    if (!live) v = make_uint4(0, 0, 0, 0);
    switch (w) {
      case 16: *reinterpret_cast<uint4*>(dst) = v; break;
      case 8: *reinterpret_cast<uint2*>(dst) = make_uint2(v.x, v.y); break;
      case 4: *reinterpret_cast<uint32_t*>(dst) = v.x; break;
      case 2: *reinterpret_cast<uint16_t*>(dst) = (uint16_t)v.x; break;
      default: *dst = (uint8_t)v.x; break;
    }
  }
  return bad;
}

// Second kernel of the fused calls.  Its workgroups (blockIdx.x) split into jobs, each with as many
// workgroups as it needs (JobRanges): first the importance weights of the batch just sampled (if
// asked for), then the claim phase of a priority update (if one is fused in), then one job per
// payload field of the sampled rows.  The small jobs come first, so their latency hides behind the
// row traffic.
__global__ void k_finish(FieldTable ft, JobRanges jr, Geom g, FinishArgs a) {
  const uint32_t t = blockIdx.y;
  const uint32_t b = blockIdx.x;
  if (b < jr.first[1]) {
    weights_job(g, t, a.B, a.size, a.beta, a.w, a.parity, b, jr.first[1]);
    return;
  }
  if (b < jr.first[2]) {
    claim_job(g, t, a.claim, b - jr.first[1], jr.first[2] - jr.first[1]);
    return;
  }
#pragma unroll
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f)
    if (b >= jr.first[2 + f] && b < jr.first[3 + f]) {
      rows_job<true>(ft, f, t, a.B, a.idx, 0, g.N, g.status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
      return;
    }
}

// Stand-alone gather (GATHER) and insert scatter: one job per payload field.
template <bool GATHER>
__global__ void k_rows(FieldTable ft, JobRanges jr, uint32_t B, const uint32_t* __restrict__ idx, uint32_t cursor,
                       uint32_t N, uint32_t* status) {
  const uint32_t t = blockIdx.y;
  const uint32_t b = blockIdx.x;
#pragma unroll
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f)
    if (b >= jr.first[2 + f] && b < jr.first[3 + f]) {
      rows_job<GATHER>(ft, f, t, B, idx, cursor, N, status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
      return;
    }
}

// Workgroups per job: weights, claim, then each field with a destination (a field's count is what
// one pass over its elements needs, capped; the movers stride when capped).
static JobRanges job_ranges(const FieldTable* ft, uint32_t rows, uint32_t block, uint32_t weights_B, uint32_t claim_B) {
  JobRanges jr{};
  uint32_t at = 0;
  jr.first[0] = at;
  at += (weights_B + block - 1) / block;
  jr.first[1] = at;
  at += (claim_B + block - 1) / block;
  jr.first[2] = at;
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f) {
    if (ft && f < ft->n_fields && ft->io[f]) {
      // two elements per lane once a field is large enough to matter, so that the whole launch stays resident
      const uint64_t elems = (uint64_t)rows * (ft->bytes[f] / ft->vec[f]);
      uint64_t n = (elems + block - 1) / block;
      if (n > 512) n = (elems + 2 * block - 1) / (2 * block);
      if (n > (1u << 20)) n = 1u << 20;
      at += (uint32_t)n;
    }
    jr.first[3 + f] = at;
  }
  return jr;
}

hipError_t launch_gather(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t B, const uint32_t* idx,
                         hipStream_t s) {
  const uint32_t block = tn.gather_block;
  const JobRanges jr = job_ranges(&ft, B, block, 0, 0);
  const uint32_t gx = jr.first[2 + kMaxFields];
  if (gx == 0) return hipSuccess;
  PER_LAUNCH(KID_GATHER, k_rows<true>, dim3(gx, g.T), dim3(block), 0, s, ft, jr, B, idx, 0, g.N, g.status);
  return hipGetLastError();
}

static hipError_t launch_finish(const Geom& g, const Tuning& tn, const FieldTable* rows, const FinishArgs& a,
                                hipStream_t s) {
  FieldTable ft{};
  if (rows) ft = *rows;
  if (!a.w && !a.has_claim) return rows ? launch_gather(g, tn, ft, a.B, a.idx, s) : hipSuccess;
  const uint32_t block = tn.gather_block;
  const JobRanges jr = job_ranges(rows ? &ft : nullptr, a.B, block, a.w ? a.B : 0u, a.has_claim ? a.claim.B : 0u);
  PER_LAUNCH(KID_FINISH, k_finish, dim3(jr.first[2 + kMaxFields], g.T), dim3(block), 0, s, ft, jr, g, a);
  return hipGetLastError();
}

hipError_t launch_scatter(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t n, uint32_t cursor,
                          hipStream_t s) {
  const uint32_t block = tn.gather_block;
  const JobRanges jr = job_ranges(&ft, n, block, 0, 0);
  const uint32_t gx = jr.first[2 + kMaxFields];
  if (gx == 0) return hipSuccess;
  PER_LAUNCH(KID_SCATTER, k_rows<false>, dim3(gx, g.T), dim3(block), 0, s, ft, jr, n, nullptr, cursor, g.N, g.status);
  return hipGetLastError();
}

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

// ---------------------------------------------------------------------------------
// insertion: leaf writes (rows go through k_rows<false>)
// ---------------------------------------------------------------------------------
// Leaf of inserted row j (ring slot cursor + j): the given value, or the running maximum.
__device__ __forceinline__ void insert_leaf(const Geom& g, uint32_t t, uint32_t n, uint32_t cursor, uint32_t j,
                                            const float* __restrict__ prio, float max_on_entry,
                                            uint32_t* __restrict__ out_idx, uint32_t& mx, bool& bad) {
  uint64_t slot = (uint64_t)cursor + j;
  if (slot >= g.N) slot -= g.N;
  if (out_idx) out_idx[(size_t)t * n + j] = (uint32_t)slot;
  float* leaf = g.level[0] + (size_t)t * g.stride[0] + slot;
  if (prio) {
    const float v = prio[(size_t)t * n + j];
    if (valid_priority(v)) {
      *leaf = v;
      const uint32_t vb = v > 0.0f ? __float_as_uint(v) : 0u;
      mx = vb > mx ? vb : mx;
    } else {
      bad = true;
    }
  } else {
    *leaf = max_on_entry;   // running maximum as it was when the call started
  }
}

__global__ void k_insert_leaves(Geom g, uint32_t n, uint32_t cursor, const float* __restrict__ prio,
                                uint32_t* __restrict__ out_idx) {
  const uint32_t t = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t mx = 0;
  bool bad = false;
  if (j < n) insert_leaf(g, t, n, cursor, j, prio, prio ? 0.0f : g.max_v[t], out_idx, mx, bad);
  if (prio) {
    raise_max(g, t, mx, read_max_bits(g, t));
    if (bad) atomicOr(&g.status[t], 2u);
  }
}

// A small insert as one kernel, one workgroup per tree: the rows, the leaves, and every ancestor
// of the touched ring slots up to the root.  The touched nodes of a height form at most two
// contiguous ranges (narrowed by K per height), known before anything is read, so the child groups
// of all of them, at every height, are fetched into LDS in one trip; the new leaves and then each
// height's new sums are patched into the staged groups of the height above, and the heights are
// finished from LDS without going back to memory.
// stale_hb != 0: the last update left the heights above stale_hb to their next reader; they are
// then recomputed here in full instead of only over the touched ranges.
constexpr int kInsertHeights = 32;
struct InsertPlan {
  Range2 r[kInsertHeights];        // touched nodes of height h + 1
  uint32_t off[kInsertHeights];    // where their child groups start in LDS (floats)
};
struct InsertArgs {                // one kernel argument, so that both parts sit at known offsets of the segment
  Geom g;
  InsertPlan plan;
};

// position of node among the touched nodes of its height (the two ranges back to back)
__device__ __forceinline__ uint32_t plan_pos(const Range2& r, uint32_t node) {
  return node >= r.a0 && node < r.b0 ? node - r.a0 : (r.b0 - r.a0) + (node - r.a1);
}

template <int LOGK>
__global__ void __launch_bounds__(1024)
k_insert_small(InsertArgs a, FieldTable ft, uint32_t n, uint32_t cursor, const float* __restrict__ prio,
               uint32_t* __restrict__ out_idx) {
  const Geom& g = a.g;
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  extern __shared__ __attribute__((aligned(16))) float staged[];
  __shared__ LevelTable tab;
  __shared__ Range2 s_r[kInsertHeights];
  __shared__ uint32_t s_off[kInsertHeights];
  const uint32_t t = blockIdx.x;
  const uint32_t H = g.H;
  PER_TRACE_DECL;
  PER_MARK(0);
  fill_level_table(H, t, &tab);
  if (threadIdx.x >= 64 && threadIdx.x < 64 + H) {
    const InsertPlan* pk = kernarg_at<InsertPlan>(offsetof(InsertArgs, plan));
    s_r[threadIdx.x - 64] = pk->r[threadIdx.x - 64];
    s_off[threadIdx.x - 64] = pk->off[threadIdx.x - 64];
  }
  // the rows need none of the tables: their trip to memory overlaps the fetch of the tables
  (void)move_rows_one_workgroup<false>(ft, t, (uint64_t)t * n, n, cursor, g.N, nullptr);
  __syncthreads();
  PER_MARK(1);
  // ---- everything that is read: the child groups of all touched nodes, the running maximum
  for (uint32_t h = 1; h <= H; ++h) {
    const Range2 r = s_r[h - 1];
    const uint32_t c0 = r.b0 - r.a0, cnt = c0 + (r.b1 - r.a1);
    const float* child = tab.lvl[h - 1];
    for (uint32_t e = threadIdx.x; e < cnt * K; e += blockDim.x) {
      const uint32_t pos = e >> LOGK;
      const uint32_t node = pos < c0 ? r.a0 + pos : r.a1 + (pos - c0);
      staged[s_off[h - 1] + e] = child[(size_t)node * K + (e & (K - 1))];
    }
  }
  const float max_on_entry = prio ? 0.0f : g.max_v[t];
  uint32_t max_seen = 0;
  if (prio) max_seen = read_max_bits(g, t);
  __syncthreads();
  PER_MARK(2);
  // ---- leaves (stores only), the new ones also into their staged groups
  uint32_t mx = 0;
  bool bad = false;
  for (uint32_t j = threadIdx.x; j < n; j += blockDim.x) {
    uint64_t slot = (uint64_t)cursor + j;
    if (slot >= g.N) slot -= g.N;
    if (out_idx) out_idx[(size_t)t * n + j] = (uint32_t)slot;
    float v = max_on_entry;
    bool ok = true;
    if (prio) {
      v = prio[(size_t)t * n + j];
      ok = valid_priority(v);
      const uint32_t vb = ok && v > 0.0f ? __float_as_uint(v) : 0u;
      mx = vb > mx ? vb : mx;
      bad = bad || !ok;
    }
    if (ok) {
      tab.lvl[0][slot] = v;
      staged[s_off[0] + plan_pos(s_r[0], (uint32_t)(slot >> LOGK)) * K + ((uint32_t)slot & (K - 1))] = v;
    }
  }
  if (prio) {
    raise_max(g, t, mx, max_seen);
    if (bad) atomicOr(&g.status[t], 2u);
  }
  __syncthreads();
  PER_MARK(3);
  // ---- heights 1 .. H from the staged groups
  const unsigned q = threadIdx.x % LPS;
  const uint32_t grp = threadIdx.x / LPS, ngrp = blockDim.x / LPS;
  for (uint32_t h = 1; h <= H; ++h) {
    const Range2 r = s_r[h - 1];
    const uint32_t c0 = r.b0 - r.a0, cnt = c0 + (r.b1 - r.a1);
    float* par = tab.lvl[h];
    for (uint32_t base = 0; base < cnt; base += ngrp) {
      const uint32_t pos = base + grp;
      const bool ok = pos < cnt;
      const float sum = group_sum<LOGK>(staged + s_off[h - 1] + (size_t)(ok ? pos : 0u) * K, q);
      if (ok && q == 0) {
        const uint32_t node = pos < c0 ? r.a0 + pos : r.a1 + (pos - c0);
        par[node] = sum;
        if (h < H) staged[s_off[h] + plan_pos(s_r[h], node >> LOGK) * K + (node & (K - 1))] = sum;
      }
    }
    lds_barrier();   // the next height reads the staged groups only
  }
  PER_MARK(4);
  PER_FLUSH();
}

hipError_t launch_insert_leaves(const Geom& g, const Tuning& tn, uint32_t n, uint32_t cursor, const float* prio,
                                uint32_t* out_idx, hipStream_t s) {
  PER_LAUNCH(KID_INSERT_LEAVES, k_insert_leaves, dim3((n + 255) / 256, g.T), dim3(256), 0, s, g, n, cursor, prio,
             out_idx);
  return hipGetLastError();
}

// True when an insert of n rows is small enough for k_insert_small: few bytes to move and few
// nodes per height for one workgroup.
bool insert_fits_one_workgroup(const Geom& g, const FieldTable* ft, uint32_t n) {
  uint64_t bytes = 0;
  if (ft)
    for (uint32_t f = 0; f < ft->n_fields; ++f)
      if (ft->io[f]) bytes += (uint64_t)n * ft->bytes[f];
  return n <= 4096 && bytes <= 256 * 1024;
}

template <int LOGK>
static hipError_t launch_insert_small_k(const Geom& g, const Tuning& tn, const FieldTable* ft, uint32_t n,
                                        uint32_t cursor, const float* prio, uint32_t* out_idx, uint32_t stale_hb,
                                        hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  FieldTable f{};
  if (ft) f = *ft;
  InsertArgs a{};
  a.g = g;
  InsertPlan& plan = a.plan;
  const uint64_t end = (uint64_t)cursor + n;
  Range2 r;
  r.a0 = cursor;
  r.b0 = (uint32_t)(end < g.N ? end : g.N);
  r.a1 = 0;
  r.b1 = (uint32_t)(end > g.N ? end - g.N : 0);
  uint32_t floats = 0;
  for (uint32_t h = 1; h <= g.H; ++h) {
    if (r.b0 > r.a0) { r.a0 >>= LOGK; r.b0 = ((r.b0 - 1) >> LOGK) + 1; }
    if (r.b1 > r.a1) { r.a1 >>= LOGK; r.b1 = ((r.b1 - 1) >> LOGK) + 1; }
    if (r.b1 > r.a1 && r.a0 < r.b1) { r.a0 = 0; r.a1 = r.b1 = 0; }   // the two ranges met: one range
    if (stale_hb && h > stale_hb) r = Range2{0, g.n[h], 0, 0};
    plan.r[h - 1] = r;
    plan.off[h - 1] = floats;
    floats += ((r.b0 - r.a0) + (r.b1 - r.a1)) * K;
  }
  uint32_t block = (n * Fan<LOGK>::LPS + 63) / 64 * 64;
  if (block < 256) block = 256;
  if (block > 1024) block = 1024;
  PER_LAUNCH(KID_INSERT_SMALL, k_insert_small<LOGK>, dim3(g.T), dim3(block), (size_t)floats * 4, s, a, f, n, cursor, prio,
             out_idx);
  return hipGetLastError();
}

hipError_t launch_insert_small(const Geom& g, const Tuning& tn, const FieldTable* ft, uint32_t n, uint32_t cursor,
                               const float* prio, uint32_t* out_idx, uint32_t stale_hb, hipStream_t s) {
#define CALL(L) launch_insert_small_k<L>(g, tn, ft, n, cursor, prio, out_idx, stale_hb, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

// ---------------------------------------------------------------------------------
// priority update: claim (last writer), then one tree pass
// ---------------------------------------------------------------------------------
// Heights 1 .. hb of the tree pass at fixed kernel-argument offsets (slot j = height j + 1).
constexpr int kSubSlots = 13;
struct SubLevels {
  float* ptr[kSubSlots];          // that height of tree 0
  uint32_t stride[kSubSlots];     // floats between trees
  uint32_t n[kSubSlots];          // real nodes of that height
  uint32_t lds_off[kSubSlots];    // where the workgroup keeps its part of that height (floats)
  uint32_t lds_floats;            // total
  uint32_t hb;
};

// Tree pass.  Workgroup b of tree t owns the subtree under node b of height hb and keeps the
// subtree's nodes of heights 1 .. hb in LDS.
//  0. In one trip it fetches its height-1 nodes and the dirty bits of the leaves below them.
//  1. Each height-1 node with a dirty leaf is rebuilt by LPS lanes: they read its K leaves and,
//     for the dirty ones only, the stamp entry, whose lower word is the value of the batch
//     element that won that leaf; it replaces the leaf (and is stored); the K values are
//     summed pairwise.  The dirty bits are cleared at the end.
//  2. Heights 2 .. hb of the subtree are recomputed from LDS and stored.
//  3. Above hb every node counts the arrivals of its children's workgroups; the last one to
//     arrive recomputes it and carries on upwards, so the root is written by whichever
//     workgroup finishes last.  No workgroup ever waits for another.  When there are only a
//     few nodes at height hb this step is skipped (chain == 0): the agent-scope fences it
//     needs cost more than recomputing those heights in the next kernel that reads them.
constexpr uint32_t kDirtyListCap = 2048;
constexpr uint32_t kLazyTopNodes = 4096;

// The work of workgroup b of tree t (b = its subtree's root at height hb).
template <int LOGK>
__device__ __forceinline__ void tree_job(const Geom& g, const SubLevels& sl, uint32_t t, uint32_t b, uint32_t chain) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  extern __shared__ __attribute__((aligned(16))) float sub[];   // 16-byte LDS accesses need the alignment
  __shared__ uint32_t s_list[kDirtyListCap];
  __shared__ uint32_t s_bits[kDirtyListCap];
  __shared__ uint32_t s_bits_hi[LOGK == 6 ? kDirtyListCap : 1];
  __shared__ uint32_t s_wave[16];
  __shared__ uint32_t s_last;
  const uint32_t hb = sl.hb;
  const unsigned lane = threadIdx.x & 63u;
  const unsigned q = threadIdx.x % LPS;
  const uint32_t grp = threadIdx.x / LPS;
  const uint32_t ngrp = blockDim.x / LPS;

  PER_TRACE_DECL;
  PER_MARK(0);
  PER_MARK_HWID(15);
  // ---- 0. this subtree's height-1 nodes and their dirty flags
  const uint32_t sh1 = (hb - 1) * LOGK;
  const uint32_t n1 = sl.n[0];
  const uint32_t n1_pad = (n1 + K - 1) / K * K;
  const uint32_t lo1 = b << sh1;
  const uint32_t hi1 = min(n1, (b + 1) << sh1);
  float* lvl1 = sl.ptr[0] + (size_t)t * sl.stride[0];
  uint32_t* dirty = g.dirty + (size_t)t * g.dirty_stride;
  float* leaves = g.level[0] + (size_t)t * g.stride[0];
  const uint2* owner = reinterpret_cast<const uint2*>(g.owner) + (size_t)t * g.owner_stride;   // (value, stamp)
  // the K dirty bits of one height-1 node
  auto node_bits = [&](uint32_t node) -> unsigned long long {
    if constexpr (LOGK == 6) {
      const uint2 w = *reinterpret_cast<const uint2*>(dirty + 2 * (size_t)node);
      return ((unsigned long long)w.y << 32) | w.x;
    } else if constexpr (LOGK == 5) {
      return dirty[node];
    } else {
      const uint32_t bit0 = node << LOGK;
      return (dirty[bit0 >> 5] >> (bit0 & 31u)) & ((1u << K) - 1u);
    }
  };
  // one node per thread and sweep; the first sweep's bits are fetched together with the height-1 nodes
  const uint32_t f_first = lo1 + threadIdx.x;
  unsigned long long bits_first = 0;
  if (f_first < hi1) bits_first = node_bits(f_first);
  for (uint32_t i = threadIdx.x; i < sl.lds_floats; i += blockDim.x) {
    const uint32_t gi = lo1 + i;
    sub[i] = (i < sl.lds_off[1] || hb == 1) && gi < n1_pad ? lvl1[gi] : 0.0f;   // slot 0 from memory, the rest zero
  }
  // compact the dirty nodes into s_list / s_bits: ballot within the wave, wave totals through LDS
  const uint32_t nwaves = blockDim.x >> 6;
  uint32_t nd = 0;
  for (uint32_t f0 = lo1; f0 < hi1; f0 += blockDim.x) {
    const uint32_t f = f0 + threadIdx.x;
    unsigned long long bits = 0;
    if (f0 == lo1) bits = bits_first;
    else if (f < hi1) bits = node_bits(f);
    const unsigned long long m = __ballot(bits != 0);
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (lane == 0) s_wave[threadIdx.x >> 6] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = nd, total = nd;
    for (uint32_t wv = 0; wv < nwaves; ++wv) {
      const uint32_t c = s_wave[wv];
      if (wv < (threadIdx.x >> 6)) before += c;
      total += c;
    }
    if (bits != 0) {
      s_list[before + rank] = f;
      s_bits[before + rank] = (uint32_t)bits;
      if constexpr (LOGK == 6) s_bits_hi[before + rank] = (uint32_t)(bits >> 32);
    }
    nd = total;
    __syncthreads();
  }
  PER_MARK(1);

  if (nd > 0) {
    // ---- 1. rebuild the dirty height-1 nodes (list order is irrelevant: nodes are independent).
    // Two nodes per lane group and sweep, the loads of both issued before the first store: a
    // second sweep would otherwise cost a second trip to memory.
    using LeafVec = typename std::conditional<LOGK == 1, float2, float4>::type;
    struct Item {
      bool ok;
      uint32_t node, my;
      size_t at;
      LeafVec c;
      uint2 s[4];
    };
    // A set bit means the leaf was claimed in this batch: its stamp entry holds the winner's value.
    auto fetch = [&](uint32_t item) -> Item {
      Item it;
      it.ok = item < nd;
      const uint32_t li = it.ok ? item : nd - 1;
      it.node = s_list[li];
      unsigned long long bits = s_bits[li];
      if constexpr (LOGK == 6) bits |= (unsigned long long)s_bits_hi[li] << 32;
      if constexpr (LOGK == 1) {
        it.my = (uint32_t)bits & 3u;
        it.at = (size_t)it.node * 2;
      } else {
        it.my = (uint32_t)(bits >> (4 * q)) & 0xFu;
        it.at = (size_t)it.node * K + 4 * q;
      }
      it.c = *reinterpret_cast<const LeafVec*>(leaves + it.at);
#pragma unroll
      for (int k = 0; k < (LOGK == 1 ? 2 : 4); ++k) {
        it.s[k] = make_uint2(0, 0);
        if (it.my & (1u << k)) it.s[k] = owner[it.at + k];
      }
      return it;
    };
    auto finish = [&](Item& it) {
      float sum;
      if constexpr (LOGK == 1) {
        if (it.my & 1u) it.c.x = __uint_as_float(it.s[0].x);
        if (it.my & 2u) it.c.y = __uint_as_float(it.s[1].x);
        sum = it.c.x + it.c.y;
      } else {
        if (it.my & 1u) it.c.x = __uint_as_float(it.s[0].x);
        if (it.my & 2u) it.c.y = __uint_as_float(it.s[1].x);
        if (it.my & 4u) it.c.z = __uint_as_float(it.s[2].x);
        if (it.my & 8u) it.c.w = __uint_as_float(it.s[3].x);
        sum = (it.c.x + it.c.y) + (it.c.z + it.c.w);
#pragma unroll
        for (int k = 0; k < Fan<LOGK>::LOGLPS; ++k) sum = sum + __shfl_xor(sum, 1 << k);
      }
      return sum;
    };
    auto store = [&](const Item& it, float sum) {
      if (it.ok && it.my) *reinterpret_cast<LeafVec*>(leaves + it.at) = it.c;
      if (it.ok && q == 0) {
        lvl1[it.node] = sum;
        sub[it.node - lo1] = sum;
      }
    };
    for (uint32_t base = 0; base < nd; base += 2 * ngrp) {
      Item i0 = fetch(base + grp);
      if (base + ngrp < nd) {   // uniform over the workgroup
        Item i1 = fetch(base + ngrp + grp);
        PER_MARK(4);
        const float sum0 = finish(i0);
        const float sum1 = finish(i1);
        PER_MARK(5);
        store(i0, sum0);
        store(i1, sum1);
      } else {
        PER_MARK(4);
        const float sum0 = finish(i0);
        PER_MARK(5);
        store(i0, sum0);
      }
    }
    PER_MARK(2);
    // ---- 2. heights 2 .. hb of this subtree, from LDS
#pragma unroll
    for (int j = 1; j < kSubSlots; ++j) {
      if ((uint32_t)j < hb) {
        __syncthreads();
        const uint32_t sh = (hb - 1 - (uint32_t)j) * LOGK;
        const uint32_t a = b << sh;
        const uint32_t cnt = min(sl.n[j], (b + 1) << sh) - a;   // real nodes of this height in the subtree
        float* par = sl.ptr[j] + (size_t)t * sl.stride[j];
        for (uint32_t base = 0; base < cnt; base += ngrp) {
          const uint32_t e = base + grp;
          const bool ok = e < cnt;
          const float sum = group_sum<LOGK>(sub + sl.lds_off[j - 1] + (size_t)(ok ? e : 0u) * K, q);
          if (ok && q == 0) {
            par[a + e] = sum;
            sub[sl.lds_off[j] + e] = sum;
          }
        }
      }
    }
  }

  PER_MARK(3);
  PER_FLUSH();
  // The flags are cleared only now: a wait for loaded data also waits for every earlier store
  // of the wave, so stores that nothing depends on go last.
  for (uint32_t i = threadIdx.x; i < nd; i += blockDim.x) {
    const uint32_t node = s_list[i];
    if constexpr (LOGK == 6) {
      dirty[2 * (size_t)node] = 0;
      dirty[2 * (size_t)node + 1] = 0;
    } else {
      dirty[(node << LOGK) >> 5] = 0;   // for K < 32 the word is shared with neighbours of the same subtree
    }
  }
  // ---- 3. above the subtree: the last child to arrive recomputes the parent
  if (!chain) return;   // the heights above hb are left to their next reader
  uint32_t node = b;
  for (uint32_t h = hb + 1; h <= g.H; ++h) {
    const uint32_t parent = node >> LOGK;
    const uint32_t nchild = min((uint32_t)K, g.n[h - 1] - parent * K);
    __syncthreads();
    if (threadIdx.x == 0) {
      __threadfence();   // this workgroup's node writes are visible before its arrival is counted
      uint32_t* cnt = g.arrive + (size_t)t * g.arrive_stride + g.arrive_off[h] + parent;
      const uint32_t old = atomicAdd(cnt, 1u);
      const bool last = old == nchild - 1;
      if (last) *cnt = 0;   // ready for the next call
      s_last = last ? 1u : 0u;
      __threadfence();   // and the siblings' writes are visible to the reads below
    }
    __syncthreads();
    if (!s_last) return;
    if (threadIdx.x < 64) {
      const float sum = group_sum<LOGK>(g.level[h - 1] + (size_t)t * g.stride[h - 1] + (size_t)parent * K, lane % LPS);
      if (lane == 0) g.level[h][(size_t)t * g.stride[h] + parent] = sum;
    }
    node = parent;
  }
}

// Two 1024-lane workgroups share a compute unit only while a wave stays within an eighth of the
// SIMD's scalar and vector registers; with one more scalar register than that the second workgroup
// waits for the first to end and the kernel takes half as long again.
template <int LOGK>
__global__ void __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8)))
k_update_tree(Geom g, SubLevels sl, uint32_t chain) {
  tree_job<LOGK>(g, sl, blockIdx.y, blockIdx.x, chain);
}

// Second kernel of a fused step whose claim phase rode in the sampling kernel: the tree pass
// (workgroups 0 .. tree_blocks-1) and, beside it, what is left of the sampling call: the
// importance weights and the rows of the sampled indices (JobRanges, offset by tree_blocks).  The
// tree pass is a chain of dependent memory trips and the row traffic fills the gaps; launched with
// workgroups of at most 512 lanes so that the two kinds share the compute units.
template <int LOGK>
__global__ void __launch_bounds__(512)
k_tree_finish(Geom g, SubLevels sl, uint32_t chain, uint32_t tree_blocks, FieldTable ft, JobRanges jr, FinishArgs a) {
  const uint32_t t = blockIdx.y;
  if (blockIdx.x < tree_blocks) {
    tree_job<LOGK>(g, sl, t, blockIdx.x, chain);
    return;
  }
  const uint32_t b = blockIdx.x - tree_blocks;
  if (b < jr.first[1]) {
    weights_job(g, t, a.B, a.size, a.beta, a.w, a.parity, b, jr.first[1]);
    return;
  }
#pragma unroll
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f)
    if (b >= jr.first[2 + f] && b < jr.first[3 + f]) {
      rows_job<true>(ft, f, t, a.B, a.idx, 0, g.N, g.status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
      return;
    }
}

// Height of the workgroup roots of the tree pass: the whole tree for small trees, else the
// lowest height whose subtrees hold at least 64 height-1 nodes (so that dirty words are never
// shared between workgroups).
static uint32_t tree_pass_height(const Geom& g) {
  if (g.n[1] <= kDirtyListCap) return g.H;
  uint32_t hb = 1;
  while (hb < g.H && (1ull << ((hb - 1) * g.logK)) < 64) ++hb;
  return hb;
}

// Heights above this one may be left stale by an update (0: never).
uint32_t lazy_top_height(const Geom& g, const Tuning& tn) {
  const uint32_t hb = tree_pass_height(g);
  return tn.lazy_top && hb < g.H && g.n[hb] <= kLazyTopNodes ? hb : 0u;
}

// Sub-level descriptors, workgroup size and LDS floats of the tree pass for update batches of B.
template <int LOGK>
static hipError_t tree_pass_shape(const Geom& g, const Tuning& tn, uint32_t B, SubLevels* out, uint32_t* tblock_out) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t hb = tree_pass_height(g);
  if (hb > (uint32_t)kSubSlots) return hipErrorInvalidValue;   // cannot happen for fanouts and capacities accepted at create
  SubLevels sl{};
  sl.hb = hb;
  uint32_t off = 0;
  for (uint32_t h = 1; h <= hb; ++h) {
    const uint32_t j = h - 1;
    sl.ptr[j] = g.level[h];
    sl.stride[j] = g.stride[h];
    sl.n[j] = g.n[h];
    sl.lds_off[j] = off;
    // nodes of this height under one workgroup root, padded to whole child groups
    const uint64_t full = 1ull << ((hb - h) * LOGK);
    const uint64_t padded = h < hb ? ((uint64_t)g.n[h] + K - 1) / K * K : 1;
    off += (uint32_t)(full < padded ? full : padded);
  }
  sl.lds_floats = off;
  // Unless told otherwise: enough lane groups to rebuild in one sweep twice the dirty height-1 nodes a
  // subtree gets on average (never more than it has), so that small batches do not launch idle waves.
  uint32_t tblock = tn.tree_block;
  if (tblock == 0) {
    const uint64_t per_subtree = hb > 1 ? sl.lds_off[1] : 1;
    uint64_t expect = 2 * ((uint64_t)B + g.n[hb] - 1) / g.n[hb];
    if (expect > per_subtree) expect = per_subtree;
    uint64_t want = expect * Fan<LOGK>::LPS;
    if (hb > 2) {   // the dense heights of the subtree want a lane group per height-2 node
      const uint64_t dense = (uint64_t)(sl.lds_off[2] - sl.lds_off[1]) * Fan<LOGK>::LPS;
      if (dense > want) want = dense;
    }
    tblock = (uint32_t)(want > 1024 ? 1024 : (want + 63) / 64 * 64);
    if (tblock < 64) tblock = 64;
  }
  *out = sl;
  *tblock_out = tblock;
  return hipSuccess;
}

template <int LOGK>
static hipError_t launch_tree_k(const Geom& g, const Tuning& tn, uint32_t B, hipStream_t s) {
  SubLevels sl;
  uint32_t tblock;
  hipError_t e = tree_pass_shape<LOGK>(g, tn, B, &sl, &tblock);
  if (e != hipSuccess) return e;
  PER_LAUNCH(KID_UPDATE_TREE, k_update_tree<LOGK>, dim3(g.n[sl.hb], g.T), dim3(tblock), (size_t)sl.lds_floats * 4, s, g,
             sl, lazy_top_height(g, tn) ? 0u : 1u);
  return hipGetLastError();
}

// The tree pass of an update batch of B together with the weights and row jobs in `a` / `rows`.
template <int LOGK>
static hipError_t launch_tree_finish_k(const Geom& g, const Tuning& tn, uint32_t B, const FieldTable* rows,
                                       const FinishArgs& a, hipStream_t s) {
  SubLevels sl;
  uint32_t tblock;
  hipError_t e = tree_pass_shape<LOGK>(g, tn, B, &sl, &tblock);
  if (e != hipSuccess) return e;
  if (tblock > 512) tblock = 512;   // half the lanes of a compute unit are left to the other jobs
  FieldTable ft{};
  if (rows) ft = *rows;
  const JobRanges jr = job_ranges(rows ? &ft : nullptr, a.B, tblock, a.w ? a.B : 0u, 0u);
  const uint32_t tree_blocks = g.n[sl.hb];
  PER_LAUNCH(KID_TREE_FINISH, k_tree_finish<LOGK>, dim3(tree_blocks + jr.first[2 + kMaxFields], g.T), dim3(tblock),
             (size_t)sl.lds_floats * 4, s, g, sl, lazy_top_height(g, tn) ? 0u : 1u, tree_blocks, ft, jr, a);
  return hipGetLastError();
}

template <int LOGK>
static hipError_t launch_update_k(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s) {
  const uint32_t block = tn.update_block;
  PER_LAUNCH(KID_UPDATE_CLAIM, k_update_claim, dim3((c.B + block - 1) / block, g.T), dim3(block), 0, s, g, c);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_tree_k<LOGK>(g, tn, c.B, s);
}

hipError_t launch_update(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s) {
#define CALL(L) launch_update_k<L>(g, tn, c, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

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

// ---------------------------------------------------------------------------------
// a stream of steps on an LDS-resident tree (small buffers)
// ---------------------------------------------------------------------------------
// The paper keeps the sum tree of its Replay Manager in on-chip memory and lets one kernel, started
// once, work through a stream of requests (Section V-A, "RM on FPGA": buffers of 10K to 100K entries,
// autorun kernels that need no launch per request).  The counterpart here: when all heights of a
// tree fit the LDS of one compute unit, one workgroup per tree loads the tree once, runs a whole
// list of steps (insert -> sample -> gather -> update, the order of the separate calls) against
// the LDS copy, and stores the tree back at the end.  Every tree access of a step is then an LDS
// access; only rows, inputs and outputs travel to memory.  Results are those of the separate calls.
//
// Update inside one workgroup: a valid element raises the leaf (reinterpreted as an integer) to
// a marker above every valid priority pattern, 0x80000001 + its position, by an LDS atomic max; the
// element that finds its own marker afterwards is the last writer and stores its value; then
// every valid element recomputes its ancestors height by height (elements that share a parent
// store the same sum).
struct StreamKernelArgs {           // one kernel argument, so that both parts sit at known offsets of the segment
  Geom g;
  StreamArgs a;
};

// Sum of the 4*N children behind g4 in the balanced pairwise order, by a single lane.
template <int N>
__device__ __forceinline__ float sum_chunks(const float4* g4) {
  if constexpr (N == 1) {
    const float4 x = g4[0];
    return (x.x + x.y) + (x.z + x.w);
  } else {
    return sum_chunks<N / 2>(g4) + sum_chunks<N / 2>(g4 + N / 2);
  }
}
template <int LOGK>
__device__ __forceinline__ float lane_group_sum(const float* grp) {
  if constexpr (LOGK == 1) {
    const float2 c = *reinterpret_cast<const float2*>(grp);
    return c.x + c.y;
  } else {
    return sum_chunks<(1 << LOGK) / 4>(reinterpret_cast<const float4*>(grp));
  }
}

// Every active lane recomputes the ancestors of its leaf in the LDS tree, one height per barrier.
template <int LOGK>
__device__ __forceinline__ void resum_paths_lds(float* tree, const uint32_t* off, uint32_t H, bool active, uint32_t leaf) {
  constexpr int K = Fan<LOGK>::K;
  for (uint32_t h = 1; h <= H; ++h) {
    __syncthreads();
    if (active) {
      const uint32_t parent = leaf >> (h * LOGK);
      tree[off[h] + parent] = lane_group_sum<LOGK>(tree + off[h - 1] + (size_t)parent * K);
    }
  }
}

template <int LOGK>
__global__ void __launch_bounds__(1024)
k_run_steps(StreamKernelArgs ka) {
  constexpr int K = Fan<LOGK>::K;
  const Geom& g = ka.g;
  const StreamArgs& a = ka.a;
  extern __shared__ __attribute__((aligned(16))) float tree[];
  __shared__ LevelTable tab;
  __shared__ uint32_t s_off[kMaxHeight + 2];
  __shared__ uint32_t s_max, s_vmin, s_flags;
  const uint32_t t = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const uint32_t H = g.H, N = g.N, T = g.T, B = a.B, n_ins = a.n_insert;
  fill_level_table(H, t, &tab);
  if (tid >= 64 && tid <= 64 + H + 1)
    s_off[tid - 64] = kernarg_at<StreamArgs>(offsetof(StreamKernelArgs, a))->off[tid - 64];
  if (tid == 0) {
    s_max = read_max_bits(g, t);
    s_flags = 0;
  }
  __syncthreads();
  for (uint32_t h = 0; h <= H; ++h) {   // the whole tree, zero padding included
    const float* lvl = tab.lvl[h];
    float* dst = tree + s_off[h];
    for (uint32_t e = tid; e < s_off[h + 1] - s_off[h]; e += blockDim.x) dst[e] = lvl[e];
  }
  uint32_t* s_idx = reinterpret_cast<uint32_t*>(tree + s_off[H + 1]);   // indices sampled in the current step
  uint32_t* leaf_bits = reinterpret_cast<uint32_t*>(tree + s_off[0]);
  uint32_t cursor = a.cursor, size = a.size;
  uint32_t flags = 0;
  PER_TRACE_DECL;

  for (uint32_t s = 0; s < a.n_steps; ++s) {
    PER_MARK(0);
    const size_t bo = ((size_t)s * T + t) * B + tid;
    // inputs of this step, fetched before the tree work
    float u_i = 0.0f, up_v = 0.0f;
    uint32_t up_i = 0;
    if (tid < B) {
      u_i = a.u[bo];
      if (a.upd_prio) {
        up_v = a.upd_prio[bo];
        if (!a.upd_is_sampled) up_i = a.upd_idx[bo];
      }
    }
    const float beta = a.beta[s];

    // ---- insertion: rows, leaves (given value or the running maximum on entry), ancestors
    if (n_ins) {
      (void)move_rows_one_workgroup<false>(a.ins, t, ((uint64_t)s * T + t) * n_ins, n_ins, cursor, N, nullptr);
      __syncthreads();   // (also: the tree is loaded, the last step's update is complete)
      const float max_on_entry = __uint_as_float(s_max);
      __syncthreads();
      bool ok = false;
      uint32_t slot = 0;
      if (tid < n_ins) {
        uint64_t sl = (uint64_t)cursor + tid;
        if (sl >= N) sl -= N;
        slot = (uint32_t)sl;
        float v = max_on_entry;
        ok = true;
        if (a.ins_prio) {
          v = a.ins_prio[((size_t)s * T + t) * n_ins + tid];
          ok = valid_priority(v);
          if (ok && v > 0.0f) atomicMax(&s_max, __float_as_uint(v));
          if (!ok) flags |= 2u;
        }
        if (ok) tree[s_off[0] + slot] = v;
      }
      resum_paths_lds<LOGK>(tree, s_off, H, ok, slot);
      const uint64_t end = (uint64_t)cursor + n_ins;
      cursor = (uint32_t)(end >= N ? end - N : end);
      size = size + n_ins > N ? N : size + n_ins;
    }
    if (tid == 0) s_vmin = 0x7F800000u;
    __syncthreads();
    PER_MARK(1);

    // ---- priority sampling and importance weights
    const float total = tree[s_off[H]];
    uint32_t node = 0xFFFFFFFFu;
    float val = 0.0f;
    if (total > 0.0f) {
      const uint32_t si = tid < B ? tid : B - 1;
      float r = ((float)si + u_i) * (total / (float)B);
      node = 0;
      val = total;
      for (uint32_t h = H; h-- > 0;) {
        unsigned child;
        descend_lane<LOGK>(tree + s_off[h] + (size_t)node * K, r, child, val);
        node = node * K + child;
      }
      if (a.out_w && tid < B) atomicMin(&s_vmin, __float_as_uint(val));
    } else if (tid == 0) {
      flags |= 4u;
    }
    if (tid < B) {
      s_idx[tid] = node;
      a.out_idx[bo] = node;
      if (a.out_prio) a.out_prio[bo] = val;
    }
    __syncthreads();
    if (a.out_w && tid < B)
      a.out_w[bo] = total > 0.0f ? importance_weight(val, __uint_as_float(s_vmin), total, size, beta) : 0.0f;

    PER_MARK(2);
    // ---- rows of the sampled indices
    if (move_rows_one_workgroup<true>(a.rows, t, ((uint64_t)s * T + t) * B, B, 0, N, s_idx)) flags |= 1u;

    PER_MARK(3);
    // ---- priority update: last writer by LDS atomics, then the ancestors
    if (a.upd_prio) {
      const uint32_t i = a.upd_is_sampled ? node : up_i;
      bool valid = false;
      if (tid < B) {
        if (!(i < size)) flags |= 1u;
        else if (!valid_priority(up_v)) flags |= 2u;
        else valid = true;
      }
      const uint32_t mark = 0x80000001u + tid;
      if (valid) atomicMax(&leaf_bits[i], mark);
      __syncthreads();
      const bool won = valid && leaf_bits[i] == mark;
      __syncthreads();
      if (won) tree[s_off[0] + i] = up_v;
      if (valid && up_v > 0.0f) atomicMax(&s_max, __float_as_uint(up_v));
      resum_paths_lds<LOGK>(tree, s_off, H, valid, i);
    }
    __syncthreads();
    PER_MARK(4);
  }
  PER_FLUSH();

  // ---- the tree goes back to memory
  for (uint32_t h = 0; h <= H; ++h) {
    float* lvl = tab.lvl[h];
    const float* src = tree + s_off[h];
    for (uint32_t e = tid; e < tab.n[h]; e += blockDim.x) lvl[e] = src[e];
  }
  if (tid == 0) g.max_v[t] = __uint_as_float(s_max);
  if (flags) atomicOr(&s_flags, flags);
  __syncthreads();
  if (tid == 0 && s_flags) atomicOr(&g.status[t], s_flags);
}

// LDS floats of a whole tree (every height padded to whole child groups), or 0 if it cannot be
// held beside the step kernel's other LDS data.
constexpr uint32_t kStreamLdsBytes = 156 * 1024;
uint32_t stream_tree_floats(const Geom& g, uint32_t* off) {
  uint64_t floats = 0;
  for (uint32_t h = 0; h <= g.H; ++h) {
    if (off) off[h] = (uint32_t)floats;
    floats += h < g.H ? ((uint64_t)g.n[h] + g.K - 1) / g.K * g.K : 4;   // (the root padded to 16 bytes)
    if (floats * 4 > kStreamLdsBytes) return 0;
  }
  if (off) off[g.H + 1] = (uint32_t)floats;
  return (floats + 1024) * 4 <= kStreamLdsBytes ? (uint32_t)floats : 0u;
}

template <int LOGK>
static hipError_t launch_run_steps_k(const Geom& g, const Tuning& tn, StreamArgs a, hipStream_t s) {
  StreamKernelArgs ka{};
  ka.g = g;
  ka.a = a;
  const uint32_t floats = stream_tree_floats(g, ka.a.off);
  if (!floats) return hipErrorInvalidValue;
  const size_t bytes = ((size_t)floats + 1024) * 4;   // the tree and the sampled indices of one step
  if (bytes > 64 * 1024) {   // more than the default dynamic LDS limit has to be requested per kernel
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_run_steps<LOGK>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
  }
  // always the largest workgroup, also for small batches: measured faster than a workgroup of the batch's
  // size (the tree copy and the row movers use all lanes)
  PER_LAUNCH(KID_RUN_STEPS, k_run_steps<LOGK>, dim3(g.T), dim3(1024), bytes, s, ka);
  return hipGetLastError();
}

hipError_t launch_run_steps(const Geom& g, const Tuning& tn, const StreamArgs& a, hipStream_t s) {
#define CALL(L) launch_run_steps_k<L>(g, tn, a, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

// ---------------------------------------------------------------------------------
// priority retrieval
// ---------------------------------------------------------------------------------
__global__ void k_get_priority(Geom g, uint32_t n, const uint32_t* __restrict__ idx, float* __restrict__ out) {
  const uint32_t t = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const uint32_t i = idx[(size_t)t * n + j];
  if (i < g.N) {
    out[(size_t)t * n + j] = g.level[0][(size_t)t * g.stride[0] + i];
  } else {
    out[(size_t)t * n + j] = 0.0f;
    atomicOr(&g.status[t], 1u);
  }
}

hipError_t launch_get_priority(const Geom& g, const Tuning& tn, uint32_t n, const uint32_t* idx, float* out,
                               hipStream_t s) {
  PER_LAUNCH(KID_GET_PRIORITY, k_get_priority, dim3((n + 255) / 256, g.T), dim3(256), 0, s, g, n, idx, out);
  return hipGetLastError();
}

}  // namespace per
