// Priority sampling (with the claim phase and the uniforms it can carry), importance weights, and the launcher of the fused sampling calls.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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
         uint32_t weight_mode, int stale, uint32_t claim_blocks, ClaimArgs c, int claim_mode, RngArgs rng) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  constexpr int ROW = K + 4;                  // staging row, floats
  using Vec = typename std::conditional<LOGK == 1, float2, float4>::type;
  constexpr int VF = sizeof(Vec) / 4;
  touch_kernel_arguments<kernarg_lines<Geom, TopCopy, uint32_t, uint32_t, float, const float*, uint32_t*, float*, float*, uint32_t,
                                       int, uint32_t, ClaimArgs, int, RngArgs>()>();
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
  // which buffer of partial batch minima this call fills (stable while this kernel runs: the weights job of
  // the call before has written it), fetched in that same trip
  uint32_t vbuf = 0;
  const bool partial_minima = out_w && sample_blocks > 1;
  if (partial_minima) vbuf = read_word_with_the_loads(g.vnext + t);   // (its low bit; taken where it is used, so that nothing waits for the word here)
  // the new priority of this lane's sample and the running maximum, likewise
  float upd_v = 0.0f;
  uint32_t max_seen = 0;
  uint32_t claim_first = 1;
  if (claim_mode == 1) {
    upd_v = c.prio[o];
    max_seen = read_max_bits(g, t);
    claim_first = claim_base(g, t, c.group_mode);
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

  // The first workgroup of each tree puts the heights rebuilt above back into memory (also when nothing can be
  // sampled: the host has noted that this kernel makes them current).
  auto store_rebuilt_top = [&]() {
    if (stale >= 0 && bx == 0) {
#pragma unroll
      for (int i = 0; i < kTopSlots; ++i)
        if (i < stale) {
          float* dst = g.level[H - 1 - (uint32_t)i] + (size_t)t * g.stride[H - 1 - (uint32_t)i];
          for (uint32_t j = threadIdx.x; j < tc.nreal[i]; j += blockDim.x) dst[j] = lds[off[i] + j];
        }
      if (threadIdx.x == 0) g.root[(size_t)t * g.root_stride] = total;
    }
  };

  if (!(total > 0.0f)) {   // nothing can be sampled from this tree (uniform over the block)
    store_rebuilt_top();
    if (active) {
      out_idx[o] = 0xFFFFFFFFu;
      if (out_prio) out_prio[o] = 0.0f;
      if (out_w) out_w[o] = 0.0f;
    }
    // (a fused update of these samples finds no valid index: every element is out of range)
    if (bx == 0 && threadIdx.x == 0) {
      atomicOr(&g.status[t], claim_mode == 1 ? 5u : 4u);
      if (partial_minima) g.vcur[t] = not_before_here(vbuf) & 1u;   // the weights job of this call runs all the same
      if (claim_mode == 1) leave_claim_base(g, t, c.group_mode, true, claim_first);
    }
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
  // earlier store of the wave.
  store_rebuilt_top();
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
      if (weight_mode & kWeightBufferNorm) mm = buffer_min_bits(g, t, weight_mode);   // (uniform over the launch)
      if (active) out_w[o] = importance_weight(val, __uint_as_float(mm), beta);
    } else {                // partial minima, spread over kVminSlots addresses; the weights job finishes
      if (active) out_w[o] = val;
      vbuf = not_before_here(vbuf) & 1u;
      if (bx == 0 && threadIdx.x == 0) g.vcur[t] = vbuf;   // tells the weights job of this call which buffer it is
      if (lane == 0)
        atomicMin(&g.vmin[((size_t)vbuf * g.T + t) * kVminSlots + ((bx * (blockDim.x >> 6) + wave) % kVminSlots)], m);
    }
  }
  if (claim_mode == 1) {   // element s of the update batch is this lane's own sample
    uint32_t mx = 0, flags = 0;
    if (active) claim_element(g, t, size, c.group_mode, claim_first, s, node, upd_v, mx, flags);
    raise_max(g, t, mx, max_seen);
    if (flags) atomicOr(&g.status[t], flags);
    leave_claim_base(g, t, c.group_mode, bx == 0 && threadIdx.x == 0, claim_first);
  }
}

// Finishes the importance weights of tree t: folds the partial minima that the sampling kernel of this
// call has left in one of the two vmin buffers and turns the sampled values left in w into weights.
// Called by whole workgroups of any size.  Which buffer: vcur, written by that sampling kernel.  The
// first workgroup re-arms the other buffer and makes it the one the next sampling kernel fills (vnext;
// only kernels of later calls read that word).  Nothing of this alternation lives on the host, so a
// captured call can be replayed.  `mode`: see kWeightBufferNorm.
__device__ __forceinline__ void weights_job(const Geom& g, uint32_t t, uint32_t B, uint32_t size, float beta,
                                            float* __restrict__ w, uint32_t mode, uint32_t job_block,
                                            uint32_t job_blocks) {
  __shared__ uint32_t s_wmin[16];
  if (job_block != 0 && job_block * blockDim.x >= B) return;   // nothing to do for this workgroup
  // (both buffers are fetched beside the word that says which one counts: one trip instead of two)
  const uint32_t* part0 = g.vmin + (size_t)t * kVminSlots;
  const uint32_t* part1 = g.vmin + ((size_t)g.T + t) * kVminSlots;
  uint32_t m0 = 0x7F800000u, m1 = 0x7F800000u;
  const uint32_t vword = read_word_with_the_loads(g.vcur + t);
  for (uint32_t j = threadIdx.x; j < kVminSlots; j += blockDim.x) {
    m0 = part0[j] < m0 ? part0[j] : m0;
    m1 = part1[j] < m1 ? part1[j] : m1;
  }
  const uint32_t vbuf = not_before_here(vword) & 1u;
  uint32_t m = wave_min_u32(vbuf ? m1 : m0);
  if ((threadIdx.x & 63u) == 0) s_wmin[threadIdx.x >> 6] = m;
  if (job_block == 0) {
    for (uint32_t j = threadIdx.x; j < kVminSlots; j += blockDim.x)
      g.vmin[((size_t)(vbuf ^ 1u) * g.T + t) * kVminSlots + j] = 0x7F800000u;
    if (threadIdx.x == 0) g.vnext[t] = vbuf ^ 1u;
  }
  __syncthreads();
  uint32_t mm = 0x7F800000u;
  for (uint32_t wv = 0; wv < (blockDim.x >> 6); ++wv) mm = s_wmin[wv] < mm ? s_wmin[wv] : mm;
  // No minimum at all means that nothing could be sampled (the tree's total was zero): weights 0.  (The root
  // itself must not be consulted here: a tree pass running beside this job may already have rewritten it.)
  const bool nothing_sampled = mm == 0x7F800000u;
  if (mode & kWeightBufferNorm) mm = buffer_min_bits(g, t, mode);   // (uniform over the launch)
  for (uint32_t i = job_block * blockDim.x + threadIdx.x; i < B; i += job_blocks * blockDim.x) {
    const size_t o = (size_t)t * B + i;
    w[o] = nothing_sampled ? 0.0f : importance_weight(w[o], __uint_as_float(mm), beta);
  }
}

__global__ void k_weights(Geom g, uint32_t B, uint32_t size, float beta, float* __restrict__ w, uint32_t mode) {
  weights_job(g, blockIdx.y, B, size, beta, w, mode, blockIdx.x, gridDim.x);
}

template <int LOGK>
static hipError_t launch_resum_top_k(const Geom& g, const Tuning& tn, uint32_t hb, hipStream_t s);
static hipError_t launch_finish(const Geom& g, const Tuning& tn, const FieldTable* rows, const FinishArgs& a,
                                hipStream_t s);
template <int LOGK>
static hipError_t launch_tree_k(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s);
template <int LOGK>
static hipError_t launch_tree_finish_k(const Geom& g, const Tuning& tn, const ClaimArgs& c, const FieldTable* rows,
                                       const FinishArgs& a, hipStream_t s);

// Sampling call with whatever is fused into it.  rows: gather of the sampled rows.  claim: a priority
// update whose claim phase runs where claim_mode says (CLAIM_INLINE / CLAIM_BLOCKS: in the sampling
// kernel, the tree pass then shares the second kernel with the weights and row jobs; CLAIM_FINISH: in
// the second kernel, the tree pass is a third).
template <int LOGK>
static hipError_t launch_sample_k(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, float beta,
                                  const float* u, const RngArgs& rng, uint32_t* out_idx, float* out_w,
                                  float* out_prio, uint32_t weight_mode, uint32_t stale_hb, const FieldTable* rows,
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
  e = grant_lds<&k_sample<LOGK>>(tn, bytes);
  if (e != hipSuccess) return e;
  if (!claim) claim_mode = CLAIM_NONE;
  const bool claim_here = claim_mode == CLAIM_INLINE || claim_mode == CLAIM_BLOCKS;
  uint32_t claim_blocks = 0;
  if (claim_mode == CLAIM_BLOCKS) {
    claim_blocks = (claim->B + block - 1) / block;
    if (claim_blocks > 4096) claim_blocks = 4096;   // the claim job strides
  }
  PER_LAUNCH(KID_SAMPLE, k_sample<LOGK>, dim3(gx + claim_blocks, g.T), dim3(block), bytes, s, g, tc, B, size, beta, u,
             out_idx, out_prio, out_w, weight_mode, stale, claim_blocks, claim_here ? *claim : ClaimArgs{},
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
    a.weight_mode = weight_mode;
    if (claim_here) {   // second kernel: tree pass beside the weights and the rows
      if (rows || finish_weights) return launch_tree_finish_k<LOGK>(g, tn, *claim, rows, a, s);
      return launch_tree_k<LOGK>(g, tn, *claim, s);
    }
    // second kernel: rows, weights and the claim phase; the tree pass follows
    a.has_claim = claim ? 1u : 0u;
    if (claim) a.claim = *claim;
    e = launch_finish(g, tn, rows, a, s);
    if (e != hipSuccess || !claim) return e;
    return launch_tree_k<LOGK>(g, tn, *claim, s);
  }
  if (!finish_weights) return e;
  PER_LAUNCH(KID_WEIGHTS, k_weights, dim3((B + 255) / 256, g.T), dim3(256), 0, s, g, B, size, beta, out_w, weight_mode);
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
                         const RngArgs& rng, uint32_t* out_idx, float* out_w, float* out_prio, uint32_t weight_mode,
                         uint32_t stale_hb, const FieldTable* rows, const ClaimArgs* claim, int claim_mode,
                         hipStream_t s) {
#define CALL(L) launch_sample_k<L>(g, tn, B, size, beta, u, rng, out_idx, out_w, out_prio, weight_mode, stale_hb, rows, claim, claim_mode, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}
