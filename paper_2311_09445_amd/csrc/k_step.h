// One iteration of Listing 2 whose update targets the batch it draws, with sampling and update in one kernel.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// sampling and the update of the sampled batch, one workgroup per subtree
// ---------------------------------------------------------------------------------
// Stratified targets grow with the sample number and the walk is monotone in the target, so the samples
// that end under one node of the tree are a contiguous run of sample numbers.  Workgroup b of tree t owns
// the subtree under node b of height ho ("owner height").  It finds its run of samples, walks them down
// (the heights ho .. H-1 of the whole tree and the heights 1 .. ho-1 of its own subtree from LDS copies, the
// leaf groups from memory), and then applies the update of exactly those samples to its own subtree:
// every leaf, every height-1 node and every higher node of the subtree is read and written by this
// workgroup only, so the update needs no claim phase, no atomics and no second pass over the leaf groups
// (they are still in LDS from the walk).  Sampling sees the tree as it was before the call because a
// workgroup finishes all its walks before it changes anything, and what all workgroups read, the nodes of
// height ho, is never written in place: the new value of node b goes to the other one of two arrays (the
// level array itself and a side array), and the workgroup that finishes last makes that one current.
// The heights above ho are rebuilt in LDS from height ho by every workgroup (a few child groups) and are
// left stale in memory, as after any update.
//
// Last writer: element j of the update targets the leaf drawn by sample pos[j] (no map: by sample j).  The
// samples of one leaf are neighbours in a workgroup's run, so the winner of a leaf is the largest j among
// the elements aimed at that run of samples.  With a map, builder workgroups in front of the grid first
// record for every sample the largest j aimed at it (an atomic max into a scratch word per sample that the
// sample's lane takes back out with an exchange); the owners wait for them at the point where they need the
// words, which the builders, being dispatched first and waiting for nothing, always reach.
constexpr int kStepTop = 4;          // most heights ho .. H-1
constexpr int kStepSub = 4;          // most heights 1 .. ho-1
constexpr uint32_t kStepPad = 4;     // sample numbers looked at in front of the estimated start of the run
constexpr uint32_t kNoKey = 0xFFFFFFFFu;
constexpr uint32_t kStepSpinLimit = 1u << 20;   // polls of the builders' counter before an owner gives up

struct StepShape {
  float* top_ptr[kStepTop];        // height ho + i of tree 0 (i = 0: the level array of height ho)
  uint32_t top_stride[kStepTop];   // floats between trees
  uint32_t top_cnt[kStepTop];      // floats kept in LDS: whole child groups, n[ho+i+1] * K
  uint32_t top_n[kStepTop];        // real nodes n[ho+i]
  uint32_t top_off[kStepTop];      // where in LDS (floats)
  float* sub_ptr[kStepSub];        // height 1 + i of tree 0
  uint32_t sub_stride[kStepSub];
  uint32_t sub_cnt[kStepSub];      // nodes of that height under one owner: K^(ho-1-i)
  uint32_t sub_pad[kStepSub];      // nodes of that height in memory, padded to whole groups
  uint32_t sub_off[kStepSub];      // where in LDS (floats)
  uint32_t n_top, n_sub;           // H - ho, ho - 1
  uint32_t rows_off;               // LDS: (block + 1) staging rows of K + 4 floats (16-byte aligned)
  uint32_t key_off;                // LDS: key[block + 2], wpos[block + 1], wval[block + 1], touch[block + 1]
  uint32_t owners;                 // n[ho]: owner workgroups per tree
  uint32_t builders;               // builder workgroups per tree in front of them (0: no position map)
  float* side;                     // [T][side_stride] second array for the nodes of height ho
  uint32_t side_stride;
  uint32_t* ctl;                   // [T][4]: which array is current (0: the level array), builders done, owners done, spare
  uint32_t* inv;                   // [T][inv_stride] per sample: 1 + the largest update element aimed at it (zero between calls)
  uint32_t inv_stride;
};

// Pairwise sum of the K floats of a staged row, in the order of group_sum.
template <int LOGK>
__device__ __forceinline__ float row_sum(const float* row) {
  if constexpr (LOGK == 1) {
    return row[0] + row[1];
  } else {
    constexpr int C = (1 << LOGK) / 4;
    const float4* r4 = reinterpret_cast<const float4*>(row);
    float s[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const float4 x = r4[c];
      s[c] = (x.x + x.y) + (x.z + x.w);
    }
#pragma unroll
    for (int w = C; w > 1; w >>= 1)
#pragma unroll
      for (int c = 0; c < w / 2; ++c) s[c] = s[2 * c] + s[2 * c + 1];
    return s[0];
  }
}

// The update of one chunk of a workgroup's samples, on LDS arrays indexed by slot: slot 0 carries what the
// chunk before left open, slot 1 + i belongs to lane i.
//   key[slot]   leaf of the slot's sample (kNoKey: none); key[block + 1] is always kNoKey
//   wpos[slot]  1 + the largest update element aimed at that sample (0: none), wval[slot] its value
//   rows[slot]  the K leaves of the sample's group as staged for the walk (K + 4 floats apart)
//   touch[slot] (group heads only) a leaf of the group was rewritten
// A run of equal keys is one leaf; its last writer is the largest wpos in the run.  A run of keys with equal
// key >> LOGK is one child group; the row of its first slot (the head) collects the new leaf values, and at
// the end of the run its pairwise sum is the new height-1 node.  When the chunk is not the workgroup's
// last, the runs that reach its last slot stay open and move to slot 0 of the next chunk.
// Three phases, a workgroup barrier after each; thread i works on slot i, thread 0 also on slot `block`.
struct ChunkLds {
  uint32_t* key;
  uint32_t* wpos;
  float* wval;
  uint32_t* touch;
  float* rows;
};
template <int LOGK>
__device__ __forceinline__ uint32_t group_head(const ChunkLds& c, uint32_t slot) {
  const uint32_t g = c.key[slot] >> LOGK;
  uint32_t h = slot;
  while (h > 0 && c.key[h - 1] != kNoKey && (c.key[h - 1] >> LOGK) == g) --h;
  return h;
}
// Phase A: the slot that ends a leaf's run hands the winner's value to the group head's row and to memory.
template <int LOGK>
__device__ __forceinline__ void chunk_leaves(const ChunkLds& c, uint32_t slot, uint32_t block, bool last_chunk,
                                             float* __restrict__ leaves, uint32_t& open_pos, float& open_val) {
  constexpr int K = 1 << LOGK;
  constexpr int ROW = K + 4;
  const uint32_t k = c.key[slot];
  if (k == kNoKey) return;
  const bool open = slot == block && !last_chunk;
  if (!open && c.key[slot + 1] == k) return;   // the run goes on
  uint32_t best = c.wpos[slot];
  float bv = c.wval[slot];
  uint32_t j = slot;
  while (j > 0 && c.key[j - 1] == k) {
    --j;
    if (c.wpos[j] > best) {
      best = c.wpos[j];
      bv = c.wval[j];
    }
  }
  if (open) {
    open_pos = best;
    open_val = bv;
    return;
  }
  if (best) {
    const uint32_t h = group_head<LOGK>(c, j);
    c.rows[(size_t)h * ROW + (k & (uint32_t)(K - 1))] = bv;
    c.touch[h] = 1u;
    leaves[k] = bv;
  }
}
// Phase B: the slot that ends a group's run recomputes the height-1 node from the head's row.  Returns the head
// of the run that stays open (only for slot == block of a chunk that is not the last), else kNoKey.
template <int LOGK>
__device__ __forceinline__ uint32_t chunk_groups(const ChunkLds& c, uint32_t slot, uint32_t block, bool last_chunk,
                                                 float* __restrict__ lvl1, float* sub1, uint32_t lo1) {
  constexpr int K = 1 << LOGK;
  constexpr int ROW = K + 4;
  const uint32_t k = c.key[slot];
  if (k == kNoKey) return kNoKey;
  const uint32_t g = k >> LOGK;
  const bool open = slot == block && !last_chunk;
  if (!open && c.key[slot + 1] != kNoKey && (c.key[slot + 1] >> LOGK) == g) return kNoKey;   // the run goes on
  const uint32_t h = group_head<LOGK>(c, slot);
  if (open) return h;
  if (c.touch[h]) {
    const float sum = row_sum<LOGK>(c.rows + (size_t)h * ROW);
    lvl1[g] = sum;
    sub1[g - lo1] = sum;
  }
  return kNoKey;
}

template <int LOGK>
__global__ void __launch_bounds__(512)
k_step(Geom g, StepShape sh, uint32_t B, uint32_t size, const float* __restrict__ u, RngArgs rng,
       uint32_t* __restrict__ out_idx, float* __restrict__ out_prio, float* __restrict__ out_w,
       const float* __restrict__ upd_prio, const uint32_t* __restrict__ upd_pos) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  constexpr int ROW = K + 4;
  static_assert(LOGK >= 3, "the staged walk needs K >= 8");
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ uint32_t s_u32[8];
  __shared__ double s_est;
  const uint32_t t = blockIdx.y;
  const uint32_t tid = threadIdx.x;
  const uint32_t BD = blockDim.x;
  const unsigned lane = tid & 63u;
  const unsigned wave = tid >> 6;
  uint32_t* ctl = sh.ctl + (size_t)t * 4;
  uint32_t* inv = sh.inv + (size_t)t * sh.inv_stride;
  const int n_top = (int)sh.n_top, n_sub = (int)sh.n_sub;

  // which of the two arrays holds the nodes of height ho (stable while this kernel runs: the workgroup that
  // finishes last flips it)
  const uint32_t sel = read_word_with_the_loads(ctl) & 1u;
  const float* cur_ho = sel ? sh.side + (size_t)t * sh.side_stride : sh.top_ptr[0] + (size_t)t * sh.top_stride[0];
  float* new_ho = sel ? sh.top_ptr[0] + (size_t)t * sh.top_stride[0] : sh.side + (size_t)t * sh.side_stride;

  // ------------------------------------------------------------------ builder workgroups (position map only)
  if (blockIdx.x < sh.builders) {
    const uint32_t max_seen = read_max_bits(g, t);
    uint32_t mx = 0, f_idx = 0, f_prio = 0, acc = 0;
    for (uint32_t j = blockIdx.x * BD + tid; j < B; j += sh.builders * BD) {
      const uint32_t at = upd_pos[(size_t)t * B + j];
      const float v = upd_prio[(size_t)t * B + j];
      if (!(at < B)) f_idx = 1u;
      else if (!valid_priority(v)) f_prio = 2u;
      else {
        acc |= atomicMax(&inv[at], j + 1u);   // (returning: its arrival says that it has been performed)
        const uint32_t vb = v > 0.0f ? __float_as_uint(v) : 0u;
        mx = vb > mx ? vb : mx;
      }
    }
    // nothing can be sampled (and no element is valid) exactly when no node of height ho is positive
    int positive = 0;
    for (uint32_t i = tid; i < sh.top_n[0]; i += BD) positive |= cur_ho[i] > 0.0f ? 1 : 0;
    positive = __syncthreads_or(positive);
    if (positive) {
      raise_max(g, t, mx, max_seen);
      if (f_idx | f_prio) atomicOr(&g.status[t], f_idx | f_prio);
    } else if (B) {
      if (tid == 0) atomicOr(&g.status[t], 1u);
    }
    asm volatile("" ::"v"(acc));
    __syncthreads();   // every lane's atomics have returned
    if (tid == 0) atomicAdd(ctl + 1, 1u);
    return;
  }

  // ------------------------------------------------------------------ owner workgroup b
  const uint32_t b = blockIdx.x - sh.builders;
  float* top = lds;                                   // heights ho .. H-1, at top_off[i]
  float* sub = lds;                                   // heights 1 .. ho-1 of the own subtree, at sub_off[i]
  ChunkLds c;
  c.rows = lds + sh.rows_off;
  c.key = reinterpret_cast<uint32_t*>(lds + sh.key_off);
  c.wpos = c.key + (BD + 2);
  c.wval = reinterpret_cast<float*>(c.wpos + (BD + 1));
  c.touch = reinterpret_cast<uint32_t*>(c.wval + (BD + 1));

  PER_TRACE_DECL;
  PER_MARK(0);
  // ---- trip 1: height ho of the whole tree, the own subtree's heights, control words
  uint32_t vbuf = 0;
  if (out_w) vbuf = read_word_with_the_loads(g.vnext + t);
  const uint32_t max_seen = read_max_bits(g, t);
  for (uint32_t i = tid; i < sh.top_cnt[0]; i += BD) top[sh.top_off[0] + i] = i < sh.top_n[0] ? cur_ho[i] : 0.0f;
#pragma unroll
  for (int i = 0; i < kStepSub; ++i) {
    if (i < n_sub) {
      const uint32_t first = b * sh.sub_cnt[i];       // first node of height 1 + i under b
      const float* src = sh.sub_ptr[i] + (size_t)t * sh.sub_stride[i];
      for (uint32_t e = tid; e < sh.sub_cnt[i]; e += BD)
        sub[sh.sub_off[i] + e] = first + e < sh.sub_pad[i] ? src[first + e] : 0.0f;
    }
  }
  __syncthreads();
  // the heights above ho, from LDS (in memory they may be stale)
  PER_MARK(1);
  {
    const unsigned q = tid % LPS;
    const uint32_t grp = tid / LPS, ngrp = BD / LPS;
#pragma unroll
    for (int i = 1; i < kStepTop; ++i) {
      if (i < n_top) {
        for (uint32_t base = 0; base < sh.top_cnt[i]; base += ngrp) {
          const uint32_t j = base + grp;
          const bool real = j < sh.top_n[i];
          const float sum = group_sum<LOGK>(top + sh.top_off[i - 1] + (size_t)(real ? j : 0u) * K, q);
          if (q == 0 && j < sh.top_cnt[i]) top[sh.top_off[i] + j] = real ? sum : 0.0f;
        }
        __syncthreads();
      }
    }
  }
  float total;
  {
    const float* rootgrp = top;   // group 0 of height H-1
#pragma unroll
    for (int i = 0; i < kStepTop; ++i)
      if (i == n_top - 1) rootgrp = top + sh.top_off[i];
    total = row_sum<LOGK>(rootgrp);
  }
  const bool leader = b == 0 && tid == 0;
  PER_MARK(2);

  // The end of every owner: the last one to finish makes the other array of height ho current (if the tree was
  // changed) and puts the counters back to zero for the next call.
  auto finish_owner = [&](bool changed) {
    if (leader && out_w) g.vcur[t] = not_before_here(vbuf) & 1u;
    __syncthreads();   // this workgroup's lanes have issued all their stores
    if (tid == 0) {
      const uint32_t old = atomicAdd(ctl + 2, 1u);
      if (old == sh.owners - 1u) {
        if (changed) ctl[0] = sel ^ 1u;
        ctl[1] = 0u;
        ctl[2] = 0u;
      }
    }
  };
  // Waits until every builder workgroup has recorded its elements.  The builders come first in the grid and wait
  // for nothing, so the wait ends; it is bounded all the same, and a workgroup that gives up says so.
  auto wait_for_builders = [&]() -> bool {
    if (!sh.builders) return true;
    if (tid == 0) {
      uint32_t spins = 0, ok = 1;
      while (__hip_atomic_load(ctl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < sh.builders) {
        if (++spins > kStepSpinLimit) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
      s_u32[0] = ok;
      if (!ok) atomicOr(&g.status[t], 8u);
    }
    __syncthreads();
    const bool ok = s_u32[0] != 0;
    __syncthreads();
    return ok;
  };

  if (!(total > 0.0f)) {   // nothing can be sampled from this tree; workgroup b reports a slice of the batch
    const bool waited = wait_for_builders();
    for (uint32_t s = b * BD + tid; s < B; s += sh.owners * BD) {
      const size_t o = (size_t)t * B + s;
      out_idx[o] = 0xFFFFFFFFu;
      if (out_prio) out_prio[o] = 0.0f;
      if (out_w) out_w[o] = 0.0f;
      if (sh.builders && waited) inv[s] = 0u;   // (the builders have recorded nothing: no element is valid)
    }
    // (without a map every element is out of range too; with one the builders have said so)
    if (leader) atomicOr(&g.status[t], sh.builders ? 4u : 5u);
    finish_owner(false);
    return;
  }
  const float seg = total / (float)B;

  // ---- where this workgroup's run of samples starts, to within a few: the mass in front of node b over seg
  if (wave == 0) {
    double p = 0.0;
    for (uint32_t e = lane; e < (uint32_t)n_top * K; e += 64) {
      const uint32_t i = e >> LOGK, j = e & (uint32_t)(K - 1);
      const uint32_t node = shr64(b, i * LOGK), sib = node & (uint32_t)(K - 1);
      uint32_t off_i = sh.top_off[0];
#pragma unroll
      for (int k = 1; k < kStepTop; ++k)
        if ((uint32_t)k == i) off_i = sh.top_off[k];
      if (j < sib) p += (double)top[off_i + (node - sib) + j];
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) p += __shfl_xor(p, m);
    if (lane == 0) s_est = p / (double)seg;
  }
  __syncthreads();
  const double est = s_est;
  PER_MARK(3);
  const uint32_t s_guess = est >= (double)B ? B : (est > 0.0 ? (uint32_t)est : 0u);   // (not a number: 0)
  uint32_t s0 = s_guess > kStepPad ? s_guess - kStepPad : 0u;

  // walks a target down the heights H-1 .. ho in LDS; returns the node of height ho it lands in
  auto walk_top = [&](float& r, float& val) -> uint32_t {
    uint32_t node = 0;
#pragma unroll
    for (int i = kStepTop - 1; i >= 0; --i) {
      if (i < n_top) {
        unsigned child;
        descend_lane<LOGK>(top + sh.top_off[i] + (size_t)node * K, r, child, val);
        node = node * K + child;
      }
    }
    return node;
  };
  auto uniform_of = [&](uint32_t s) -> float { return rng.on ? counter_uniform(rng, s, t) : u[(size_t)t * B + s]; };
  // the node of height ho that sample s lands in (samples beyond the batch: beyond every node)
  auto landing = [&](uint32_t s) -> uint32_t {
    if (!(s < B)) return 0xFFFFFFFFu;
    float r = ((float)s + uniform_of(s)) * seg, val = total;
    return walk_top(r, val);
  };
  // smallest s in [0, B] whose sample lands in a node >= bound; by one wave, 64 probes per round
  auto first_at_or_after = [&](uint32_t bound) -> uint32_t {
    uint32_t lo = 0, hi = B;
    while (lo < hi) {
      const uint32_t span = hi - lo, stride = (span + 63u) / 64u;
      const uint64_t s64 = (uint64_t)lo + (uint64_t)lane * stride;
      const bool probe = s64 < hi;
      const bool ge = !probe || landing((uint32_t)s64) >= bound;
      const unsigned long long m = __ballot(ge);
      if (m == 0ull) {
        lo = lo + 63u * stride + 1u;
      } else {
        const uint32_t f = (uint32_t)__ffsll((long long)m) - 1u;
        const uint64_t at = (uint64_t)lo + (uint64_t)f * stride;
        if (f > 0) lo = lo + (f - 1u) * stride + 1u;
        if (at < hi) hi = (uint32_t)at;
      }
    }
    return lo;
  };

  // ---- trip 2: the samples of the window [s0, s0 + BD): uniforms, their own new priorities
  uint32_t s = s0 + tid;
  bool in = s < B;
  float u_s = in ? uniform_of(s) : 0.0f;
  float prio_s = in ? upd_prio[(size_t)t * B + s] : 0.0f;
  float r = ((float)s + u_s) * seg, val = total;
  uint32_t node_ho = in ? walk_top(r, val) : 0xFFFFFFFFu;
  // does the window hold the whole run?  its first sample must land in front of b (or be sample 0), and a sample
  // of it must land behind b (or the batch must end in it)
  {
    const int starts = tid == 0 && (s0 == 0 || node_ho < b) ? 1 : 0;
    const int ends = (in && node_ho > b) || (tid == 0 && s0 + BD >= B) ? 1 : 0;
    if (tid == 0) s_u32[1] = 0;
    const int both = __syncthreads_or(starts) + 2 * __syncthreads_or(ends);
    if (both != 3) {
      // rare: the exact ends of the run by search, then chunks of it
      if (wave == 0) {
        const uint32_t lo = first_at_or_after(b), hi = first_at_or_after(b + 1u);
        if (lane == 0) {
          s_u32[1] = 1;
          s_u32[2] = lo;
          s_u32[3] = hi;
        }
      }
    }
    __syncthreads();
  }
  PER_MARK(4);
  const bool searched = s_u32[1] != 0;
  const uint32_t run_lo = searched ? s_u32[2] : s0, run_hi = searched ? s_u32[3] : 0u;
  const uint32_t n_chunks = searched ? (run_hi - run_lo + BD - 1u) / BD : 1u;
  const bool two_phase = n_chunks > 1;
  __syncthreads();

  const uint32_t lo1 = b * sh.sub_cnt[0];                                   // first height-1 node of the subtree
  float* leaves = g.level[0] + (size_t)t * g.stride[0];
  float* lvl1 = sh.sub_ptr[0] + (size_t)t * sh.sub_stride[0];
  float* stage = c.rows + (size_t)(1u + wave * 64u) * ROW;                  // this wave's rows: slots 1 + tid
  uint32_t mx = 0, flags = 0, vmin_bits = 0x7F800000u;
  bool builders_ok = true, waited = false;
  if (tid == 0) {
    c.key[0] = kNoKey;
    c.wpos[0] = 0;
    c.touch[0] = 0;
  }
  if (tid < 2) c.key[BD + tid] = kNoKey;   // (key[BD] is written again by the last lane; key[BD + 1] stays)

  for (uint32_t pass = 0; pass < (two_phase ? 2u : 1u); ++pass) {
    // pass 0 walks (and, when one chunk holds the run, updates); pass 1 of a long run updates chunk by chunk
    for (uint32_t ch = 0; ch < n_chunks; ++ch) {
      bool member;
      uint32_t idx = kNoKey;
      if (searched) {
        s = run_lo + ch * BD + tid;
        member = s < run_hi;
        if (pass == 0 || !two_phase) {
          u_s = member ? uniform_of(s) : 0.0f;
          r = ((float)s + u_s) * seg;
          val = total;
          (void)walk_top(r, val);
        }
        prio_s = member ? upd_prio[(size_t)t * B + s] : 0.0f;
      } else {
        member = in && node_ho == b;
      }
      const size_t o = (size_t)t * B + (member ? s : 0u);
      uint32_t x = b;   // node of height ho
      if (pass == 0) {
        // ---- the own subtree's heights from LDS
        if (!member) r = 0.0f;
#pragma unroll
        for (int i = kStepSub - 1; i >= 0; --i) {
          if (i < n_sub) {
            const uint32_t local = x - b * (sh.sub_cnt[i] >> LOGK);   // x - first node of height 2 + i under b
            unsigned child;
            descend_lane<LOGK>(sub + sh.sub_off[i] + (size_t)local * K, r, child, val);
            x = x * K + child;
          }
        }
      } else {
        idx = member ? out_idx[o] : kNoKey;
        x = member ? idx >> LOGK : lo1;
      }
      // ---- trip 3: the leaf groups, staged row by row
      __syncthreads();   // (the rows of the chunk before are no longer read)
      stage_groups<LOGK, 0>(leaves, x, lane, stage);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if (pass == 0) {
        unsigned child;
        descend_lane<LOGK>(stage + lane * ROW, r, child, val);
        idx = x * K + child;
        if (member) {
          out_idx[o] = idx;
          if (out_prio) out_prio[o] = val;
          if (out_w) out_w[o] = val;
          const uint32_t vb = __float_as_uint(val);
          vmin_bits = vb < vmin_bits ? vb : vmin_bits;
        }
        if (two_phase) continue;
      }
      PER_MARK(5);
      // ---- the update of this chunk
      if (!waited) {
        builders_ok = wait_for_builders();
        waited = true;
      }
      uint32_t w = 0;
      float wv = 0.0f;
      if (member) {
        if (!(idx < size)) {
          flags |= 1u;
          if (sh.builders && builders_ok) (void)atomicExch(&inv[s], 0u);
        } else if (sh.builders) {
          if (builders_ok) {
            w = atomicExch(&inv[s], 0u);
            if (w) wv = w == s + 1u ? prio_s : upd_prio[(size_t)t * B + (w - 1u)];
          }
        } else if (valid_priority(prio_s)) {
          w = s + 1u;
          wv = prio_s;
          const uint32_t vb = wv > 0.0f ? __float_as_uint(wv) : 0u;
          mx = vb > mx ? vb : mx;
        } else {
          flags |= 2u;
        }
      }
      c.key[1 + tid] = member ? idx : kNoKey;
      c.wpos[1 + tid] = w;
      c.wval[1 + tid] = wv;
      c.touch[1 + tid] = 0u;
      PER_MARK(6);
      const bool last_chunk = ch + 1 == n_chunks;
      __syncthreads();
      uint32_t open_pos = 0;
      float open_val = 0.0f;
      chunk_leaves<LOGK>(c, tid, BD, last_chunk, leaves, open_pos, open_val);
      if (tid == 0) chunk_leaves<LOGK>(c, BD, BD, last_chunk, leaves, open_pos, open_val);
      __syncthreads();
      uint32_t open_head = chunk_groups<LOGK>(c, tid, BD, last_chunk, lvl1, sub + sh.sub_off[0], lo1);
      if (tid == 0) open_head = chunk_groups<LOGK>(c, BD, BD, last_chunk, lvl1, sub + sh.sub_off[0], lo1);
      __syncthreads();
      PER_MARK(7);
      if (!last_chunk) {   // what stays open moves to slot 0 (thread 0 has worked on slot BD)
        if (tid == 0) {
          s_u32[4] = open_head;
          s_u32[5] = c.key[BD];
          s_u32[6] = open_pos;
          s_u32[7] = __float_as_uint(open_val);
        }
        __syncthreads();
        const uint32_t h = s_u32[4];
        float carry = 0.0f;
        if (h != kNoKey && tid < (uint32_t)K) carry = c.rows[(size_t)h * ROW + tid];
        const uint32_t touched = h != kNoKey ? c.touch[h] : 0u;
        __syncthreads();
        if (h != kNoKey && tid < (uint32_t)K) c.rows[tid] = carry;
        if (tid == 0) {
          c.key[0] = h != kNoKey ? s_u32[5] : kNoKey;
          c.wpos[0] = s_u32[6];
          c.wval[0] = __uint_as_float(s_u32[7]);
          c.touch[0] = touched;
        }
      }
    }
    if (pass == 0 && two_phase) __syncthreads();   // the indices written above are read back by the second pass
  }

  // ---- the heights 2 .. ho-1 of the subtree and node b itself, from LDS; what changed is stored
  __syncthreads();
  {
    const unsigned q = tid % LPS;
    const uint32_t grp = tid / LPS, ngrp = BD / LPS;
#pragma unroll
    for (int i = 1; i < kStepSub; ++i) {
      if (i < n_sub) {
        const uint32_t first = b * sh.sub_cnt[i];
        float* dst = sh.sub_ptr[i] + (size_t)t * sh.sub_stride[i];
        for (uint32_t base = 0; base < sh.sub_cnt[i]; base += ngrp) {
          const uint32_t e = base + grp;
          const bool ok = e < sh.sub_cnt[i];
          const float sum = group_sum<LOGK>(sub + sh.sub_off[i - 1] + (size_t)(ok ? e : 0u) * K, q);
          if (ok && q == 0) {
            float* mine = sub + sh.sub_off[i] + e;
            if (__float_as_uint(*mine) != __float_as_uint(sum)) {
              *mine = sum;
              dst[first + e] = sum;
            }
          }
        }
        __syncthreads();
      }
    }
    // node b: the sum of its K children, the nodes of height ho-1 of the subtree
    uint32_t off_last = sh.sub_off[0];
#pragma unroll
    for (int i = 1; i < kStepSub; ++i)
      if (i == n_sub - 1) off_last = sh.sub_off[i];
    if (tid < 64) {
      const float sum = group_sum<LOGK>(sub + off_last, lane % LPS);
      if (lane == 0) new_ho[b] = sum;
    }
  }
  PER_MARK(8);
  // ---- what is left: batch minimum for the weights, running maximum, flags
  if (out_w) {
    const uint32_t m = wave_min_u32(vmin_bits);
    if (lane == 0 && m != 0x7F800000u)
      atomicMin(&g.vmin[((size_t)(not_before_here(vbuf) & 1u) * g.T + t) * kVminSlots + ((b * (BD >> 6) + wave) % kVminSlots)], m);
  }
  if (!sh.builders) raise_max(g, t, mx, max_seen);
  if (flags) atomicOr(&g.status[t], flags);
  PER_MARK(9);
  PER_FLUSH();
  finish_owner(true);
}

// The side array's values become the level array's (for kernels that read height ho from the level array).
__global__ void k_step_settle(StepShape sh) {
  const uint32_t t = blockIdx.x;
  uint32_t* ctl = sh.ctl + (size_t)t * 4;
  if (!(ctl[0] & 1u)) return;   // (uniform over the workgroup)
  const float* side = sh.side + (size_t)t * sh.side_stride;
  float* lvl = sh.top_ptr[0] + (size_t)t * sh.top_stride[0];
  for (uint32_t i = threadIdx.x; i < sh.top_n[0]; i += blockDim.x) lvl[i] = side[i];
  __syncthreads();
  if (threadIdx.x == 0) ctl[0] = 0u;
}

// The owner height of a tree for k_step, or 0 when the kernel does not fit it: the lowest height, not below the
// tree pass's own workgroup roots, with at most 2048 nodes over all trees, whose subtrees (heights 1 .. ho-1)
// and the heights from it to the root are small enough for LDS.
uint32_t step_owner_height(const Geom& g) {
  if (g.logK < 3) return 0;
  for (uint32_t ho = tree_pass_height(g) < 2 ? 2 : tree_pass_height(g); ho + 1 <= g.H; ++ho) {
    if ((uint64_t)g.n[ho] * g.T > 2048 || g.n[ho] > kLazyTopNodes) continue;
    if (g.H - ho > (uint32_t)kStepTop || ho - 1 > (uint32_t)kStepSub) return 0;
    uint64_t sub = 0;
    for (uint32_t l = 1; l < ho; ++l) sub += 1ull << ((ho - l) * g.logK);
    if (sub > 16384) return 0;
    return ho;
  }
  return 0;
}

// Workgroup size for a batch of B samples per tree: room for one and a half times the average run of samples
// per owner, within what the staging rows leave of the LDS; 0 when the runs would be too long for one chunk
// (the separate kernels are the better choice then).
template <int LOGK>
static uint32_t step_block(const Geom& g, uint32_t ho, uint32_t B) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t most = K >= 32 ? 256u : 512u;
  const uint64_t avg = ((uint64_t)B + g.n[ho] - 1) / g.n[ho];
  const uint64_t want = avg + avg / 2 + 2 * kStepPad + 8;
  if (want > most) return 0;
  const uint32_t block = (uint32_t)((want + 63) / 64 * 64);
  return block < 64 ? 64 : block;
}

template <int LOGK>
static hipError_t launch_step_k(const Geom& g, const Tuning& tn, uint32_t block, uint32_t B, uint32_t size, const float* u,
                                const RngArgs& rng, uint32_t* out_idx, float* out_prio, float* out_w,
                                const float* upd_prio, const uint32_t* upd_pos, hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t ho = g.step_ho;
  StepShape sh{};
  sh.n_top = g.H - ho;
  sh.n_sub = ho - 1;
  uint32_t off = 0;
  for (uint32_t i = 0; i < sh.n_top; ++i) {
    const uint32_t l = ho + i;
    sh.top_ptr[i] = g.level[l];
    sh.top_stride[i] = g.stride[l];
    sh.top_cnt[i] = g.n[l + 1] * K;
    sh.top_n[i] = g.n[l];
    sh.top_off[i] = off;
    off += sh.top_cnt[i];
  }
  for (uint32_t i = 0; i < sh.n_sub; ++i) {
    const uint32_t l = 1 + i;
    sh.sub_ptr[i] = g.level[l];
    sh.sub_stride[i] = g.stride[l];
    sh.sub_cnt[i] = 1u << ((ho - l) * LOGK);
    sh.sub_pad[i] = (uint32_t)(((uint64_t)g.n[l] + K - 1) / K * K);
    sh.sub_off[i] = off;
    off += sh.sub_cnt[i];
  }
  off = (off + 3u) / 4u * 4u;
  sh.rows_off = off;
  off += (block + 1u) * (K + 4);
  sh.key_off = off;
  off += (block + 2u) + 3u * (block + 1u);
  sh.owners = g.n[ho];
  sh.builders = 0;
  if (upd_pos) {
    sh.builders = (B + 4u * block - 1u) / (4u * block);   // about four elements per builder lane
    if (sh.builders > 64) sh.builders = 64;
  }
  sh.side = g.step_side;
  sh.side_stride = g.step_side_stride;
  sh.ctl = g.step_ctl;
  sh.inv = reinterpret_cast<uint32_t*>(g.owner);
  sh.inv_stride = 2u * g.owner_stride;
  const size_t bytes = (size_t)off * 4;
  hipError_t e = grant_lds<&k_step<LOGK>>(tn, bytes);
  if (e != hipSuccess) return e;
  PER_LAUNCH(KID_STEP, k_step<LOGK>, dim3(sh.builders + sh.owners, g.T), dim3(block), bytes, s, g, sh, B, size, u, rng,
             out_idx, out_prio, out_w, upd_prio, upd_pos);
  return hipGetLastError();
}

// Block size k_step would run a batch of B with, 0 when it does not take that batch (or that tree).
uint32_t step_fits(const Geom& g, uint32_t B) {
  if (!g.step_ho || B == 0 || (uint64_t)B > 2ull * g.owner_stride) return 0;
  switch (g.logK) {
    case 3: return step_block<3>(g, g.step_ho, B);
    case 4: return step_block<4>(g, g.step_ho, B);
    case 5: return step_block<5>(g, g.step_ho, B);
    case 6: return step_block<6>(g, g.step_ho, B);
    default: return 0;
  }
}

// Sampling and the update of the sampled batch in one kernel, then the rows and the weights in a second.
hipError_t launch_step(const Geom& g, const Tuning& tn, uint32_t block, uint32_t B, uint32_t size, float beta,
                       const float* u, const RngArgs& rng, uint32_t* out_idx, float* out_w, float* out_prio,
                       uint32_t weight_mode, const FieldTable* rows, const float* upd_prio, const uint32_t* upd_pos,
                       hipStream_t s) {
  hipError_t e;
  switch (g.logK) {
    case 3: e = launch_step_k<3>(g, tn, block, B, size, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, s); break;
    case 4: e = launch_step_k<4>(g, tn, block, B, size, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, s); break;
    case 5: e = launch_step_k<5>(g, tn, block, B, size, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, s); break;
    case 6: e = launch_step_k<6>(g, tn, block, B, size, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, s); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess || (!rows && !out_w)) return e;
  FinishArgs a{};
  a.B = B;
  a.idx = out_idx;
  a.w = out_w;
  a.size = size;
  a.beta = beta;
  a.weight_mode = weight_mode;
  return launch_finish(g, tn, rows, a, s);
}

// Makes the level array of the owner height current again after k_step calls (see k_step_settle).
hipError_t launch_step_settle(const Geom& g, const Tuning& tn, hipStream_t s) {
  if (!g.step_ho) return hipSuccess;
  StepShape sh{};
  sh.top_ptr[0] = g.level[g.step_ho];
  sh.top_stride[0] = g.stride[g.step_ho];
  sh.top_n[0] = g.n[g.step_ho];
  sh.side = g.step_side;
  sh.side_stride = g.step_side_stride;
  sh.ctl = g.step_ctl;
  PER_LAUNCH(KID_STEP_SETTLE, k_step_settle, dim3(g.T), dim3(256), 0, s, sh);
  return hipGetLastError();
}
