// Second half of a priority update: the tree pass (alone, or beside the row gather and the weights).
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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
  uint32_t list_cap;              // height-1 nodes under one workgroup root: entries of the workgroup's node list
  uint32_t hb;
  uint32_t group_batch;           // size of the batch if it claimed through the group entries, else 0
};

// Tree pass.  Workgroup b of tree t owns the subtree under node b of height hb and keeps the
// subtree's nodes of heights 1 .. hb in LDS.
//  0. In one trip it fetches its height-1 nodes, the dirty bits of the leaves below them and the
//     entries of their claim groups.
//  1. Each height-1 node with a claimed leaf (a dirty bit, or the leaf of a group entry written by
//     this batch) is rebuilt by LPS lanes: they read its K leaves and, for the dirty ones only,
//     the stamp entry, whose lower word is the value of the batch element that won that leaf; it
//     replaces the leaf (and is stored), and so does the value of the group entry, which wins
//     against a dirty bit of the same leaf (it is the latest element of its group); the K values
//     are summed pairwise.  Dirty bits and used leaf stamps are cleared at the end.
//  2. Heights 2 .. hb of the subtree are recomputed from LDS and stored.
//  3. Above hb every node counts the arrivals of its children's workgroups; the last one to
//     arrive recomputes it and carries on upwards, so the root is written by whichever
//     workgroup finishes last.  No workgroup ever waits for another.  When there are only a
//     few nodes at height hb this step is skipped (chain == 0): the agent-scope fences it
//     needs cost more than recomputing those heights in the next kernel that reads them.
constexpr uint32_t kDirtyListCap = 2048;
// Largest hb that tree_pass_height can give a fanout: the whole tree when it has at most kDirtyListCap
// height-1 nodes (H <= 1 + ceil(log_K 2048)), else the lowest height whose subtrees hold 64 of them.
template <int LOGK>
constexpr int kMaxPassHeight = LOGK == 1 ? 13 : LOGK == 2 ? 7 : LOGK == 3 ? 5 : LOGK <= 5 ? 4 : 3;

// The work of workgroup b of tree t (b = its subtree's root at height hb).  TRACK_MIN: also renew min1
// (smallest positive leaf) of every rebuilt height-1 node; a compile-time choice, because even as a
// never-taken branch that code cost the pass half a microsecond.
template <int LOGK, bool TRACK_MIN>
__device__ __forceinline__ void tree_job(const Geom& g, const SubLevels& sl, uint32_t t, uint32_t b, uint32_t chain) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  // dynamic LDS: the subtree's nodes, then the list of claimed height-1 nodes (see tree_lds_bytes)
  extern __shared__ __attribute__((aligned(16))) float sub[];   // 16-byte LDS accesses need the alignment
  uint2* s_entry = reinterpret_cast<uint2*>(sub + (sl.lds_floats + 3u) / 4u * 4u);
  uint32_t* s_list = reinterpret_cast<uint32_t*>(s_entry + sl.list_cap);
  uint32_t* s_bits = s_list + sl.list_cap;
  [[maybe_unused]] uint32_t* s_bits_hi = s_bits + sl.list_cap;   // K = 64 only
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
  uint2* owner = reinterpret_cast<uint2*>(g.owner) + (size_t)t * g.owner_stride;   // (value, stamp)
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
  // the claim group entry of a height-1 node if this batch wrote it for a leaf of that node:
  // (value bits, 0x80000000 | leaf within the node), else y = 0
  uint2* groups = g.nclaim + (size_t)t * g.nclaim_stride;
  // first stamp of this batch, left by its claim phase (a batch that claimed leaf by leaf has no entries)
  const uint32_t floor = sl.group_batch ? read_word_with_the_loads(g.sfloor + t) : 0xFFFFFFFFu;
  // (fetched here, decoded there: the comparison would make the wave wait for the entry, and the floor, before it
  // issues the loads that follow)
  auto fetch_entry = [&](uint32_t node) -> uint2 { return groups[LOGK >= 5 ? node : (node << LOGK) >> 5]; };
  auto decode_entry = [&](uint2 e, uint32_t node) -> uint2 {
    bool mine = (e.y >> 6) >= floor;
    if constexpr (LOGK < 5) mine = mine && ((e.y & 31u) >> LOGK) == (node & ((32u >> LOGK) - 1u));
    e.y = mine ? 0x80000000u | (e.y & (uint32_t)(K - 1)) : 0u;
    return e;
  };
  // one node per thread and sweep; the first sweep's bits are fetched together with the height-1 nodes
  const uint32_t f_first = lo1 + threadIdx.x;
  unsigned long long bits_first = 0;
  uint2 entry_first = make_uint2(0, 0);
  if (f_first < hi1) {
    bits_first = node_bits(f_first);
    entry_first = fetch_entry(f_first);
  }
  {
    // slot 0 from memory, the rest zero.  The first four sweeps' loads are issued together (a sweep that
    // waits for its load before the next one starts costs a trip to memory each).
    auto from_memory = [&](uint32_t i) { return (i < sl.lds_off[1] || hb == 1) && lo1 + i < n1_pad; };
    const uint32_t i0 = threadIdx.x, i1 = threadIdx.x + blockDim.x, i2 = i1 + blockDim.x, i3 = i2 + blockDim.x;
    float v0 = 0.0f, v1 = 0.0f, v2 = 0.0f, v3 = 0.0f;
    if (i0 < sl.lds_floats && from_memory(i0)) v0 = lvl1[lo1 + i0];
    if (i1 < sl.lds_floats && from_memory(i1)) v1 = lvl1[lo1 + i1];
    if (i2 < sl.lds_floats && from_memory(i2)) v2 = lvl1[lo1 + i2];
    if (i3 < sl.lds_floats && from_memory(i3)) v3 = lvl1[lo1 + i3];
    if (i0 < sl.lds_floats) sub[i0] = v0;
    if (i1 < sl.lds_floats) sub[i1] = v1;
    if (i2 < sl.lds_floats) sub[i2] = v2;
    if (i3 < sl.lds_floats) sub[i3] = v3;
    for (uint32_t i = threadIdx.x + 4 * blockDim.x; i < sl.lds_floats; i += blockDim.x)
      sub[i] = from_memory(i) ? lvl1[lo1 + i] : 0.0f;
  }
  // compact the claimed nodes into s_list / s_bits / s_entry: ballot within the wave, wave totals through LDS
  const uint32_t nwaves = blockDim.x >> 6;
  uint32_t nd = 0;
  for (uint32_t f0 = lo1; f0 < hi1; f0 += blockDim.x) {
    const uint32_t f = f0 + threadIdx.x;
    unsigned long long bits = 0;
    uint2 entry = make_uint2(0, 0);
    if (f0 == lo1) {
      bits = bits_first;
      entry = entry_first;
    } else if (f < hi1) {
      bits = node_bits(f);
      entry = fetch_entry(f);
    }
    entry = decode_entry(entry, f);
    if (!(f < hi1)) entry.y = 0;
    const bool listed = bits != 0 || entry.y != 0;
    const unsigned long long m = __ballot(listed);
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (lane == 0) s_wave[threadIdx.x >> 6] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = nd, total = nd;
    for (uint32_t wv = 0; wv < nwaves; ++wv) {
      const uint32_t c = s_wave[wv];
      if (wv < (threadIdx.x >> 6)) before += c;
      total += c;
    }
    if (listed) {
      s_list[before + rank] = f;
      s_bits[before + rank] = (uint32_t)bits;
      s_entry[before + rank] = entry;
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
      uint2 e;
      uint32_t mn;   // (TRACK_MIN only)
    };
    // A set bit means the leaf was claimed leaf by leaf in this batch: its stamp entry holds the winner's value.
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
      it.e = s_entry[li];
#pragma unroll
      for (int k = 0; k < (LOGK == 1 ? 2 : 4); ++k) {
        it.s[k] = make_uint2(0, 0);
        if (it.my & (1u << k)) it.s[k] = owner[it.at + k];
      }
      return it;
    };
    auto finish = [&](Item& it) {
      float sum;
      // the group entry's leaf, if it is one of this lane's
      const uint32_t el = it.e.y & 63u;
      const bool here = it.e.y != 0 && (LOGK == 1 || (el >> 2) == q);
      const uint32_t sel = here ? 1u << (el & (LOGK == 1 ? 1u : 3u)) : 0u;
      const float ev = __uint_as_float(it.e.x);
      if constexpr (LOGK == 1) {
        if (it.my & 1u) it.c.x = __uint_as_float(it.s[0].x);
        if (it.my & 2u) it.c.y = __uint_as_float(it.s[1].x);
        if (sel & 1u) it.c.x = ev;
        if (sel & 2u) it.c.y = ev;
        it.my |= sel;
        sum = it.c.x + it.c.y;
        if constexpr (TRACK_MIN) it.mn = min_u32(positive_bits(it.c.x), positive_bits(it.c.y));
      } else {
        if (it.my & 1u) it.c.x = __uint_as_float(it.s[0].x);
        if (it.my & 2u) it.c.y = __uint_as_float(it.s[1].x);
        if (it.my & 4u) it.c.z = __uint_as_float(it.s[2].x);
        if (it.my & 8u) it.c.w = __uint_as_float(it.s[3].x);
        if (sel & 1u) it.c.x = ev;
        if (sel & 2u) it.c.y = ev;
        if (sel & 4u) it.c.z = ev;
        if (sel & 8u) it.c.w = ev;
        it.my |= sel;
        sum = butterfly_sum<Fan<LOGK>::LOGLPS>((it.c.x + it.c.y) + (it.c.z + it.c.w));
        if constexpr (TRACK_MIN) {
          uint32_t m = min_u32(min_u32(positive_bits(it.c.x), positive_bits(it.c.y)),
                               min_u32(positive_bits(it.c.z), positive_bits(it.c.w)));
          it.mn = butterfly_min<Fan<LOGK>::LOGLPS>(m);
        }
      }
      return sum;
    };
    auto store = [&](const Item& it, float sum) {
      if (it.ok && it.my) *reinterpret_cast<LeafVec*>(leaves + it.at) = it.c;
      if (it.ok && q == 0) {
        // (nontemporal: the scattered 4-byte stores then leave for memory while the pass goes on, instead
        // of all being written back when the kernel ends; measured - 0.15 us per step.  The same for the
        // upper heights, which the next kernel reads first, cost + 1.2 us.)
        __builtin_nontemporal_store(sum, lvl1 + it.node);
        sub[it.node - lo1] = sum;
        if constexpr (TRACK_MIN) g.min1[(size_t)t * g.min1_stride + it.node] = it.mn;
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
    // (unrolled over the slots, so that the per-height facts come out of the kernel arguments at fixed
    // offsets; read through a table in LDS instead, they cost the pass 0.3 us)
    // K = 2: the last six heights (at most 64 nodes below them) are a wave's reduction tree: lane i holds node i,
    // and every step of the butterfly is one more height (left + right; the partner lane adds right + left, the
    // same bits), so those heights cost a lane exchange each instead of a pass over LDS with a barrier.
    [[maybe_unused]] const uint32_t j_wave = LOGK == 1 ? (hb > 7 ? hb - 6 : 1u) : hb;   // first slot the wave computes
#pragma unroll
    for (int j = 1; j < kMaxPassHeight<LOGK>; ++j) {
      if ((uint32_t)j < hb && (LOGK != 1 || (uint32_t)j < j_wave)) {
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
    if constexpr (LOGK == 1) {
      if (hb > 1) {
        __syncthreads();
        if (threadIdx.x < 64u) {
          const uint32_t children = 1u << (hb - j_wave);   // nodes of slot j_wave - 1 under b (zeros beyond the real ones)
          float v = lane < children ? sub[sl.lds_off[j_wave - 1] + lane] : 0.0f;
          for (uint32_t k = 1; j_wave - 1 + k < hb; ++k) {
            v = v + __shfl_xor(v, 1 << (k - 1));
            const uint32_t js = j_wave - 1 + k;             // the slot (height js + 1) this step has made
            const uint32_t sh = hb - 1 - js;
            const uint32_t a = b << sh;
            const uint32_t cnt = min(sl.n[js], (b + 1) << sh) - a;
            const uint32_t e = lane >> k;
            if ((lane & ((1u << k) - 1u)) == 0 && e < cnt) (sl.ptr[js] + (size_t)t * sl.stride[js])[a + e] = v;
          }
        }
      }
    }
  }

  PER_MARK(3);
  PER_FLUSH();
  // The dirty bits and the stamps of the dirty leaves are cleared again (both arrays are all zero between
  // batches).  Only now: a wait for loaded data also waits for every earlier store of the wave, so
  // stores that nothing depends on go last.
  for (uint32_t i = threadIdx.x; i < nd; i += blockDim.x) {
    const uint32_t node = s_list[i];
    unsigned long long bits = s_bits[i];
    if constexpr (LOGK == 6) bits |= (unsigned long long)s_bits_hi[i] << 32;
    if (bits) {
      if constexpr (LOGK == 6) {
        dirty[2 * (size_t)node] = 0;
        dirty[2 * (size_t)node + 1] = 0;
      } else {
        dirty[(node << LOGK) >> 5] = 0;   // for K < 32 the word is shared with neighbours of the same subtree
      }
      while (bits) {   // (few leaves: those that met another leaf of their group, or a batch claiming leaf by leaf)
        owner[(size_t)node * K + (uint32_t)(__ffsll((long long)bits) - 1)] = make_uint2(0, 0);
        bits &= bits - 1;
      }
    }
  }
  // The stamp counter of the group entries: the next batch starts after this one; when that is beyond the
  // turning point, every workgroup clears the entries of its subtree instead and the counter starts over.
  if (sl.group_batch) {
    const bool turn = floor + sl.group_batch > kGroupStampTurn;   // (uniform over the launch)
    if (turn) {
      const uint32_t e_lo = LOGK >= 5 ? lo1 : (lo1 << LOGK) >> 5;
      const uint32_t e_hi = LOGK >= 5 ? hi1 : (uint32_t)((((unsigned long long)hi1 << LOGK) + 31u) >> 5);
      for (uint32_t e = e_lo + threadIdx.x; e < e_hi; e += blockDim.x) groups[e] = make_uint2(0, 0);
    }
    if (b == 0 && threadIdx.x == 0) g.sbase[t] = turn ? 1u : floor + sl.group_batch;
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

// What a sampling kernel that carried an insertion has left in max_pend (read by the caller when its workgroup
// started) goes into the running maximum; one workgroup per tree does this, after its share of the tree pass.
__device__ __forceinline__ void fold_pending_max(const Geom& g, uint32_t t, uint32_t pend_word) {
  const uint32_t pend = not_before_here(pend_word);
  if (threadIdx.x == 0 && pend) {
    atomicMax(reinterpret_cast<uint32_t*>(&g.max_v[t]), pend);
    g.max_pend[t] = 0u;
  }
}

// Workgroups of at most 512 lanes: two 1024-lane workgroups share a compute unit only while a wave
// stays within an eighth of the SIMD's scalar and vector registers (with one scalar register more the
// second workgroup waits for the first to end and the kernel takes half as long again), and holding
// the compiler to that budget made it spill; 512 lanes run the pass just as fast.
template <int LOGK, bool TRACK_MIN>
__global__ void __launch_bounds__(512)
k_update_tree(Geom g, SubLevels sl, uint32_t chain) {
  const uint32_t pend = (chain & 2u) && blockIdx.x == 0 ? read_word_with_the_loads(&g.max_pend[blockIdx.y]) : 0u;
  tree_job<LOGK, TRACK_MIN>(g, sl, blockIdx.y, blockIdx.x, chain & 1u);
  if ((chain & 2u) && blockIdx.x == 0) fold_pending_max(g, blockIdx.y, pend);
}

// Second kernel of a fused step whose claim phase rode in the sampling kernel: the tree pass
// (workgroups 0 .. tree_blocks-1) and, beside it, what is left of the sampling call: the
// importance weights and the rows of the sampled indices (JobRanges, offset by tree_blocks).  The
// tree pass is a chain of dependent memory trips and the row traffic fills the gaps; launched with
// workgroups of at most 512 lanes so that the two kinds share the compute units.  Held to 96 scalar
// registers (it needs no scratch memory for that; the row jobs' argument tables would take a few more),
// which the many small trees of a multi-tree buffer gain from (one big tree neither gains nor loses).
// Three such workgroups are resident per compute unit where the machine reserves 16 more scalar
// registers per wave; a cap of 80 makes it four, measured slower: the jobs then slow each other down
// in the memory system by more than the earlier start of the row jobs gives back.
template <int LOGK, bool TRACK_MIN, bool WIDE>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_num_sgpr(96)))
k_tree_finish(Geom g, SubLevels sl, uint32_t chain, uint32_t tree_blocks, FieldTable ft, JobRanges jr, FinishArgs a) {
  // (the lines of the arguments asked for in one batch, through one scalar register: this kernel has none to spare;
  // by the first four waves only: with every wave of a 512-lane workgroup at it, the step of 65 536 samples on 2^24
  // leaves loses 0.3 us where the small workloads gain as much)
  if (threadIdx.x < 256u)
    touch_kernel_arguments_through_one_register<kernarg_lines<Geom, SubLevels, uint32_t, uint32_t, FieldTable, JobRanges, FinishArgs>() < kTouchLines
                                                    ? kernarg_lines<Geom, SubLevels, uint32_t, uint32_t, FieldTable, JobRanges, FinishArgs>() : kTouchLines>();
  const uint32_t t = blockIdx.y;
  if (blockIdx.x < tree_blocks) {
    const uint32_t pend = (chain & 2u) && blockIdx.x == 0 ? read_word_with_the_loads(&g.max_pend[t]) : 0u;
    tree_job<LOGK, TRACK_MIN>(g, sl, t, blockIdx.x, chain & 1u);
    if ((chain & 2u) && blockIdx.x == 0) fold_pending_max(g, t, pend);
    return;
  }
  const uint32_t b = blockIdx.x - tree_blocks;
  PER_TRACE_DECL;
  PER_MARK(0);
  PER_MARK_HWID(15);
  if (b < jr.first[1]) {
    weights_job(g, t, a.B, a.size, a.beta, a.w, a.weight_mode, b, jr.first[1]);
    PER_MARK(3);
    PER_FLUSH();
    return;
  }
  const uint32_t f = job_field(jr, b);
  if (jr.whole_rows) {
    extern __shared__ __attribute__((aligned(16))) uint8_t stage[];
    move_whole_rows(ft, jr, t, a.B, a.idx, g.N, g.status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f], stage);
  } else if (f < (uint32_t)kMaxFields)
    rows_job<true, WIDE>(ft, f, t, a.B, a.idx, 0, g.N, g.status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
  PER_MARK(3);
  PER_FLUSH();
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

// Dynamic LDS of a tree-pass workgroup: its subtree's nodes (padded to 16 bytes), then per listed
// height-1 node the group entry (8 bytes), the node number and the dirty bits (4 bytes each; 8 for K = 64).
template <int LOGK>
static size_t tree_lds_bytes(const SubLevels& sl) {
  return ((size_t)(sl.lds_floats + 3u) / 4u * 4u + (size_t)sl.list_cap * (LOGK == 6 ? 5u : 4u)) * 4u;
}

// Sub-level descriptors and workgroup size of the tree pass for the update batch claimed with `c`.
template <int LOGK>
static hipError_t tree_pass_shape(const Geom& g, const Tuning& tn, const ClaimArgs& c, SubLevels* out,
                                  uint32_t* tblock_out) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t B = c.B;
  const uint32_t hb = tree_pass_height(g);
  if (hb > (uint32_t)kSubSlots || hb > (uint32_t)kMaxPassHeight<LOGK>)
    return hipErrorInvalidValue;   // cannot happen for fanouts and capacities accepted at create
  SubLevels sl{};
  sl.hb = hb;
  sl.group_batch = c.group_mode ? c.B : 0u;
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
  sl.list_cap = hb > 1 ? sl.lds_off[1] : 1u;
  // Unless told otherwise: enough lane groups to rebuild in one sweep twice the dirty height-1 nodes a
  // subtree gets on average (never more than it has), so that small batches do not launch idle waves.
  uint32_t tblock = tn.tree_block;
  if (tblock == 0) {
    const uint64_t per_subtree = hb > 1 ? sl.lds_off[1] : 1;
    uint64_t expect = 2 * ((uint64_t)B + g.n[hb] - 1) / g.n[hb];
    if ((uint64_t)g.n[hb] * g.T >= 2048) expect = (expect + 1) / 2;   // many small subtrees (many trees): more workgroups resident instead
    if (expect > per_subtree) expect = per_subtree;
    uint64_t want = expect * Fan<LOGK>::LPS;
    if (hb > 2) {   // the dense heights of the subtree want a lane group per height-2 node
      const uint64_t dense = (uint64_t)(sl.lds_off[2] - sl.lds_off[1]) * Fan<LOGK>::LPS;
      if (dense > want) want = dense;
    }
    tblock = (uint32_t)(want > 1024 ? 1024 : (want + 63) / 64 * 64);
    if (tblock < 64) tblock = 64;
    // A lane per height-1 node of the subtree when the launch stays small (at most eight waves per compute unit
    // of a 256-unit device): the list of claimed nodes is then made in one sweep, and every further sweep would
    // cost a trip to memory of its own (measured on one tree of 2^20 leaves at K = 16:
    // 14.1 -> 13.1 us per step of 32 samples, 14.1 -> 13.6 of 4096).
    const uint64_t one_sweep = per_subtree > 1024 ? 1024 : (per_subtree + 63) / 64 * 64;
    if (one_sweep > tblock && (uint64_t)g.n[hb] * g.T * (one_sweep / 64) <= 4096) tblock = (uint32_t)one_sweep;
    // ... and no more waves than that over the whole launch for a large batch either: workgroups that wait for a
    // second round cost more than the sweeps that smaller ones add (2^22 leaves at K = 16, 65 536 elements: 8.1 us
    // with 512 lanes, 5.6 with 256).
    const uint64_t groups = (uint64_t)g.n[hb] * g.T;
    const uint64_t room = groups >= 4096 ? 1 : 4096 / groups;   // waves per workgroup
    if (tblock > room * 64) tblock = (uint32_t)(room * 64);
  }
  *out = sl;
  *tblock_out = tblock;
  return hipSuccess;
}

template <int LOGK>
static hipError_t launch_tree_k(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s) {
  SubLevels sl;
  uint32_t tblock;
  hipError_t e = tree_pass_shape<LOGK>(g, tn, c, &sl, &tblock);
  if (e != hipSuccess) return e;
  if (tblock > 512) tblock = 512;
  const uint32_t chain = (lazy_top_height(g, tn) ? 0u : 1u) | (c.fold_max ? 2u : 0u);
  if (c.track_min) {
    PER_LAUNCH(KID_UPDATE_TREE, (k_update_tree<LOGK, true>), dim3(g.n[sl.hb], g.T), dim3(tblock), tree_lds_bytes<LOGK>(sl),
               s, g, sl, chain);
  } else {
    PER_LAUNCH(KID_UPDATE_TREE, (k_update_tree<LOGK, false>), dim3(g.n[sl.hb], g.T), dim3(tblock), tree_lds_bytes<LOGK>(sl),
               s, g, sl, chain);
  }
  return hipGetLastError();
}

// The tree pass of the update batch claimed with `c` together with the weights and row jobs in `a` / `rows`.
template <int LOGK>
static hipError_t launch_tree_finish_k(const Geom& g, const Tuning& tn, const ClaimArgs& c, const FieldTable* rows,
                                       const FinishArgs& a, hipStream_t s) {
  SubLevels sl;
  uint32_t tblock;
  hipError_t e = tree_pass_shape<LOGK>(g, tn, c, &sl, &tblock);
  if (e != hipSuccess) return e;
  if (tblock > 512) tblock = 512;   // half the lanes of a compute unit are left to the other jobs
  FieldTable ft{};
  if (rows) ft = *rows;
  const JobRanges jr = job_ranges(rows ? &ft : nullptr, a.B, tblock, a.w ? a.B : 0u, 0u, g.T, tn.whole_rows);
  const uint32_t tree_blocks = g.n[sl.hb];
  size_t lds = tree_lds_bytes<LOGK>(sl);
  if (lds < whole_rows_lds(jr)) lds = whole_rows_lds(jr);
  const uint32_t chain = (lazy_top_height(g, tn) ? 0u : 1u) | (c.fold_max ? 2u : 0u);
  const dim3 grid(tree_blocks + jr.first[2 + kMaxFields], g.T);
  const bool wide = !jr.whole_rows && any_field_moves_wide(rows ? &ft : nullptr);
#define PER_TREE_FINISH(TM, WD)                                                                                        \
  PER_LAUNCH(KID_TREE_FINISH, (k_tree_finish<LOGK, TM, WD>), grid, dim3(tblock), lds, s, g, sl, chain, tree_blocks, ft, jr, a)
  if (c.track_min) {
    if (wide) { PER_TREE_FINISH(true, true); } else { PER_TREE_FINISH(true, false); }
  } else {
    if (wide) { PER_TREE_FINISH(false, true); } else { PER_TREE_FINISH(false, false); }
  }
#undef PER_TREE_FINISH
  return hipGetLastError();
}

template <int LOGK>
static hipError_t launch_update_k(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s) {
  const uint32_t block = tn.update_block;
  PER_LAUNCH(KID_UPDATE_CLAIM, k_update_claim, dim3((c.B + block - 1) / block, g.T), dim3(block), 0, s, g, c);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_tree_k<LOGK>(g, tn, c, s);
}

hipError_t launch_update(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s) {
#define CALL(L) launch_update_k<L>(g, tn, c, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}
