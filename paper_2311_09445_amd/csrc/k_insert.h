// Insertion: leaf writes, and the single-kernel insert of a few rows.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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
constexpr uint32_t kInsertSmallRows = 4096;   // most rows one workgroup takes
struct InsertPlan {
  Range2 r[kInsertHeights];        // touched nodes of height h + 1
  uint32_t off[kInsertHeights];    // where their child groups start in LDS (floats)
  uint32_t chain_from;             // from this height on one wave holds a lane group per touched node of every height
  uint32_t single_from;            // from this height on every height has one touched node, and one wave a lane group per height
};
struct InsertArgs {                // one kernel argument, so that both parts sit at known offsets of the segment
  Geom g;
  InsertPlan plan;
  uint32_t track_min;              // also renew min1 (smallest positive leaf) of the touched height-1 nodes
};

template <int LOGK>
__global__ void __launch_bounds__(1024)
k_insert_small(InsertArgs a, FieldTable ft, uint32_t n, uint32_t cursor, const float* __restrict__ prio,
               uint32_t* __restrict__ out_idx, const uint32_t* __restrict__ protect, uint32_t n_protect) {
  // (the lines read through the scalar cache: the first words and the scalars' pointers of the geometry, and what
  // follows the plan; the per-height tables of geometry and plan are fetched by vector loads, a lane per height)
  if (threadIdx.x < 256u) touch_kernel_argument_lines<(1u << 0) | (3u << 12) | (0xFu << 24)>();
  const Geom& g = a.g;
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  extern __shared__ __attribute__((aligned(16))) float staged[];
  __shared__ LevelTable tab;
  __shared__ Range2 s_r[kInsertHeights];
  __shared__ uint32_t s_off[kInsertHeights];
  __shared__ uint32_t s_skip[kInsertSmallRows / 32];   // bit j: row j is deferred (its slot is protected)
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
  // Collision-free insertion (Section IV-B): a row whose ring slot is named by the protected batch is
  // deferred.  The batch is scanned once; an index inside the ring window [cursor, cursor + n) marks its row.
  if (protect) {
    for (uint32_t w = threadIdx.x; w < kInsertSmallRows / 32; w += blockDim.x) s_skip[w] = 0;
    __syncthreads();
    for (uint32_t k = threadIdx.x; k < n_protect; k += blockDim.x) {
      const uint32_t i = protect[(size_t)t * n_protect + k];
      if (i < g.N) {
        const uint32_t j = i >= cursor ? i - cursor : i + (g.N - cursor);   // position in the ring window
        if (j < n) atomicOr(&s_skip[j >> 5], 1u << (j & 31u));
      }
    }
    __syncthreads();
  }
  // the rows need none of the tables: their trip to memory overlaps the fetch of the tables
  (void)move_rows_one_workgroup<false>(ft, t, (uint64_t)t * n, n, cursor, g.N, nullptr, protect ? s_skip : nullptr);
  __syncthreads();
  PER_MARK(1);
  // ---- everything that is read: the child groups of all touched nodes, the running maximum
  // (one flat index space over the staged floats of all heights, so that every lane's loads are on their way before
  // anything waits: a loop per height made a trip to memory per height)
  {
    const Range2 top_r = s_r[H - 1];
    const uint32_t total = s_off[H - 1] + ((top_r.b0 - top_r.a0) + (top_r.b1 - top_r.a1)) * K;
    for (uint32_t e0 = threadIdx.x; e0 < total; e0 += blockDim.x) {
      uint32_t hi = 0;   // the height below the staged group: the number of heights whose groups start at or before e0, less one
      for (uint32_t k = 1; k < H; ++k) hi += e0 >= s_off[k] ? 1u : 0u;
      const Range2 r = s_r[hi];
      const uint32_t e = e0 - s_off[hi];
      const uint32_t c0 = r.b0 - r.a0;
      const uint32_t pos = e >> LOGK;
      const uint32_t node = pos < c0 ? r.a0 + pos : r.a1 + (pos - c0);
      staged[e0] = as_global(tab.lvl[hi])[(size_t)node * K + (e & (K - 1))];
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
    const bool deferred = protect && ((s_skip[j >> 5] >> (j & 31u)) & 1u);
    if (out_idx) out_idx[(size_t)t * n + j] = deferred ? 0xFFFFFFFFu : (uint32_t)slot;
    if (deferred) continue;
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
      as_global(tab.lvl[0])[slot] = v;
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
  // From chain_from on the first wave finishes the heights alone: what it patches into the staged groups of the
  // next height it reads back itself, so no workgroup barrier stands between those heights (a barrier and the loop
  // around it cost three times the sum itself).
  const unsigned q = threadIdx.x % LPS;
  const uint32_t grp = threadIdx.x / LPS, ngrp = blockDim.x / LPS;
  const uint32_t chain_from = kernarg_at<InsertPlan>(offsetof(InsertArgs, plan))->chain_from;
  // (what the chained heights need to know of each height sits in the registers of lane h - 1 and is read from
  // there: fetched from LDS per height, it stood in front of every sum)
  const uint32_t ml = (threadIdx.x & 63u) < H ? (threadIdx.x & 63u) : 0u;
  const Range2 mr = s_r[ml];
  const uint32_t moff = s_off[ml];
  const unsigned long long mlvl = reinterpret_cast<unsigned long long>(tab.lvl[ml + 1]);
  auto lane_word = [](uint32_t v, uint32_t l) -> uint32_t { return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l); };
  const uint32_t single_from = kernarg_at<InsertPlan>(offsetof(InsertArgs, plan))->single_from;
  for (uint32_t h = 1; h < single_from && h <= H; ++h) {
    const bool chained = h >= chain_from;
    if (chained && threadIdx.x >= 64) break;
    if (chained) {
      const uint32_t a0 = lane_word(mr.a0, h - 1), b0 = lane_word(mr.b0, h - 1), a1 = lane_word(mr.a1, h - 1), b1 = lane_word(mr.b1, h - 1);
      const uint32_t o = lane_word(moff, h - 1);
      const uint32_t c0 = b0 - a0, cnt = c0 + (b1 - a1);
      float* par = reinterpret_cast<float*>(((unsigned long long)lane_word((uint32_t)(mlvl >> 32), h - 1) << 32) |
                                            lane_word((uint32_t)mlvl, h - 1));
      const uint32_t pos = grp;
      const bool ok = pos < cnt;
      const float sum = group_sum<LOGK>(staged + o + (size_t)(ok ? pos : 0u) * K, q);
      uint32_t mn = kNoMin;
      if (a.track_min && h == 1) mn = group_min_positive<LOGK>(staged + s_off[0] + (size_t)(ok ? pos : 0u) * K, q);
      if (ok && q == 0) {
        const uint32_t node = pos < c0 ? a0 + pos : a1 + (pos - c0);
        as_global(par)[node] = sum;
        if (a.track_min && h == 1) g.min1[(size_t)t * g.min1_stride + node] = mn;
        if (h < H) {
          Range2 up;
          up.a0 = lane_word(mr.a0, h);
          up.b0 = lane_word(mr.b0, h);
          up.a1 = lane_word(mr.a1, h);
          up.b1 = lane_word(mr.b1, h);
          staged[lane_word(moff, h) + plan_pos(up, node >> LOGK) * K + (node & (K - 1))] = sum;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      continue;
    }
    const Range2 r = s_r[h - 1];
    const uint32_t c0 = r.b0 - r.a0, cnt = c0 + (r.b1 - r.a1);
    float* par = tab.lvl[h];
    for (uint32_t base = 0; base < cnt; base += ngrp) {
      const uint32_t pos = base + grp;
      const bool ok = pos < cnt;
      const float sum = group_sum<LOGK>(staged + s_off[h - 1] + (size_t)(ok ? pos : 0u) * K, q);
      uint32_t mn = kNoMin;
      if (a.track_min && h == 1)   // the staged groups of height 0 hold the leaves of every touched height-1 node
        mn = group_min_positive<LOGK>(staged + s_off[0] + (size_t)(ok ? pos : 0u) * K, q);
      if (ok && q == 0) {
        const uint32_t node = pos < c0 ? r.a0 + pos : r.a1 + (pos - c0);
        as_global(par)[node] = sum;
        if (a.track_min && h == 1) g.min1[(size_t)t * g.min1_stride + node] = mn;
        if (h < H) staged[s_off[h] + plan_pos(s_r[h], node >> LOGK) * K + (node & (K - 1))] = sum;
      }
    }
    lds_barrier();   // the next height reads the staged groups only
  }
  // ---- the heights with a single touched node: lane group i of the first wave holds the staged group of height
  // single_from + i in registers; going up, the sum of the height below is put into its place in the group above
  // (a register select) and that group is summed, a handful of instructions per height (the loop above spends
  // about sixty, which is what a height costs there, not its trip through LDS).
  if (single_from <= H && threadIdx.x < 64u) {
    const uint32_t mine = threadIdx.x / LPS;              // this lane's group
    const uint32_t hs = single_from + mine;               // its height
    const bool live = hs <= H;
    const uint32_t src = live ? hs : single_from;
    const float* grp_at = staged + s_off[src - 1];
    float c0, c1v, c2v = 0.0f, c3v = 0.0f;
    if constexpr (LOGK == 1) {
      const float2 c = *reinterpret_cast<const float2*>(grp_at);
      c0 = c.x;
      c1v = c.y;
    } else {
      const float4 c = *reinterpret_cast<const float4*>(grp_at + 4 * q);
      c0 = c.x;
      c1v = c.y;
      c2v = c.z;
      c3v = c.w;
    }
    const uint32_t my_node = s_r[src - 1].a0;             // (one range of one node)
    float* my_level = tab.lvl[src];
    uint32_t mn = kNoMin;
    if (a.track_min && single_from == 1) mn = group_min_positive<LOGK>(staged + s_off[0], q);   // (meant for lane group 0 only)
    float fin = 0.0f, below = 0.0f;
    uint32_t node_below = 0;
    const uint32_t count = H - single_from + 1;
    for (uint32_t i = 0; i < count; ++i) {
      const uint32_t node_here = lane_word(my_node, i * LPS);
      if (i > 0) {
        const uint32_t ci = node_below - node_here * K;   // the node of the height below is child ci of this one
        const bool here = mine == i && (LOGK == 1 || q == (ci >> 2));
        const uint32_t e = LOGK == 1 ? ci : (ci & 3u);
        c0 = here && e == 0 ? below : c0;
        c1v = here && e == 1 ? below : c1v;
        c2v = here && e == 2 ? below : c2v;
        c3v = here && e == 3 ? below : c3v;
      }
      float sum;
      if constexpr (LOGK == 1) sum = c0 + c1v;
      else sum = butterfly_sum<Fan<LOGK>::LOGLPS>((c0 + c1v) + (c2v + c3v));
      fin = mine == i ? sum : fin;
      below = __int_as_float((int)lane_word((uint32_t)__float_as_int(sum), i * LPS));
      node_below = node_here;
    }
    if (live && q == 0) {
      as_global(my_level)[my_node] = fin;
      if (a.track_min && hs == 1) g.min1[(size_t)t * g.min1_stride + my_node] = mn;
    }
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
static uint32_t tree_pass_height(const Geom& g);
bool insert_fits_one_workgroup(const Geom& g, const FieldTable* ft, uint32_t n) {
  uint64_t bytes = 0;
  if (ft)
    for (uint32_t f = 0; f < ft->n_fields; ++f)
      if (ft->io[f]) bytes += (uint64_t)n * ft->bytes[f];
  if (n > kInsertSmallRows || bytes > 256 * 1024) return false;
  // the staged child groups must fit the dynamic LDS a kernel gets without asking for more (64 KB, of which
  // the kernel's tables take about 2 KB): an upper bound over every ring position, with the heights an
  // update may have left stale taken whole
  const uint32_t hb = tree_pass_height(g);
  const bool lazy = hb < g.H && g.n[hb] <= kLazyTopNodes;
  uint64_t floats = 0;
  for (uint32_t h = 1; h <= g.H; ++h) {
    uint64_t nodes = (((uint64_t)n - 1) >> (h * g.logK < 63 ? h * g.logK : 63)) + 3;   // two ranges, each may straddle a node
    if (nodes > g.n[h] || (lazy && h > hb)) nodes = g.n[h];
    floats += nodes * g.K;
  }
  return floats * 4 <= 60 * 1024;
}

template <int LOGK>
static hipError_t launch_insert_small_k(const Geom& g, const Tuning& tn, const FieldTable* ft, uint32_t n,
                                        uint32_t cursor, const float* prio, uint32_t* out_idx, uint32_t stale_hb,
                                        const uint32_t* protect, uint32_t n_protect, bool track_min, hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  FieldTable f{};
  if (ft) f = *ft;
  InsertArgs a{};
  a.g = g;
  a.track_min = track_min ? 1u : 0u;
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
  plan.single_from = g.H + 1;
  for (uint32_t h = g.H; h >= 1; --h) {
    const Range2& rr = plan.r[h - 1];
    if ((rr.b0 - rr.a0) + (rr.b1 - rr.a1) != 1 || rr.b0 - rr.a0 != 1) break;
    if ((uint64_t)(g.H - h + 1) * Fan<LOGK>::LPS > 64) break;
    plan.single_from = h;
  }
  plan.chain_from = g.H + 1;
  for (uint32_t h = g.H; h >= 1; --h) {
    const Range2& rr = plan.r[h - 1];
    if ((uint64_t)((rr.b0 - rr.a0) + (rr.b1 - rr.a1)) * Fan<LOGK>::LPS > 64) break;
    plan.chain_from = h;
  }
  uint32_t block = (n * Fan<LOGK>::LPS + 63) / 64 * 64;
  // (enough lanes to move all row elements in one sweep: a second sweep is a second trip to memory)
  uint64_t row_elements = 0;
  for (uint32_t i = 0; i < f.n_fields; ++i)
    if (f.io[i]) row_elements += (uint64_t)n * (f.bytes[i] / f.vec[i]);
  if (row_elements > block) block = (uint32_t)((row_elements > 1024 ? 1024 : row_elements) + 63) / 64 * 64;
  if (block < 256) block = 256;
  if (block > 1024) block = 1024;
  PER_LAUNCH(KID_INSERT_SMALL, k_insert_small<LOGK>, dim3(g.T), dim3(block), (size_t)floats * 4, s, a, f, n, cursor, prio,
             out_idx, protect, n_protect);
  return hipGetLastError();
}

hipError_t launch_insert_small(const Geom& g, const Tuning& tn, const FieldTable* ft, uint32_t n, uint32_t cursor,
                               const float* prio, uint32_t* out_idx, uint32_t stale_hb, const uint32_t* protect,
                               uint32_t n_protect, bool track_min, hipStream_t s) {
#define CALL(L) launch_insert_small_k<L>(g, tn, ft, n, cursor, prio, out_idx, stale_hb, protect, n_protect, track_min, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}
