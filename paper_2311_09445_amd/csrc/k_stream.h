// A list of steps in one launch on an LDS-resident tree.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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
// A tree whose leaves do not fit beside the rest (MEM) keeps heights 1 .. H in LDS and its leaves in memory: the
// paper's 100K-entry buffers at small fanouts are of that size.  The workgroup is still the only one that
// touches the tree while the kernel runs, so its own leaf stores, made visible to its other waves by a
// barrier, are all the coherence that takes; every operation then costs a trip or two to memory for the leaf
// groups it reads (sampling: the last level of the walk; insert and update: the groups whose sums change).
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
// (leaves_mem: the leaves in memory, or null when they are part of the LDS copy)
template <int LOGK>
__device__ __forceinline__ void resum_paths_lds(float* tree, const uint32_t* off, uint32_t H, bool active, uint32_t leaf,
                                                const float* leaves_mem) {
  constexpr int K = Fan<LOGK>::K;
  for (uint32_t h = 1; h <= H; ++h) {
    __syncthreads();   // (also makes the leaf stores of the other waves visible: one compute unit, one first-level cache)
    if (active) {
      const uint32_t parent = leaf >> (h * LOGK);
      if (h == 1 && leaves_mem) tree[off[h] + parent] = lane_group_sum<LOGK>(leaves_mem + (size_t)parent * K);
      else tree[off[h] + parent] = lane_group_sum<LOGK>(tree + off[h - 1] + (size_t)parent * K);
    }
  }
}

// One tree in the LDS of its workgroup, and the few words the operations below share.
struct LdsTree {
  float* tree;              // heights 0 .. H back to back, zero padding included (height 0 left out when leaves_mem is set)
  float* leaves_mem;        // null, or the tree's leaves in memory (zero padded to whole groups)
  const uint32_t* off;      // off[h]: where height h starts (floats); off[H + 1]: all floats
  uint32_t* sampled;        // [1024] indices of the latest sampling operation
  uint32_t* max_bits;       // running maximum priority (fp32 bits)
  uint32_t* vmin_bits;      // minimum of the batch being sampled (fp32 bits)
  uint32_t* bmin_bits;      // smallest positive leaf of the tree (fp32 bits), when the weights are relative to it
  uint32_t* skip;           // [32] bit j: row j of the insertion under way is deferred
  uint32_t H, N;
};

// The three operations are called by all 1024 lanes of the workgroup.  Each leaves the tree
// consistent, but its last phase may still be under way in other waves when it returns: the next
// operation starts with a barrier of its own (lds_sample), or the caller places one.

// Insertion of n <= 1024 rows: rows, leaves (given value, or the running maximum on entry), ancestors.
// prio, out_idx and protect point at this tree's part (or are null).
template <int LOGK>
__device__ __forceinline__ void lds_insert(const LdsTree& lt, const FieldTable& rows, uint32_t t, uint64_t dense_row0,
                                           uint32_t n, const float* prio, uint32_t* out_idx, const uint32_t* protect,
                                           uint32_t n_protect, uint32_t& cursor, uint32_t& size, uint32_t& flags) {
  const uint32_t tid = threadIdx.x;
  const uint32_t N = lt.N;
  if (protect) {   // collision-free insertion: rows aimed at a protected slot are deferred (see k_insert_small)
    if (tid < 32) lt.skip[tid] = 0;
    __syncthreads();
    for (uint32_t k = tid; k < n_protect; k += blockDim.x) {
      const uint32_t i = protect[k];
      if (i < N) {
        const uint32_t j = i >= cursor ? i - cursor : i + (N - cursor);   // position in the ring window
        if (j < n) atomicOr(&lt.skip[j >> 5], 1u << (j & 31u));
      }
    }
    __syncthreads();
  }
  (void)move_rows_one_workgroup<false>(rows, t, dense_row0, n, cursor, N, nullptr, protect ? lt.skip : nullptr);
  __syncthreads();   // (also: the tree is loaded, the operation before this one is complete)
  const float max_on_entry = __uint_as_float(*lt.max_bits);
  __syncthreads();
  bool ok = false;
  uint32_t slot = 0;
  if (tid < n) {
    uint64_t sl = (uint64_t)cursor + tid;
    if (sl >= N) sl -= N;
    slot = (uint32_t)sl;
    const bool deferred = protect && ((lt.skip[tid >> 5] >> (tid & 31u)) & 1u);
    if (out_idx) out_idx[tid] = deferred ? 0xFFFFFFFFu : slot;
    if (!deferred) {
      float v = max_on_entry;
      ok = true;
      if (prio) {
        v = prio[tid];
        ok = valid_priority(v);
        if (ok && v > 0.0f) atomicMax(lt.max_bits, __float_as_uint(v));
        if (!ok) flags |= 2u;
      }
      if (ok) (lt.leaves_mem ? lt.leaves_mem : lt.tree + lt.off[0])[slot] = v;
    }
  }
  resum_paths_lds<LOGK>(lt.tree, lt.off, lt.H, ok, slot, lt.leaves_mem);
  const uint64_t end = (uint64_t)cursor + n;
  cursor = (uint32_t)(end >= N ? end - N : end);
  size = size + n > N ? N : size + n;
}

// Priority sampling of B <= 1024 indices with importance weights, and the rows of the sampled
// indices.  u_i: this lane's uniform (lanes >= B: any value).  out_idx (never null), out_w, out_prio
// point at this tree's part.  Returns this lane's index.
template <int LOGK>
__device__ __forceinline__ uint32_t lds_sample(const LdsTree& lt, const FieldTable& rows, uint32_t t, uint64_t dense_row0,
                                               uint32_t B, float u_i, float beta, uint32_t* out_idx, float* out_w,
                                               float* out_prio, bool buffer_norm, uint32_t& flags) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t tid = threadIdx.x;
  if (tid == 0) {
    *lt.vmin_bits = kNoMin;
    *lt.bmin_bits = kNoMin;
  }
  __syncthreads();
  const float total = lt.tree[lt.off[lt.H]];
  if (buffer_norm && out_w) {   // weights relative to the whole tree: its smallest positive leaf, by a sweep over the LDS copy
    uint32_t m = kNoMin;
    const float* all_leaves = lt.leaves_mem ? lt.leaves_mem : lt.tree + lt.off[0];
    for (uint32_t e = tid; e < lt.N; e += blockDim.x) m = min_u32(m, positive_bits(all_leaves[e]));
    m = wave_min_u32(m);
    if ((tid & 63u) == 0 && m != kNoMin) atomicMin(lt.bmin_bits, m);
  }
  uint32_t node = 0xFFFFFFFFu;
  float val = 0.0f;
  if (total > 0.0f) {
    const uint32_t si = tid < B ? tid : B - 1;
    float r = ((float)si + u_i) * (total / (float)B);
    node = 0;
    val = total;
    for (uint32_t h = lt.H; h-- > 0;) {
      unsigned child;
      if (h == 0 && lt.leaves_mem) descend_lane<LOGK>(lt.leaves_mem + (size_t)node * K, r, child, val);
      else descend_lane<LOGK>(lt.tree + lt.off[h] + (size_t)node * K, r, child, val);
      node = node * K + child;
    }
    if (out_w && tid < B) atomicMin(lt.vmin_bits, __float_as_uint(val));
  } else if (tid == 0) {
    flags |= 4u;
  }
  if (tid < B) {
    lt.sampled[tid] = node;
    out_idx[tid] = node;
    if (out_prio) out_prio[tid] = val;
  }
  __syncthreads();
  // (the weights, a power per sample, are computed while the rows are on their way: every lane that
  // owns a sample also owns a row element of the first sweep, so no wave runs the power twice)
  auto weights = [&]() {
    if (out_w && tid < B)
      out_w[tid] = total > 0.0f ? importance_weight(val, __uint_as_float(buffer_norm ? *lt.bmin_bits : *lt.vmin_bits), beta)
                                : 0.0f;
  };
  if (move_rows_one_workgroup<true>(rows, t, dense_row0, B, 0, lt.N, lt.sampled, nullptr, weights)) flags |= 1u;
  return node;
}

// Priority update of B <= 1024 elements: lane tid < B sets leaf i to v.  Last writer by LDS
// atomics (see the head of this file), then the ancestors.
template <int LOGK>
__device__ __forceinline__ void lds_update(const LdsTree& lt, uint32_t B, uint32_t i, float v, uint32_t size,
                                           uint32_t& flags) {
  const uint32_t tid = threadIdx.x;
  bool valid = false;
  if (tid < B) {
    if (!(i < size)) flags |= 1u;
    else if (!valid_priority(v)) flags |= 2u;
    else valid = true;
  }
  const uint32_t mark = 0x80000001u + tid;
  bool won;
  if (lt.leaves_mem) {   // (the markers go through memory: atomics there, and a read that passes by the first-level cache)
    uint32_t* leaf_bits = reinterpret_cast<uint32_t*>(lt.leaves_mem);
    if (valid) atomicMax(&leaf_bits[i], mark);
    __syncthreads();
    won = valid && __hip_atomic_load(&leaf_bits[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == mark;
    __syncthreads();
    if (won) lt.leaves_mem[i] = v;
  } else {
    uint32_t* leaf_bits = reinterpret_cast<uint32_t*>(lt.tree + lt.off[0]);
    if (valid) atomicMax(&leaf_bits[i], mark);
    __syncthreads();
    won = valid && leaf_bits[i] == mark;
    __syncthreads();
    if (won) lt.tree[lt.off[0] + i] = v;
  }
  if (valid && v > 0.0f) atomicMax(lt.max_bits, __float_as_uint(v));
  resum_paths_lds<LOGK>(lt.tree, lt.off, lt.H, valid, i, lt.leaves_mem);
}

// Loads every height of tree t into LDS (lanes 64 .. 64 + H + 1 have filled s_off, lane 0 the maximum).  The heights
// are arrays of their own in memory and lie back to back in LDS; the copy runs over the LDS floats as one range, eight
// per lane in flight and all loads of a round before its first store, so that a tree of a dozen heights is not a dozen
// trips to memory one after the other.
__device__ __forceinline__ void lds_tree_load(const LevelTable& tab, const LdsTree& lt) {
  constexpr int R = 8;
  const uint32_t h_first = lt.leaves_mem ? 1u : 0u;
  const uint32_t begin = lt.off[h_first], end = lt.off[lt.H + 1];
  for (uint32_t base = begin; base < end; base += (uint32_t)R * blockDim.x) {
    float v[R];
    uint32_t h = h_first;   // (the height of this lane's element: found anew per round, then it only grows)
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const uint32_t e = base + (uint32_t)k * blockDim.x + threadIdx.x;
      v[k] = 0.0f;
      if (e < end) {
        while (h < lt.H && e >= lt.off[h + 1]) ++h;
        v[k] = tab.lvl[h][e - lt.off[h]];
      }
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const uint32_t e = base + (uint32_t)k * blockDim.x + threadIdx.x;
      if (e < end) lt.tree[e] = v[k];
    }
  }
}
// ... and back to memory, with the running maximum and the flags the lanes have collected.
__device__ __forceinline__ void lds_tree_store(const Geom& g, uint32_t t, const LevelTable& tab, const LdsTree& lt,
                                               uint32_t flags, uint32_t* s_flags) {
  for (uint32_t h = lt.leaves_mem ? 1u : 0u; h <= lt.H; ++h) {
    float* lvl = tab.lvl[h];
    const float* src = lt.tree + lt.off[h];
    for (uint32_t e = threadIdx.x; e < tab.n[h]; e += blockDim.x) lvl[e] = src[e];
  }
  if (threadIdx.x == 0) g.max_v[t] = __uint_as_float(*lt.max_bits);
  if (flags) atomicOr(s_flags, flags);
  __syncthreads();
  if (threadIdx.x == 0 && *s_flags) atomicOr(&g.status[t], *s_flags);
}

template <int LOGK>
__global__ void __launch_bounds__(1024)
k_run_steps(StreamKernelArgs ka) {
  const Geom& g = ka.g;
  const StreamArgs& a = ka.a;
  extern __shared__ __attribute__((aligned(16))) float tree[];
  __shared__ LevelTable tab;
  __shared__ uint32_t s_off[kMaxHeight + 2];
  __shared__ uint32_t s_max, s_vmin, s_bmin, s_flags;
  const uint32_t t = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const uint32_t H = g.H, T = g.T, B = a.B, n_ins = a.n_insert;
  fill_level_table(H, t, &tab);
  if (tid >= 64 && tid <= 64 + H + 1)
    s_off[tid - 64] = kernarg_at<StreamArgs>(offsetof(StreamKernelArgs, a))->off[tid - 64];
  if (tid == 0) {
    s_max = read_max_bits(g, t);
    s_flags = 0;
  }
  __syncthreads();
  LdsTree lt;
  lt.tree = tree;
  lt.leaves_mem = a.leaves_in_memory ? tab.lvl[0] : nullptr;
  lt.off = s_off;
  lt.sampled = reinterpret_cast<uint32_t*>(tree + s_off[H + 1]);
  lt.max_bits = &s_max;
  lt.vmin_bits = &s_vmin;
  lt.bmin_bits = &s_bmin;
  lt.skip = nullptr;
  lt.H = H;
  lt.N = g.N;
  lds_tree_load(tab, lt);
  uint32_t cursor = a.cursor, size = a.size;
  uint32_t flags = 0;

  for (uint32_t s = 0; s < a.n_steps; ++s) {
    const size_t bo = ((size_t)s * T + t) * B;
    // inputs of this step, fetched before the tree work
    float u_i = 0.0f, up_v = 0.0f;
    uint32_t up_i = 0;
    if (tid < B) {
      u_i = a.u[bo + tid];
      if (a.upd_prio) {
        up_v = a.upd_prio[bo + tid];
        if (!a.upd_is_sampled) up_i = a.upd_idx[bo + tid];
      }
    }
    const float beta = a.beta[s];
    if (n_ins) {
      const uint64_t io = ((uint64_t)s * T + t) * n_ins;
      lds_insert<LOGK>(lt, a.ins, t, io, n_ins, a.ins_prio ? a.ins_prio + io : nullptr, nullptr, nullptr, 0, cursor, size,
                       flags);
    }
    const uint32_t node = lds_sample<LOGK>(lt, a.rows, t, ((uint64_t)s * T + t) * B, B, u_i, beta, a.out_idx + bo,
                                           a.out_w ? a.out_w + bo : nullptr, a.out_prio ? a.out_prio + bo : nullptr,
                                           a.buffer_norm != 0, flags);
    if (a.upd_prio) lds_update<LOGK>(lt, B, a.upd_is_sampled ? node : up_i, up_v, size, flags);
    __syncthreads();
  }
  lds_tree_store(g, t, tab, lt, flags, &s_flags);
}

// ---------------------------------------------------------------------------------
// a queue of op-coded requests on an LDS-resident tree
// ---------------------------------------------------------------------------------
// The same workgroup-per-tree arrangement, driven by a queue of requests in memory instead of a
// fixed step: each request names its operation (the paper's unified operation code, Section V-A)
// and is decoded when its turn comes.  The queue's length is fixed at launch; the kernel ends after
// its last request.
struct QueueKernelArgs {            // one kernel argument (Geom first: see fill_level_table)
  Geom g;
  QueueArgs a;
};

template <int LOGK>
__global__ void __launch_bounds__(1024)
k_run_requests(QueueKernelArgs ka) {
  const Geom& g = ka.g;
  const QueueArgs& a = ka.a;
  extern __shared__ __attribute__((aligned(16))) float tree[];
  __shared__ LevelTable tab;
  __shared__ FieldTable s_ft;        // the buffer's columns with the current request's row arrays
  __shared__ uint32_t s_off[kMaxHeight + 2];
  __shared__ uint32_t s_skip[32];
  __shared__ uint32_t s_max, s_vmin, s_bmin, s_flags;
  const uint32_t t = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const uint32_t H = g.H;
  fill_level_table(H, t, &tab);
  if (tid >= 64 && tid <= 64 + H + 1)
    s_off[tid - 64] = kernarg_at<QueueArgs>(offsetof(QueueKernelArgs, a))->off[tid - 64];
  if (tid == 0) {
    s_max = read_max_bits(g, t);
    s_flags = 0;
    s_ft = a.fields;
  }
  __syncthreads();
  LdsTree lt;
  lt.tree = tree;
  lt.leaves_mem = a.leaves_in_memory ? tab.lvl[0] : nullptr;
  lt.off = s_off;
  lt.sampled = reinterpret_cast<uint32_t*>(tree + s_off[H + 1]);
  lt.max_bits = &s_max;
  lt.vmin_bits = &s_vmin;
  lt.bmin_bits = &s_bmin;
  lt.skip = s_skip;
  lt.H = H;
  lt.N = g.N;
  lds_tree_load(tab, lt);
  uint32_t cursor = a.cursor, size = a.size;
  uint32_t flags = 0;
  uint32_t last_node = 0xFFFFFFFFu;   // this lane's index from the latest sampling request

  for (uint32_t r = 0; r < a.n_requests; ++r) {
    const per_request& q = a.queue[r];
    const uint32_t n = q.n;
    const size_t to = (size_t)t * n;
    __syncthreads();   // the request before this one is complete (and has finished with s_ft)
    if (tid < (uint32_t)kMaxFields) s_ft.io[tid] = static_cast<uint8_t*>(q.field[tid]);
    __syncthreads();
    if (q.op == PER_OP_INSERT) {
      lds_insert<LOGK>(lt, s_ft, t, to, n, q.prio ? q.prio + to : nullptr, q.idx ? q.idx + to : nullptr,
                       q.protect ? q.protect + (size_t)t * q.n_protect : nullptr, q.n_protect, cursor, size, flags);
    } else if (q.op == PER_OP_SAMPLE) {
      const float u_i = tid < n ? q.u[to + tid] : 0.0f;
      last_node = lds_sample<LOGK>(lt, s_ft, t, to, n, u_i, q.beta, q.idx + to, q.out_weight ? q.out_weight + to : nullptr,
                                   q.out_prio ? q.out_prio + to : nullptr, a.buffer_norm != 0, flags);
    } else if (q.op == PER_OP_UPDATE) {
      float v = 0.0f;
      uint32_t i = last_node;
      if (tid < n) {
        v = q.prio[to + tid];
        if (q.idx) i = q.idx[to + tid];
      }
      lds_update<LOGK>(lt, n, i, v, size, flags);
    }
  }
  __syncthreads();
  lds_tree_store(g, t, tab, lt, flags, &s_flags);
}

// LDS floats of a tree's copy (every height padded to whole child groups), or 0 if it cannot be held beside the step
// kernel's other LDS data.  The whole tree if that fits; else the heights 1 .. H, the leaves staying in memory
// (*leaves_in_memory says which).
constexpr uint32_t kStreamLdsBytes = 156 * 1024;
uint32_t stream_tree_floats(const Geom& g, uint32_t* off, uint32_t* leaves_in_memory) {
  for (uint32_t skip = 0; skip < 2; ++skip) {
    uint64_t floats = 0;
    bool fits = true;
    for (uint32_t h = 0; h <= g.H && fits; ++h) {
      if (off) off[h] = (uint32_t)floats;
      if (h == 0 && skip) continue;
      floats += h < g.H ? ((uint64_t)g.n[h] + g.K - 1) / g.K * g.K : 4;   // (the root padded to 16 bytes)
      fits = floats * 4 <= kStreamLdsBytes;
    }
    if (!fits || (floats + 1024) * 4 > kStreamLdsBytes || (skip && g.H < 2)) continue;
    if (off) off[g.H + 1] = (uint32_t)floats;
    if (leaves_in_memory) *leaves_in_memory = skip;
    return (uint32_t)floats;
  }
  return 0u;
}

template <int LOGK>
static hipError_t launch_run_steps_k(const Geom& g, const Tuning& tn, StreamArgs a, hipStream_t s) {
  StreamKernelArgs ka{};
  ka.g = g;
  ka.a = a;
  const uint32_t floats = stream_tree_floats(g, ka.a.off, &ka.a.leaves_in_memory);
  if (!floats) return hipErrorInvalidValue;
  const size_t bytes = ((size_t)floats + 1024) * 4;   // the tree and the sampled indices of one step
  hipError_t e = grant_lds<&k_run_steps<LOGK>>(tn, bytes);
  if (e != hipSuccess) return e;
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

template <int LOGK>
static hipError_t launch_run_requests_k(const Geom& g, const Tuning& tn, const QueueArgs& a, hipStream_t s) {
  QueueKernelArgs ka{};
  ka.g = g;
  ka.a = a;
  const uint32_t floats = stream_tree_floats(g, ka.a.off, &ka.a.leaves_in_memory);
  if (!floats) return hipErrorInvalidValue;
  const size_t bytes = ((size_t)floats + 1024) * 4;   // the tree and the indices of the latest sampling request
  hipError_t e = grant_lds<&k_run_requests<LOGK>>(tn, bytes);
  if (e != hipSuccess) return e;
  PER_LAUNCH(KID_RUN_REQUESTS, k_run_requests<LOGK>, dim3(g.T), dim3(1024), bytes, s, ka);
  return hipGetLastError();
}

hipError_t launch_run_requests(const Geom& g, const Tuning& tn, const QueueArgs& a, hipStream_t s) {
#define CALL(L) launch_run_requests_k<L>(g, tn, a, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}
