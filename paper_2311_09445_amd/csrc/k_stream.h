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

    PER_MARK(2);
    // ---- rows of the sampled indices
    // (the weights, a power per sample, are computed while the rows are on their way: every lane that
    // owns a sample also owns a row element of the first sweep, so no wave runs the power twice)
    auto weights = [&]() {
      if (a.out_w && tid < B)
        a.out_w[bo] = total > 0.0f ? importance_weight(val, __uint_as_float(s_vmin), beta) : 0.0f;
    };
    if (move_rows_one_workgroup<true>(a.rows, t, ((uint64_t)s * T + t) * B, B, 0, N, s_idx, nullptr, weights)) flags |= 1u;

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
