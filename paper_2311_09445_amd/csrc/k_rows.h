// Data Storage: row gather and row scatter, and the second kernel of the fused calls.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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
// return value true.  Otherwise row j goes to ring slot cursor + j, unless bit j of skip_bits
// (a bit mask in LDS, or null) says that the row is not to be written.
// `between` is work of the caller's that every lane runs exactly once, after the lane's first load has
// been issued and before its first store (or at the end, for lanes that move nothing): per-lane
// arithmetic placed there overlaps the rows' trip to memory.  It must not contain barriers or
// cross-lane operations.
struct NothingBetween { __device__ __forceinline__ void operator()() const {} };
template <bool GATHER, typename Between = NothingBetween>
__device__ __forceinline__ bool move_rows_one_workgroup(const FieldTable& ft, uint32_t t, uint64_t dense_row0, uint32_t n,
                                                        uint32_t cursor, uint32_t N, const uint32_t* idx,
                                                        const uint32_t* skip_bits = nullptr, Between between = Between{}) {
  uint32_t first[kMaxFields + 1];
  first[0] = 0;
#pragma unroll
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f)
    first[f + 1] = first[f] + (f < ft.n_fields && ft.io[f] ? n * (ft.bytes[f] / ft.vec[f]) : 0u);
  bool bad = false;
  bool between_done = false;
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
      if (skip_bits && ((skip_bits[row >> 5] >> (row & 31u)) & 1u)) continue;
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
    if (!between_done) {
      between();
      between_done = true;
    }
    switch (w) {
      case 16: *reinterpret_cast<uint4*>(dst) = v; break;
      case 8: *reinterpret_cast<uint2*>(dst) = make_uint2(v.x, v.y); break;
      case 4: *reinterpret_cast<uint32_t*>(dst) = v.x; break;
      case 2: *reinterpret_cast<uint16_t*>(dst) = (uint16_t)v.x; break;
      default: *dst = (uint8_t)v.x; break;
    }
  }
  if (!between_done) between();
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
    weights_job(g, t, a.B, a.size, a.beta, a.w, a.weight_mode, b, jr.first[1]);
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
