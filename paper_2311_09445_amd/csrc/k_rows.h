// Data Storage: row gather and row scatter, and the second kernel of the fused calls.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// Data Storage: row gather and row scatter
// ---------------------------------------------------------------------------------
// A field of E bytes is moved by E/vec adjacent lanes, vec bytes each, so the dense side is fully
// coalesced and the storage side is coalesced within a row.
//
// Elements a lane keeps in flight per sweep, about 32 bytes: narrow fields need more elements to cover
// the same latency, and a launch over many trees must not need several rounds of workgroups.  Per
// sweep all indices are fetched first, then all rows, then everything is stored (a wait for loaded
// data also waits for earlier stores, so load -> store -> load would cost a memory trip per
// element).  Elements beyond the end are clamped to the lane's first one, so that every load is
// unconditional and the three phases stay straight-line code; only their stores are skipped.
template <typename V>
struct InFlight {
  static constexpr int U = sizeof(V) >= 16 ? 2 : sizeof(V) == 8 ? 4 : 8;
};
static uint32_t max_in_flight(uint32_t vec) { return vec >= 16 ? 2u : vec == 8 ? 4u : 8u; }

// A field whose size and addresses are multiples of 4 bytes only (17 floats, say) still moves in 16-byte
// pieces when it is long enough: pieces on 4-byte boundaries, which the target's memory instructions allow,
// the last one ending with the field and overlapping the one before it (the shared bytes are written twice
// with the same values).  A row of 68 bytes is then 5 moves instead of 17.
struct __attribute__((packed, aligned(4))) Wide16 {
  uint32_t x, y, z, w;
};
__host__ __device__ __forceinline__ bool moves_wide(uint32_t bytes, uint32_t vec) { return vec == 4 && bytes >= 32; }
// elements a row of the field is moved in, and elements a lane keeps in flight
__host__ __device__ __forceinline__ uint32_t row_elements(uint32_t bytes, uint32_t vec) {
  return moves_wide(bytes, vec) ? (bytes + 15u) / 16u : bytes / vec;
}
static uint32_t field_in_flight(uint32_t bytes, uint32_t vec) { return moves_wide(bytes, vec) ? 2u : max_in_flight(vec); }

// A lane's values for the elements of a sweep: a nested struct reached through compile-time paths only
// (an array written in unrolled loops was moved to LDS or scratch by the compiler).
template <typename T, int N>
struct Regs {
  T head;
  Regs<T, N - 1> tail;
};
template <typename T>
struct Regs<T, 0> {};
template <int K, typename T, int N>
__device__ __forceinline__ T& reg(Regs<T, N>& r) {
  if constexpr (K == 0) return r.head;
  else return reg<K - 1>(r.tail);
}

struct RowMove {                 // what the elements of one field and tree have in common
  uint8_t* col;                  // the field in row 0 of the tree
  uint8_t* io;                   // the tree's dense rows: element e sits at byte e * sizeof(V)
  const uint32_t* idx;           // the tree's indices (gather)
  uint64_t total, stride;        // elements of the job; elements between two of a lane's
  uint32_t RS, epr, cursor, N;
};

// Element K of the sweep that starts at e0 (clamped to e0 beyond the end, so that loads need no branch).
template <int K>
__device__ __forceinline__ uint64_t sweep_elem(const RowMove& m, uint64_t e0, bool& live) {
  const uint64_t e = e0 + (uint64_t)K * m.stride;
  live = e < m.total;
  return live ? e : e0;
}
// The three phases of a sweep, each over elements K .. U-1: where the stored side of every element is
// (for a gather that is a load of the index), the loads, the stores.
template <typename V, bool GATHER, int K, int U>
__device__ __forceinline__ void sweep_where(const RowMove& m, uint64_t e0, Regs<uint32_t, U>& at) {
  if constexpr (K < U) {
    bool live;
    const uint32_t row = (uint32_t)(sweep_elem<K>(m, e0, live) / m.epr);
    if constexpr (GATHER) {
      reg<K>(at) = m.idx[row];
    } else {
      uint64_t slot = (uint64_t)m.cursor + row;
      if (slot >= m.N) slot -= m.N;
      reg<K>(at) = (uint32_t)slot;
    }
    sweep_where<V, GATHER, K + 1, U>(m, e0, at);
  }
}
// (values narrower than a register are kept widened)
template <typename V>
using Held = typename std::conditional<sizeof(V) < 4, uint32_t, V>::type;
template <typename V, bool GATHER, int K, int U>
__device__ __forceinline__ void sweep_load(const RowMove& m, uint64_t e0, Regs<uint32_t, U>& at, Regs<Held<V>, U>& v,
                                           bool& bad) {
  if constexpr (K < U) {
    bool live;
    const uint64_t e = sweep_elem<K>(m, e0, live);
    if constexpr (GATHER) {
      const uint32_t within = (uint32_t)(e % m.epr);
      const bool ok = reg<K>(at) < m.N;
      bad |= !ok;
      V got = *(reinterpret_cast<const V*>(m.col + (uint64_t)(ok ? reg<K>(at) : 0u) * m.RS) + within);
      if (!ok) __builtin_memset(&got, 0, sizeof(V));
      reg<K>(v) = (Held<V>)got;
    } else {
      reg<K>(v) = (Held<V>)*(reinterpret_cast<const V*>(m.io) + e);
    }
    sweep_load<V, GATHER, K + 1, U>(m, e0, at, v, bad);
  }
}
template <typename V, bool GATHER, int K, int U>
__device__ __forceinline__ void sweep_store(const RowMove& m, uint64_t e0, Regs<uint32_t, U>& at, Regs<Held<V>, U>& v) {
  if constexpr (K < U) {
    bool live;
    const uint64_t e = sweep_elem<K>(m, e0, live);
    if (live) {
      if constexpr (GATHER) *(reinterpret_cast<V*>(m.io) + e) = (V)reg<K>(v);
      else *(reinterpret_cast<V*>(m.col + (uint64_t)reg<K>(at) * m.RS) + (uint32_t)(e % m.epr)) = (V)reg<K>(v);
    }
    sweep_store<V, GATHER, K + 1, U>(m, e0, at, v);
  }
}

// (row0, nrows: only the rows [row0, row0 + nrows) of the B rows per tree; gathers only)
template <typename V, bool GATHER>
__device__ __forceinline__ void move_rows(const FieldTable& ft, uint32_t f, uint32_t t, uint32_t B,
                                          const uint32_t* __restrict__ idx, uint32_t cursor, uint32_t N,
                                          uint32_t* status, uint32_t job_block, uint32_t job_blocks, uint32_t row0 = 0,
                                          uint32_t nrows = 0xFFFFFFFFu) {
  constexpr int U = InFlight<V>::U;
  RowMove m;
  const uint32_t E = ft.bytes[f];
  m.RS = ft.row_stride;
  m.epr = E / (uint32_t)sizeof(V);
  m.total = (uint64_t)(nrows < B - row0 ? nrows : B - row0) * m.epr;
  m.col = ft.col[f] + (uint64_t)t * ft.col_stride[f];
  m.io = ft.io[f] + ((uint64_t)t * B + row0) * E;
  m.idx = idx ? idx + (size_t)t * B + row0 : nullptr;
  m.stride = (uint64_t)job_blocks * blockDim.x;
  m.cursor = cursor;
  m.N = N;
  bool bad = false;
  for (uint64_t e0 = (uint64_t)job_block * blockDim.x + threadIdx.x; e0 < m.total; e0 += U * m.stride) {
    Regs<uint32_t, U> at;
    Regs<Held<V>, U> v;
    sweep_where<V, GATHER, 0, U>(m, e0, at);
    sweep_load<V, GATHER, 0, U>(m, e0, at, v, bad);
    sweep_store<V, GATHER, 0, U>(m, e0, at, v);
  }
  if (bad) atomicOr(&status[t], 1u);
}

// The same for a field that moves wide (see Wide16): element e of the job is piece e % epr of row e / epr,
// at byte min(16 piece, E - 16) of the field on both sides.  Kept apart from the mover above so that the
// code of that one stays as it is.  Held as plain vectors (a packed type among the held values would keep
// them out of registers).
struct WideMove {
  RowMove m;
  uint32_t E;   // bytes of the field in a row
};
__device__ __forceinline__ uint32_t wide_offset(const WideMove& w, uint64_t e) {
  const uint32_t off = 16u * (uint32_t)(e % w.m.epr);
  return off + 16u <= w.E ? off : w.E - 16u;
}
__device__ __forceinline__ uint4 load_wide(const uint8_t* p) {
  const Wide16 x = *reinterpret_cast<const Wide16*>(p);
  return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void store_wide(uint8_t* p, const uint4& h) {
  Wide16 x;
  x.x = h.x;
  x.y = h.y;
  x.z = h.z;
  x.w = h.w;
  *reinterpret_cast<Wide16*>(p) = x;
}
template <bool GATHER, int K, int U>
__device__ __forceinline__ void wide_load(const WideMove& w, uint64_t e0, Regs<uint32_t, U>& at, Regs<uint4, U>& v, bool& bad) {
  if constexpr (K < U) {
    bool live;
    const uint64_t e = sweep_elem<K>(w.m, e0, live);
    if constexpr (GATHER) {
      const bool ok = reg<K>(at) < w.m.N;
      bad |= !ok;
      uint4 got = load_wide(w.m.col + (uint64_t)(ok ? reg<K>(at) : 0u) * w.m.RS + wide_offset(w, e));
      if (!ok) got = make_uint4(0, 0, 0, 0);
      reg<K>(v) = got;
    } else {
      reg<K>(v) = load_wide(w.m.io + (e / w.m.epr) * w.E + wide_offset(w, e));
    }
    wide_load<GATHER, K + 1, U>(w, e0, at, v, bad);
  }
}
template <bool GATHER, int K, int U>
__device__ __forceinline__ void wide_store(const WideMove& w, uint64_t e0, Regs<uint32_t, U>& at, Regs<uint4, U>& v) {
  if constexpr (K < U) {
    bool live;
    const uint64_t e = sweep_elem<K>(w.m, e0, live);
    if (live) {
      if constexpr (GATHER) store_wide(w.m.io + (e / w.m.epr) * w.E + wide_offset(w, e), reg<K>(v));
      else store_wide(w.m.col + (uint64_t)reg<K>(at) * w.m.RS + wide_offset(w, e), reg<K>(v));
    }
    wide_store<GATHER, K + 1, U>(w, e0, at, v);
  }
}
template <bool GATHER>
__device__ __forceinline__ void move_rows_wide(const FieldTable& ft, uint32_t f, uint32_t t, uint32_t B,
                                               const uint32_t* __restrict__ idx, uint32_t cursor, uint32_t N,
                                               uint32_t* status, uint32_t job_block, uint32_t job_blocks, uint32_t row0 = 0,
                                               uint32_t nrows = 0xFFFFFFFFu) {
  constexpr int U = 2;
  WideMove w;
  RowMove& m = w.m;
  w.E = ft.bytes[f];
  m.RS = ft.row_stride;
  m.epr = (w.E + 15u) / 16u;
  m.total = (uint64_t)(nrows < B - row0 ? nrows : B - row0) * m.epr;
  m.col = ft.col[f] + (uint64_t)t * ft.col_stride[f];
  m.io = ft.io[f] + ((uint64_t)t * B + row0) * w.E;
  m.idx = idx ? idx + (size_t)t * B + row0 : nullptr;
  m.stride = (uint64_t)job_blocks * blockDim.x;
  m.cursor = cursor;
  m.N = N;
  bool bad = false;
  for (uint64_t e0 = (uint64_t)job_block * blockDim.x + threadIdx.x; e0 < m.total; e0 += U * m.stride) {
    Regs<uint32_t, U> at;
    Regs<uint4, U> v;
    sweep_where<uint4, GATHER, 0, U>(m, e0, at);
    wide_load<GATHER, 0, U>(w, e0, at, v, bad);
    wide_store<GATHER, 0, U>(w, e0, at, v);
  }
  if (bad) atomicOr(&status[t], 1u);
}

// Rows of several fields gathered whole.  One job per field reads every sampled row once per field, from
// workgroups on different parts of the device, so the row's memory lines are fetched once per field.  Here a
// workgroup takes `whole_rows` sampled rows per pass: the stored bytes that cover all asked-for fields come in
// as 16-byte pieces (up to kWholePieces per lane in flight) and are parked in LDS, row after row; then each
// field's dense span of those rows, which is contiguous in the caller's array, is written from LDS with
// consecutive lanes on consecutive addresses, in 16-byte stores where the span starts on such a boundary.
// `stage` holds whole_rows * whole_span bytes (at most kWholeRowsLds).
constexpr int kWholePieces = 6;
template <int K>
__device__ __forceinline__ void whole_where(uint32_t lane, uint32_t block, uint32_t items, uint32_t P,
                                            const uint32_t* __restrict__ idx, Regs<uint32_t, kWholePieces>& at,
                                            Regs<uint32_t, kWholePieces>& piece) {
  if constexpr (K < kWholePieces) {
    if ((uint32_t)K * block < items) {   // (the same for all lanes: sweeps beyond the pass's pieces are skipped whole)
      const uint32_t i = lane + (uint32_t)K * block;
      const uint32_t r = i < items ? i / P : 0u;
      reg<K>(piece) = i < items ? i - r * P : 0u;
      reg<K>(at) = idx[r];
      whole_where<K + 1>(lane, block, items, P, idx, at, piece);
    }
  }
}
template <int K>
__device__ __forceinline__ void whole_load(uint32_t block, uint32_t items, const uint8_t* base, uint32_t RS, uint32_t N,
                                           Regs<uint32_t, kWholePieces>& at, Regs<uint32_t, kWholePieces>& piece,
                                           Regs<uint4, kWholePieces>& v, bool& bad) {
  if constexpr (K < kWholePieces) {
    if ((uint32_t)K * block < items) {
      const bool ok = reg<K>(at) < N;
      bad |= !ok;
      uint4 got = *reinterpret_cast<const uint4*>(base + (uint64_t)(ok ? reg<K>(at) : 0u) * RS + 16u * reg<K>(piece));
      if (!ok) got = make_uint4(0, 0, 0, 0);
      reg<K>(v) = got;
      whole_load<K + 1>(block, items, base, RS, N, at, piece, v, bad);
    }
  }
}
template <int K>
__device__ __forceinline__ void whole_park(uint32_t lane, uint32_t block, uint32_t items, uint4* stage,
                                           Regs<uint4, kWholePieces>& v) {
  if constexpr (K < kWholePieces) {
    const uint32_t i = lane + (uint32_t)K * block;
    if (i < items) {
      stage[i] = reg<K>(v);
      whole_park<K + 1>(lane, block, items, stage, v);   // (a lane without piece K has none beyond it)
    }
  }
}
__device__ __forceinline__ void move_whole_rows(const FieldTable& ft, const JobRanges& jr, uint32_t t, uint32_t B,
                                                const uint32_t* __restrict__ idx, uint32_t N, uint32_t* status,
                                                uint32_t job_block, uint32_t job_blocks, uint8_t* stage) {
  const uint32_t R = jr.whole_rows, span = jr.whole_span, P = span >> 4;
  const uint32_t f0 = jr.whole_field;
  const uint8_t* first = ft.col[f0] + (uint64_t)t * ft.col_stride[f0];
  const uint8_t* base = first - jr.whole_lead;
  const uint32_t lane = threadIdx.x, block = blockDim.x;
  idx += (size_t)t * B;
  bool bad = false;
  for (uint32_t r0 = job_block * R; r0 < B; r0 += job_blocks * R) {
    const uint32_t rows = B - r0 < R ? B - r0 : R;
    const uint32_t items = rows * P;
    if (r0 != job_block * R) __syncthreads();   // the pass before is done with the staging bytes
    {
      Regs<uint32_t, kWholePieces> at, piece;
      Regs<uint4, kWholePieces> v;
      whole_where<0>(lane, block, items, P, idx + r0, at, piece);
      whole_load<0>(block, items, base, ft.row_stride, N, at, piece, v, bad);
      whole_park<0>(lane, block, items, reinterpret_cast<uint4*>(stage), v);
    }
    __syncthreads();
    for (uint32_t f = 0; f < ft.n_fields; ++f) {
      if (!ft.io[f]) continue;
      const uint32_t E = ft.bytes[f];
      const uint32_t foff = (uint32_t)(ft.col[f] - ft.col[f0]) + jr.whole_lead;
      uint8_t* dst = ft.io[f] + ((uint64_t)t * B + r0) * E;
      const uint32_t S = rows * E;
      if ((E & 3u) == 0 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
        for (uint32_t c = lane; 16u * c < S; c += block) {
          const uint32_t p = 16u * c;
          uint32_t row = p / E, off = p - row * E;
          uint32_t w[4];
#pragma unroll
          for (uint32_t k = 0; k < 4; ++k) {
            w[k] = p + 4u * k < S ? *reinterpret_cast<const uint32_t*>(stage + row * span + foff + off) : 0u;
            off += 4u;
            if (off >= E) {
              off = 0;
              ++row;
            }
          }
          if (p + 16u <= S) {
            *reinterpret_cast<uint4*>(dst + p) = make_uint4(w[0], w[1], w[2], w[3]);
          } else {
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
              if (p + 4u * k < S) *reinterpret_cast<uint32_t*>(dst + p + 4u * k) = w[k];
          }
        }
      } else if ((E & 3u) == 0 && (reinterpret_cast<uintptr_t>(dst) & 3u) == 0) {
        for (uint32_t p = 4u * lane; p < S; p += 4u * block) {
          const uint32_t row = p / E, off = p - row * E;
          *reinterpret_cast<uint32_t*>(dst + p) = *reinterpret_cast<const uint32_t*>(stage + row * span + foff + off);
        }
      } else {
        for (uint32_t p = lane; p < S; p += block) {
          const uint32_t row = p / E, off = p - row * E;
          dst[p] = stage[row * span + foff + off];
        }
      }
    }
  }
  if (bad) atomicOr(&status[t], 1u);
}

// The field whose row job workgroup b of the job grid belongs to (kMaxFields: none).  The ranges lie back to
// back, so it is the number of ranges that end at or before b; written without an early exit so that the
// range ends are read together, not one after the other.
__device__ __forceinline__ uint32_t job_field(const JobRanges& jr, uint32_t b) {
  uint32_t f = 0;
#pragma unroll
  for (uint32_t k = 0; k < (uint32_t)kMaxFields; ++k) f += b >= jr.first[3 + k] ? 1u : 0u;
  return f;
}

// Moves the rows of one payload field; the workgroup is number job_block of job_blocks on that field.
// WIDE: the kernel was built with the 16-byte moves on 4-byte boundaries (see Wide16); the launchers pick
// that build only when a field of the call moves that way, so that calls without one run the smaller code.
template <bool GATHER, bool WIDE>
__device__ __forceinline__ void rows_job(const FieldTable& ft, uint32_t f, uint32_t t, uint32_t B,
                                         const uint32_t* __restrict__ idx, uint32_t cursor, uint32_t N,
                                         uint32_t* status, uint32_t job_block, uint32_t job_blocks, uint32_t row0 = 0,
                                         uint32_t nrows = 0xFFFFFFFFu) {
  switch (ft.vec[f]) {
    case 16: move_rows<uint4, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks, row0, nrows); break;
    case 8: move_rows<uint2, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks, row0, nrows); break;
    case 4:
      if constexpr (WIDE) {
        if (moves_wide(ft.bytes[f], 4)) {
          move_rows_wide<GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks, row0, nrows);
          break;
        }
      }
      move_rows<uint32_t, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks, row0, nrows);
      break;
    case 2: move_rows<uint16_t, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks, row0, nrows); break;
    default: move_rows<uint8_t, GATHER>(ft, f, t, B, idx, cursor, N, status, job_block, job_blocks, row0, nrows); break;
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
    uint8_t* stored = col + slot * ft.row_stride + (uint64_t)k * w;
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

// The rows (and the slot numbers) of an insertion carried by a sampling kernel: the share of mover workgroup
// `part` of `parts` (whole rows; a workgroup moves its share in as few sweeps as it has lanes for).
__device__ __forceinline__ void ride_rows(const InsertRide& ride, uint32_t t, uint32_t N, uint32_t part, uint32_t parts) {
  const uint32_t r0 = (uint32_t)((uint64_t)ride.n * part / parts), r1 = (uint32_t)((uint64_t)ride.n * (part + 1) / parts);
  (void)move_rows_one_workgroup<false>(ride.rows, t, (uint64_t)t * ride.n + r0, r1 - r0, ride.cursor + r0, N, nullptr, nullptr);
  if (ride.out_idx)
    for (uint32_t j = r0 + threadIdx.x; j < r1; j += blockDim.x) ride.out_idx[(size_t)t * ride.n + j] = ride.cursor + j;
}

// Second kernel of the fused calls.  Its workgroups (blockIdx.x) split into jobs, each with as many
// workgroups as it needs (JobRanges): first the importance weights of the batch just sampled (if
// asked for), then the claim phase of a priority update (if one is fused in), then one job per
// payload field of the sampled rows, or a single job over whole rows (move_whole_rows) in the first
// asked-for field's range.  The small jobs come first, so their latency hides behind the row traffic.
template <bool WIDE>
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
  const uint32_t f = job_field(jr, b);
  if (jr.whole_rows) {
    extern __shared__ __attribute__((aligned(16))) uint8_t stage[];
    move_whole_rows(ft, jr, t, a.B, a.idx, g.N, g.status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f], stage);
  } else if (f < (uint32_t)kMaxFields)
    rows_job<true, WIDE>(ft, f, t, a.B, a.idx, 0, g.N, g.status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
}

// Stand-alone gather (GATHER) and insert scatter: one job per payload field (gathers: or one over whole rows).
template <bool GATHER, bool WIDE>
__global__ void k_rows(FieldTable ft, JobRanges jr, uint32_t B, const uint32_t* __restrict__ idx, uint32_t cursor,
                       uint32_t N, uint32_t* status) {
  const uint32_t t = blockIdx.y;
  const uint32_t b = blockIdx.x;
  const uint32_t f = job_field(jr, b);
  if constexpr (GATHER) {
    if (jr.whole_rows) {
      extern __shared__ __attribute__((aligned(16))) uint8_t stage[];
      move_whole_rows(ft, jr, t, B, idx, N, status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f], stage);
      return;
    }
  }
  if (f < (uint32_t)kMaxFields)
    rows_job<GATHER, WIDE>(ft, f, t, B, idx, cursor, N, status, b - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
}

// Workgroups per job: weights, claim, then each field with a destination.  A field gets the workgroups one
// pass over its elements needs with as few elements per lane (1, 2, 4 .. what its mover keeps in flight)
// as keep the field's workgroups over all trees within about one round of the device; the movers
// stride when that is not enough.
// Whether a gather of these fields moves whole rows (see move_whole_rows), and with what shape: at least two
// fields asked for, their common span of a stored row short enough that 16 rows or more fit the staging bytes
// and the pieces a workgroup keeps in flight.  Passes take a multiple of 16 rows, so that every field's dense
// span of a pass starts on a 16-byte boundary when the field's array does.
constexpr uint64_t kWholeRowsFrom = 16384;   // rows of a call (all trees) from which whole rows are the default
static bool plan_whole_rows(const FieldTable* ft, uint32_t block, JobRanges* jr) {
  if (!ft) return false;
  uint32_t asked = 0, f0 = 0;
  const uint8_t* lo = nullptr;
  const uint8_t* hi = nullptr;
  for (uint32_t f = 0; f < ft->n_fields; ++f) {
    if (!ft->io[f]) continue;
    if (!asked || ft->col[f] < lo) lo = ft->col[f], f0 = f;
    if (!asked || ft->col[f] + ft->bytes[f] > hi) hi = ft->col[f] + ft->bytes[f];
    ++asked;
  }
  if (asked < 2) return false;
  const uint32_t lead = (uint32_t)(reinterpret_cast<uintptr_t>(lo) & 15u);
  const uint64_t span = ((uint64_t)(hi - lo) + lead + 15u) / 16u * 16u;
  if (span > ft->row_stride || span > kWholeRowsLds / 16u) return false;
  uint32_t R = (uint32_t)kWholePieces * block / (uint32_t)(span / 16u);
  if (R > kWholeRowsLds / (uint32_t)span) R = kWholeRowsLds / (uint32_t)span;
  R = R / 16u * 16u;
  if (R > 64u) R = 64u;
  if (R < 16u) return false;
  jr->whole_rows = R;
  jr->whole_span = (uint32_t)span;
  jr->whole_field = f0;
  jr->whole_lead = lead;
  return true;
}

static JobRanges job_ranges(const FieldTable* ft, uint32_t rows, uint32_t block, uint32_t weights_B, uint32_t claim_B,
                            uint32_t trees, uint32_t whole_rows = 0) {
  JobRanges jr{};
  uint32_t at = 0;
  jr.first[0] = at;
  at += (weights_B + block - 1) / block;
  jr.first[1] = at;
  at += (claim_B + block - 1) / block;
  jr.first[2] = at;
  // (whole_rows: 0 never, 1 for batches long enough that the row traffic sets the time, 2 wherever the rows fit)
  const bool whole = (whole_rows == 2 || (whole_rows == 1 && (uint64_t)rows * trees >= kWholeRowsFrom)) &&
                     plan_whole_rows(ft, block, &jr);
  for (uint32_t f = 0; f < (uint32_t)kMaxFields; ++f) {
    if (whole) {
      if (f == jr.whole_field) {
        uint64_t n = ((uint64_t)rows + jr.whole_rows - 1) / jr.whole_rows;
        if (n > (1u << 20)) n = 1u << 20;
        at += (uint32_t)n;
      }
    } else if (ft && f < ft->n_fields && ft->io[f]) {
      const uint64_t elems = (uint64_t)rows * row_elements(ft->bytes[f], ft->vec[f]);
      const uint32_t most = field_in_flight(ft->bytes[f], ft->vec[f]);
      uint64_t n = 0;
      for (uint32_t per_lane = 1; per_lane <= most; per_lane *= 2) {
        n = (elems + (uint64_t)per_lane * block - 1) / ((uint64_t)per_lane * block);
        if (n * trees <= 512) break;
      }
      if (n > (1u << 20)) n = 1u << 20;
      at += (uint32_t)n;
    }
    jr.first[3 + f] = at;
  }
  return jr;
}

// staging bytes of the workgroups of a launch with these job ranges
static size_t whole_rows_lds(const JobRanges& jr) { return (size_t)jr.whole_rows * jr.whole_span; }

// true when a field of the call moves in 16-byte pieces on 4-byte boundaries
static bool any_field_moves_wide(const FieldTable* ft) {
  for (uint32_t f = 0; ft && f < ft->n_fields; ++f)
    if (ft->io[f] && moves_wide(ft->bytes[f], ft->vec[f])) return true;
  return false;
}

hipError_t launch_gather(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t B, const uint32_t* idx,
                         hipStream_t s) {
  const uint32_t block = tn.gather_block;
  const JobRanges jr = job_ranges(&ft, B, block, 0, 0, g.T, tn.whole_rows);
  const uint32_t gx = jr.first[2 + kMaxFields];
  if (gx == 0) return hipSuccess;
  const size_t lds = whole_rows_lds(jr);
  if (!jr.whole_rows && any_field_moves_wide(&ft)) {
    PER_LAUNCH(KID_GATHER, (k_rows<true, true>), dim3(gx, g.T), dim3(block), lds, s, ft, jr, B, idx, 0, g.N, g.status);
  } else {
    PER_LAUNCH(KID_GATHER, (k_rows<true, false>), dim3(gx, g.T), dim3(block), lds, s, ft, jr, B, idx, 0, g.N, g.status);
  }
  return hipGetLastError();
}

static hipError_t launch_finish(const Geom& g, const Tuning& tn, const FieldTable* rows, const FinishArgs& a,
                                hipStream_t s) {
  FieldTable ft{};
  if (rows) ft = *rows;
  if (!a.w && !a.has_claim) return rows ? launch_gather(g, tn, ft, a.B, a.idx, s) : hipSuccess;
  const uint32_t block = tn.gather_block;
  const JobRanges jr = job_ranges(rows ? &ft : nullptr, a.B, block, a.w ? a.B : 0u, a.has_claim ? a.claim.B : 0u, g.T,
                                  tn.whole_rows);
  const size_t lds = whole_rows_lds(jr);
  if (!jr.whole_rows && any_field_moves_wide(rows ? &ft : nullptr)) {
    PER_LAUNCH(KID_FINISH, k_finish<true>, dim3(jr.first[2 + kMaxFields], g.T), dim3(block), lds, s, ft, jr, g, a);
  } else {
    PER_LAUNCH(KID_FINISH, k_finish<false>, dim3(jr.first[2 + kMaxFields], g.T), dim3(block), lds, s, ft, jr, g, a);
  }
  return hipGetLastError();
}

hipError_t launch_scatter(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t n, uint32_t cursor,
                          hipStream_t s) {
  const uint32_t block = tn.gather_block;
  const JobRanges jr = job_ranges(&ft, n, block, 0, 0, g.T);
  const uint32_t gx = jr.first[2 + kMaxFields];
  if (gx == 0) return hipSuccess;
  if (any_field_moves_wide(&ft)) {
    PER_LAUNCH(KID_SCATTER, (k_rows<false, true>), dim3(gx, g.T), dim3(block), 0, s, ft, jr, n, nullptr, cursor, g.N, g.status);
  } else {
    PER_LAUNCH(KID_SCATTER, (k_rows<false, false>), dim3(gx, g.T), dim3(block), 0, s, ft, jr, n, nullptr, cursor, g.N, g.status);
  }
  return hipGetLastError();
}
