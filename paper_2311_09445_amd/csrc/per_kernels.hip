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

namespace per {

// ---------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------
template <int LOGK>
struct Fan {
  static constexpr int K = 1 << LOGK;
  static constexpr int LPS = K >= 4 ? K / 4 : 1;          // lanes per child group
  static constexpr int LOGLPS = LOGK >= 2 ? LOGK - 2 : 0;
};

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

// One K-ary level of the prefix-sum traversal (Section V-A "traversing the tree
// performing prefix sum from root to leaf"), as log2(K) binary steps:
//   go right iff the right block is non-zero and not (r < left block); then r -= left.
// On return all lanes of the group hold the chosen child, its value and the residual.
template <int LOGK>
__device__ __forceinline__ void descend_group(const float* grp, unsigned q, unsigned lane, float& r,
                                              unsigned& child, float& val) {
  if constexpr (LOGK == 1) {
    const float2 c = *reinterpret_cast<const float2*>(grp);
    const bool right = (c.y != 0.0f) && !(r < c.x);
    r = right ? r - c.x : r;
    child = right ? 1u : 0u;
    val = right ? c.y : c.x;
  } else {
    constexpr int LOGLPS = Fan<LOGK>::LOGLPS;
    constexpr int LPS = Fan<LOGK>::LPS;
    const float4 c = *reinterpret_cast<const float4*>(grp + 4 * q);
    const float p0 = c.x + c.y, p1 = c.z + c.w;
    float mine[LOGLPS + 1];
    float sib[LOGLPS + 1];
    mine[0] = p0 + p1;
#pragma unroll
    for (int k = 0; k < LOGLPS; ++k) {
      sib[k] = __shfl_xor(mine[k], 1 << k);
      mine[k + 1] = mine[k] + sib[k];
    }
    // Walk the blocks of 4*2^k children from the top.  A lane stays "on path" while the
    // decisions match its own position bits; exactly one lane of the group stays on path,
    // and up to that point it has seen the true left/right sums and residual.
    float rr = r;
    bool on = true;
#pragma unroll
    for (int k = LOGLPS - 1; k >= 0; --k) {
      const bool bit = (q >> k) & 1u;
      const float L = bit ? sib[k] : mine[k];
      const float R = bit ? mine[k] : sib[k];
      const bool right = (R != 0.0f) && !(rr < L);
      rr = right ? rr - L : rr;
      on = on && (right == bit);
    }
    // last two binary steps inside this lane's four children
    const bool r1 = (p1 != 0.0f) && !(rr < p0);
    rr = r1 ? rr - p0 : rr;
    const float a = r1 ? c.z : c.x, b = r1 ? c.w : c.y;
    const bool r0 = (b != 0.0f) && !(rr < a);
    rr = r0 ? rr - a : rr;
    float v = r0 ? b : a;
    unsigned ch = 4u * q + (r1 ? 2u : 0u) + (r0 ? 1u : 0u);
    if constexpr (LPS > 1) {
      const unsigned long long m = __ballot(on);
      const unsigned base = lane & ~(unsigned)(LPS - 1);
      const unsigned bits = (unsigned)(m >> base) & ((1u << LPS) - 1u);
      const int src = (int)base + (__ffs((int)bits) - 1);
      rr = __shfl(rr, src);
      v = __shfl(v, src);
      ch = (unsigned)__shfl((int)ch, src);
    }
    r = rr;
    child = ch;
    val = v;
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

hipError_t launch_fill_u32(uint32_t* p, uint64_t count, uint32_t value, hipStream_t s) {
  if (count == 0) return hipSuccess;
  uint64_t blocks = (count / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 16384) blocks = 16384;
  k_fill_u32<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(p, count, value);
  return hipGetLastError();
}

__global__ void k_init_scalars(Geom g, float init_max) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= g.T) return;
  g.max_v[t] = init_max;
  g.status[t] = 0;
  g.vmin[t] = 0x7F800000u;
  g.vmin[g.T + t] = 0x7F800000u;
}

hipError_t launch_init_scalars(const Geom& g, float init_max, hipStream_t s) {
  k_init_scalars<<<dim3((g.T + 63) / 64), dim3(64), 0, s>>>(g, init_max);
  return hipGetLastError();
}

// which: 0 = root of every tree, 1 = running max priority
__global__ void k_read_scalars(Geom g, int which, float* out) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= g.T) return;
  out[t] = which == 0 ? g.level[g.H][(size_t)t * g.stride[g.H]] : g.max_v[t];
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
// priority sampling
// ---------------------------------------------------------------------------------
// grid (ceil(B*LPS / block), T).  Heights h_lds .. H-1 of the block's tree are staged in
// LDS first; lower heights are read from memory, one coalesced group per sample and level.
template <int LOGK>
__global__ void k_sample(Geom g, uint32_t B, const float* __restrict__ u, uint32_t* __restrict__ out_idx,
                         float* __restrict__ out_prio, float* __restrict__ out_w, uint32_t parity,
                         uint32_t h_lds) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  extern __shared__ float lds[];
  const uint32_t t = blockIdx.y;
  const uint32_t H = g.H;

  if (h_lds < H) {
    uint32_t off = 0;
    for (int l = (int)H - 1; l >= (int)h_lds; --l) {
      const uint32_t cnt = g.n[l + 1] * (uint32_t)K;
      const float* src = g.level[l] + (size_t)t * g.stride[l];
      if constexpr (LOGK >= 2) {
        const float4* s4 = reinterpret_cast<const float4*>(src);
        float4* d4 = reinterpret_cast<float4*>(lds + off);
        for (uint32_t i = threadIdx.x; i < cnt / 4; i += blockDim.x) d4[i] = s4[i];
      } else {
        for (uint32_t i = threadIdx.x; i < cnt; i += blockDim.x) lds[off + i] = src[i];
      }
      off += cnt;
    }
    __syncthreads();
  }

  const uint32_t gt = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t s_raw = gt / LPS;
  const unsigned q = gt % LPS;
  const unsigned lane = threadIdx.x & 63u;
  const bool active = s_raw < B;
  const uint32_t s = active ? s_raw : B - 1;
  const size_t o = (size_t)t * B + s;

  const float total = g.level[H][(size_t)t * g.stride[H]];
  if (blockIdx.x == 0 && threadIdx.x == 0 && out_w) g.vmin[(parity ^ 1u) * g.T + t] = 0x7F800000u;
  if (!(total > 0.0f)) {   // nothing can be sampled from this tree
    if (active && q == 0) {
      out_idx[o] = 0xFFFFFFFFu;
      if (out_prio) out_prio[o] = 0.0f;
      if (out_w) out_w[o] = 0.0f;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&g.status[t], 4u);
    return;
  }

  const float seg = total / (float)B;
  const float pos = (float)s + u[o];
  float r = pos * seg;

  uint32_t node = 0;
  float val = total;
  uint32_t off = 0;
  for (int l = (int)H - 1; l >= 0; --l) {
    unsigned child;
    if ((uint32_t)l >= h_lds) {
      descend_group<LOGK>(lds + off + (size_t)node * K, q, lane, r, child, val);
      off += g.n[l + 1] * (uint32_t)K;
    } else {
      descend_group<LOGK>(g.level[l] + (size_t)t * g.stride[l] + (size_t)node * K, q, lane, r, child, val);
    }
    node = node * K + child;
  }

  if (active && q == 0) {
    out_idx[o] = node;
    if (out_prio) out_prio[o] = val;
    if (out_w) out_w[o] = val;   // turned into the weight by k_weights
  }
  if (out_w) {
    const uint32_t m = wave_min_u32(active ? __float_as_uint(val) : 0x7F800000u);
    if (lane == 0) atomicMin(&g.vmin[parity * g.T + t], m);
  }
}

// Importance weights (prioritized experience replay, cited in Section II-A):
// w_i = (size * v_i / total)^-beta / max_j(...), the maximum being reached at the batch
// minimum of v.  fp64 so that the result stays within 1e-6 of an fp64 reference.
__global__ void k_weights(Geom g, uint32_t B, uint32_t size, float beta, float* __restrict__ w, uint32_t parity) {
  const uint32_t t = blockIdx.y;
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  const float total = g.level[g.H][(size_t)t * g.stride[g.H]];
  const size_t o = (size_t)t * B + i;
  if (!(total > 0.0f)) { w[o] = 0.0f; return; }
  const double nb = -(double)beta;
  const double scale = (double)size / (double)total;
  const double vmin = (double)__uint_as_float(g.vmin[parity * g.T + t]);
  const double wt = pow(scale * (double)w[o], nb);
  const double wm = pow(scale * vmin, nb);
  w[o] = (float)(wt / wm);
}

template <int LOGK>
static hipError_t launch_sample_k(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, float beta,
                                  const float* u, uint32_t* out_idx, float* out_w, float* out_prio,
                                  uint32_t parity, hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  // lowest height whose levels (that height and all above, below the root) fit the LDS budget
  uint32_t h_lds = g.H;
  uint64_t bytes = 0;
  for (int l = (int)g.H - 1; l >= 0; --l) {
    const uint64_t add = (uint64_t)g.n[l + 1] * K * 4;
    if (bytes + add > tn.lds_budget_bytes) break;
    bytes += add;
    h_lds = (uint32_t)l;
  }
  const uint32_t block = tn.sample_block;
  const uint64_t threads = (uint64_t)B * LPS;
  const uint32_t gx = (uint32_t)((threads + block - 1) / block);
  hipError_t e;
  if (bytes > 64 * 1024) {   // more than the default dynamic LDS limit has to be requested per kernel
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_sample<LOGK>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
  }
  k_sample<LOGK><<<dim3(gx, g.T), dim3(block), (size_t)bytes, s>>>(g, B, u, out_idx, out_prio, out_w, parity, h_lds);
  e = hipGetLastError();
  if (e != hipSuccess || !out_w) return e;
  k_weights<<<dim3((B + 255) / 256, g.T), dim3(256), 0, s>>>(g, B, size, beta, out_w, parity);
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
                         uint32_t* out_idx, float* out_w, float* out_prio, uint32_t parity, hipStream_t s) {
#define CALL(L) launch_sample_k<L>(g, tn, B, size, beta, u, out_idx, out_w, out_prio, parity, s)
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
                                          uint32_t* status) {
  const uint32_t E = ft.bytes[f];
  const uint32_t epr = E / (uint32_t)sizeof(V);
  const uint64_t total = (uint64_t)B * epr;
  uint8_t* col = ft.col[f] + (uint64_t)t * ft.col_stride[f];
  uint8_t* io = ft.io[f] + (uint64_t)t * B * E;
  bool bad = false;
  for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (uint64_t)gridDim.x * blockDim.x) {
    const uint32_t row = (uint32_t)(e / epr);
    const uint32_t k = (uint32_t)(e - (uint64_t)row * epr);
    V* dense = reinterpret_cast<V*>(io + (uint64_t)row * E) + k;
    if constexpr (GATHER) {
      const uint32_t i = idx[(size_t)t * B + row];
      if (i < N) {
        *dense = *(reinterpret_cast<const V*>(col + (uint64_t)i * E) + k);
      } else {
        V z;
        __builtin_memset(&z, 0, sizeof(V));
        *dense = z;
        bad = true;
      }
    } else {
      uint64_t slot = (uint64_t)cursor + row;
      if (slot >= N) slot -= N;
      *(reinterpret_cast<V*>(col + slot * E) + k) = *dense;
    }
  }
  if (bad) atomicOr(&status[t], 1u);
}

template <bool GATHER>
__global__ void k_rows(FieldTable ft, uint32_t B, const uint32_t* __restrict__ idx, uint32_t cursor, uint32_t N,
                       uint32_t* status) {
  const uint32_t f = blockIdx.y, t = blockIdx.z;
  if (ft.io[f] == nullptr) return;
  switch (ft.vec[f]) {
    case 16: move_rows<uint4, GATHER>(ft, f, t, B, idx, cursor, N, status); break;
    case 8: move_rows<uint2, GATHER>(ft, f, t, B, idx, cursor, N, status); break;
    case 4: move_rows<uint32_t, GATHER>(ft, f, t, B, idx, cursor, N, status); break;
    case 2: move_rows<uint16_t, GATHER>(ft, f, t, B, idx, cursor, N, status); break;
    default: move_rows<uint8_t, GATHER>(ft, f, t, B, idx, cursor, N, status); break;
  }
}

static uint32_t rows_grid_x(const FieldTable& ft, uint32_t B, uint32_t block) {
  uint64_t most = 1;
  for (uint32_t f = 0; f < ft.n_fields; ++f) {
    if (!ft.io[f]) continue;
    const uint64_t e = (uint64_t)B * (ft.bytes[f] / ft.vec[f]);
    if (e > most) most = e;
  }
  uint64_t gx = (most + block - 1) / block;
  if (gx > 65535u * 16u) gx = 65535u * 16u;
  return (uint32_t)gx;
}

hipError_t launch_gather(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t B, const uint32_t* idx,
                         hipStream_t s) {
  if (ft.n_fields == 0) return hipSuccess;
  const uint32_t block = tn.gather_block;
  k_rows<true><<<dim3(rows_grid_x(ft, B, block), ft.n_fields, g.T), dim3(block), 0, s>>>(ft, B, idx, 0, g.N, g.status);
  return hipGetLastError();
}

hipError_t launch_scatter(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t n, uint32_t cursor,
                          hipStream_t s) {
  if (ft.n_fields == 0) return hipSuccess;
  const uint32_t block = tn.gather_block;
  k_rows<false><<<dim3(rows_grid_x(ft, n, block), ft.n_fields, g.T), dim3(block), 0, s>>>(ft, n, nullptr, cursor, g.N, g.status);
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

// Recompute, for every valid update element, its ancestor at height h.  Duplicated
// ancestors are recomputed to the same bits by several groups, which is harmless.
template <int LOGK>
__global__ void k_resum_sparse(Geom g, uint32_t h, uint32_t B, uint32_t size, const uint32_t* __restrict__ idx,
                               const float* __restrict__ prio) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t t = blockIdx.y;
  const uint32_t gt = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t e = gt / LPS;
  const unsigned q = gt % LPS;
  const uint32_t ec = e < B ? e : B - 1;
  const uint32_t i = idx[(size_t)t * B + ec];
  const bool ok = e < B && i < size && valid_priority(prio[(size_t)t * B + ec]);
  const uint32_t node = ok ? shr64(i, h * LOGK) : 0u;
  const float sum = group_sum<LOGK>(g.level[h - 1] + (size_t)t * g.stride[h - 1] + (size_t)node * K, q);
  if (ok && q == 0) g.level[h][(size_t)t * g.stride[h] + node] = sum;
}

// One workgroup per tree finishes heights h_start .. H.  Heights <= sparse_hi are done per
// update element (idx != null), the others densely over the node ranges in r (given at
// height h_start and narrowed by K per height).
template <int LOGK>
__global__ void k_resum_tail(Geom g, uint32_t h_start, Range2 r, const uint32_t* __restrict__ idx,
                             const float* __restrict__ prio, uint32_t B, uint32_t size, uint32_t sparse_hi) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t t = blockIdx.x;
  const unsigned q = threadIdx.x % LPS;
  const uint32_t grp = threadIdx.x / LPS;
  const uint32_t ngrp = blockDim.x / LPS;
  for (uint32_t h = h_start; h <= g.H; ++h) {
    const float* child = g.level[h - 1] + (size_t)t * g.stride[h - 1];
    float* par = g.level[h] + (size_t)t * g.stride[h];
    if (idx != nullptr && h <= sparse_hi) {
      for (uint32_t base = 0; base < B; base += ngrp) {
        const uint32_t e = base + grp;
        const uint32_t ec = e < B ? e : B - 1;
        const uint32_t i = idx[(size_t)t * B + ec];
        const bool ok = e < B && i < size && valid_priority(prio[(size_t)t * B + ec]);
        const uint32_t node = ok ? shr64(i, h * LOGK) : 0u;
        const float sum = group_sum<LOGK>(child + (size_t)node * K, q);
        if (ok && q == 0) par[node] = sum;
      }
    } else {
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
      k_resum_dense<LOGK><<<dim3((uint32_t)((threads + block - 1) / block), g.T), dim3(block), 0, s>>>(g, h, a, b - a);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  if (h <= g.H) {
    k_resum_tail<LOGK><<<dim3(g.T), dim3(1024), 0, s>>>(g, h, r, nullptr, nullptr, 0, 0, 0);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t launch_resum_ranges(const Geom& g, const Tuning& tn, Range2 r0, hipStream_t s) {
#define CALL(L) launch_resum_ranges_k<L>(g, tn, r0, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}

// ---------------------------------------------------------------------------------
// insertion: leaf writes (rows go through k_rows<false>)
// ---------------------------------------------------------------------------------
__global__ void k_insert_leaves(Geom g, uint32_t n, uint32_t cursor, const float* __restrict__ prio,
                                uint32_t* __restrict__ out_idx) {
  const uint32_t t = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  const bool active = j < n;
  uint32_t mx = 0;
  bool bad = false;
  if (active) {
    uint64_t slot = (uint64_t)cursor + j;
    if (slot >= g.N) slot -= g.N;
    if (out_idx) out_idx[(size_t)t * n + j] = (uint32_t)slot;
    float* leaf = g.level[0] + (size_t)t * g.stride[0] + slot;
    if (prio) {
      const float v = prio[(size_t)t * n + j];
      if (valid_priority(v)) {
        *leaf = v;
        mx = v > 0.0f ? __float_as_uint(v) : 0u;
      } else {
        bad = true;
      }
    } else {
      *leaf = g.max_v[t];   // running maximum as it was when the call started
    }
  }
  if (prio) {
    mx = wave_max_u32(mx);
    if ((threadIdx.x & 63u) == 0 && mx != 0) atomicMax(reinterpret_cast<uint32_t*>(&g.max_v[t]), mx);
    if (bad) atomicOr(&g.status[t], 2u);
  }
}

hipError_t launch_insert_leaves(const Geom& g, const Tuning& tn, uint32_t n, uint32_t cursor, const float* prio,
                                uint32_t* out_idx, hipStream_t s) {
  (void)tn;
  k_insert_leaves<<<dim3((n + 255) / 256, g.T), dim3(256), 0, s>>>(g, n, cursor, prio, out_idx);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// priority update: claim (last writer), leaf write, re-summation
// ---------------------------------------------------------------------------------
// Element j stamps its leaf with stamp_base + j by atomic max.  Stamps grow from call to
// call, so stale stamps never win and the array needs no clearing between calls.
__global__ void k_update_claim(Geom g, uint32_t B, uint32_t size, const uint32_t* __restrict__ idx,
                               const float* __restrict__ prio, uint32_t stamp_base) {
  const uint32_t t = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t mx = 0;
  uint32_t flags = 0;
  if (j < B) {
    const uint32_t i = idx[(size_t)t * B + j];
    const float v = prio[(size_t)t * B + j];
    if (!(i < size)) flags = 1u;
    else if (!valid_priority(v)) flags = 2u;
    else {
      atomicMax(&g.owner[(size_t)t * g.owner_stride + i], stamp_base + j);
      mx = v > 0.0f ? __float_as_uint(v) : 0u;
    }
  }
  mx = wave_max_u32(mx);
  if ((threadIdx.x & 63u) == 0 && mx != 0) atomicMax(reinterpret_cast<uint32_t*>(&g.max_v[t]), mx);
  if (flags) atomicOr(&g.status[t], flags);
}

__global__ void k_update_write(Geom g, uint32_t B, uint32_t size, const uint32_t* __restrict__ idx,
                               const float* __restrict__ prio, uint32_t stamp_base) {
  const uint32_t t = blockIdx.y;
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= B) return;
  const uint32_t i = idx[(size_t)t * B + j];
  const float v = prio[(size_t)t * B + j];
  if (i < size && valid_priority(v) && g.owner[(size_t)t * g.owner_stride + i] == stamp_base + j)
    g.level[0][(size_t)t * g.stride[0] + i] = v;
}

template <int LOGK>
static hipError_t launch_update_k(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, const uint32_t* idx,
                                  const float* prio, uint32_t stamp_base, hipStream_t s) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t block = tn.update_block;
  hipError_t e;
  k_update_claim<<<dim3((B + block - 1) / block, g.T), dim3(block), 0, s>>>(g, B, size, idx, prio, stamp_base);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  k_update_write<<<dim3((B + block - 1) / block, g.T), dim3(block), 0, s>>>(g, B, size, idx, prio, stamp_base);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  // heights with fewer update elements than nodes are re-summed per element, the rest densely
  uint32_t sparse_hi = 0;
  for (uint32_t h = 1; h <= g.H; ++h)
    if (B < g.n[h]) sparse_hi = h;
  uint32_t h = 1;
  for (; h <= g.H; ++h) {
    const bool sparse = h <= sparse_hi;
    const uint64_t groups = sparse ? B : g.n[h];
    if (groups * K <= kTailFloats) break;
    const uint64_t threads = groups * LPS;
    const dim3 grid((uint32_t)((threads + block - 1) / block), g.T);
    if (sparse) k_resum_sparse<LOGK><<<grid, dim3(block), 0, s>>>(g, h, B, size, idx, prio);
    else k_resum_dense<LOGK><<<grid, dim3(block), 0, s>>>(g, h, 0, g.n[h]);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (h <= g.H) {
    Range2 r{0, g.n[h], 0, 0};
    k_resum_tail<LOGK><<<dim3(g.T), dim3(1024), 0, s>>>(g, h, r, idx, prio, B, size, sparse_hi);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t launch_update(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, const uint32_t* idx,
                         const float* prio, uint32_t stamp_base, hipStream_t s) {
#define CALL(L) launch_update_k<L>(g, tn, B, size, idx, prio, stamp_base, s)
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

hipError_t launch_get_priority(const Geom& g, uint32_t n, const uint32_t* idx, float* out, hipStream_t s) {
  k_get_priority<<<dim3((n + 255) / 256, g.T), dim3(256), 0, s>>>(g, n, idx, out);
  return hipGetLastError();
}

}  // namespace per
