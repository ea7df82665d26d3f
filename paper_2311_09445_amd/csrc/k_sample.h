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
//
// RIDE: the kernel carries the insertion that precedes the sampling call (a few rows at ring slots cursor ..).
// Every sampling workgroup works the insertion out for itself: beside the top copy it fetches the child groups
// of all touched nodes of heights 1 .. hp (hp: the height the stale top is rebuilt from) and the new priorities
// of the leaves among them, sums the groups height by height, patches the sums into the top copy and rebuilds
// the top from there; on its way down through memory a lane that comes to a touched group reads the patched
// copy instead.  One more workgroup per tree, the last of the grid, does the same sums and stores them and the
// new leaves, and moves the rows (nothing here reads rows).  Its stores race with the other workgroups' loads
// of the same words, harmlessly: every word it writes is one that every reader replaces by the very value being
// written, so a reader gets the same result from the old word and from the new one.  The running maximum must
// not move while this kernel reads it as the inserted priority, so whatever would raise it here (claim lanes,
// given insert priorities) raises max_pend instead, which the tree pass of the call folds in.
// A single wave's chain of instructions is what a small batch waits for, so the patch is planned on the host
// down to LDS offsets, and the kernel's share is kept short.
struct NoRide { uint32_t none; };
// position of node among the touched nodes of its height (the two ranges back to back)
__device__ __forceinline__ uint32_t plan_pos(const Range2& r, uint32_t node) {
  return node >= r.a0 && node < r.b0 ? node - r.a0 : (r.b0 - r.a0) + (node - r.a1);
}
template <bool RIDE> using RideParam = typename std::conditional<RIDE, InsertRide, NoRide>::type;
__device__ __forceinline__ void ride_rows(const InsertRide& ride, uint32_t t, uint32_t N, uint32_t part, uint32_t parts);   // (k_rows.h)

template <int LOGK, bool RIDE>
__global__ void __launch_bounds__(1024)
k_sample(Geom g, TopCopy tc, uint32_t B, uint32_t size, float beta, const float* __restrict__ u,
         uint32_t* __restrict__ out_idx, float* __restrict__ out_prio, float* __restrict__ out_w,
         uint32_t weight_mode, int stale, uint32_t claim_blocks, ClaimArgs c, int claim_mode, RngArgs rng,
         RideParam<RIDE> ride) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  constexpr int ROW = K + 4;                  // staging row, floats
  using Vec = typename std::conditional<LOGK == 1, float2, float4>::type;
  constexpr int VF = sizeof(Vec) / 4;
  // (lines 1, 3, 6, 7, 10, 11 of the geometry hold what this kernel does not read on trees of few heights: the upper
  // ends of the per-height arrays, the arrival counters, the one-kernel step's words)
  touch_kernel_arguments<kernarg_lines<Geom, TopCopy, uint32_t, uint32_t, float, const float*, uint32_t*, float*, float*, uint32_t,
                                       int, uint32_t, ClaimArgs, int, RngArgs,
                                       typename std::conditional<RIDE, InsertRideHead, NoRide>::type>(),
                         LOGK >= 3 ? 0xCCAu : 0u>();
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
  bool is_mover = false;
  uint32_t movers = 0;
  if constexpr (RIDE) {   // the last workgroups move the rows; the first of them also stores what the insertion changes in the tree
    movers = ride.movers;
    const uint32_t first_mover = gridDim.x - movers;
    if (blockIdx.x > first_mover) {
      ride_rows(ride, t, g.N, blockIdx.x - first_mover, movers);
      return;
    }
    is_mover = blockIdx.x == first_mover;
  }
  const uint32_t bx = blockIdx.x - claim_blocks;            // sampling workgroup number
  const uint32_t sample_blocks = gridDim.x - claim_blocks - movers;

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
  // the carried insertion's LDS: behind the top copy and the waves' staging rows
  float* rl = lds + top_floats + (LOGK >= 3 ? (size_t)(blockDim.x >> 6) * 64 * ROW : (size_t)0);
  // Everything it reads is fetched in the trip of the top copy: the loads are issued here, into registers, and
  // parked in LDS once the top copy's own loads are under way (a store to LDS waits for its data).  Lane i takes
  // element i of each height's run of child groups.  A staged leaf that the insertion rewrites is replaced as it
  // is parked (by a valid new priority only).  The plan of all heights comes in one batch of scalar loads and
  // stays in registers: a single wave's chain of instructions and scalar fetches is what a small batch waits for.
  // (plain words, not structures: the compiler keeps structures that lambdas take by reference in memory)
  [[maybe_unused]] uint32_t a1 = 0, c1 = 0, o1 = 0, t1 = 0, a2 = 0, c2 = 0, o2 = 0, t2 = 0, a3 = 0, c3 = 0, o3 = 0, t3 = 0,
                            a4 = 0, c4 = 0, o4 = 0, t4 = 0;   // a: first touched node, c: how many, o: LDS offset, t: top-copy offset
  [[maybe_unused]] float rv1 = 0, rv2 = 0, rv3 = 0, rv4 = 0;
  [[maybe_unused]] float nv1 = -1.0f;   // new priority of this lane's leaf (invalid: the leaf stays)
  static_assert(kRideHeights == 4, "one register per height");
  if constexpr (RIDE) {
    // (first nodes and LDS offsets follow from the lowest height's: fewer words to hold)
    a1 = ride.h[0].a0; c1 = ride.h[0].cnt; t1 = ride.h[0].top_at;
    c2 = ride.h[1].cnt; t2 = ride.h[1].top_at;
    c3 = ride.h[2].cnt; t3 = ride.h[2].top_at;
    c4 = ride.h[3].cnt; t4 = ride.h[3].top_at;
    a2 = a1 >> LOGK; a3 = a2 >> LOGK; a4 = a3 >> LOGK;
    o1 = 0; o2 = c1 * K; o3 = o2 + c2 * K; o4 = o3 + c3 * K;
    if (threadIdx.x < c1 * K) rv1 = g.level[0][(size_t)t * g.stride[0] + (size_t)a1 * K + threadIdx.x];
    if (threadIdx.x < c2 * K) rv2 = g.level[1][(size_t)t * g.stride[1] + (size_t)a2 * K + threadIdx.x];
    if (threadIdx.x < c3 * K) rv3 = g.level[2][(size_t)t * g.stride[2] + (size_t)a3 * K + threadIdx.x];
    if (threadIdx.x < c4 * K) rv4 = g.level[3][(size_t)t * g.stride[3] + (size_t)a4 * K + threadIdx.x];
    const uint32_t j = a1 * K + threadIdx.x - ride.cursor;   // (slots below the cursor wrap to large numbers)
    if (threadIdx.x < c1 * K && j < ride.n) nv1 = ride.prio ? ride.prio[(size_t)t * ride.n + j] : g.max_v[t];
  }
  auto park_ride = [&]() {
    if constexpr (RIDE) {
      if (threadIdx.x < c1 * K) rl[o1 + threadIdx.x] = valid_priority(nv1) ? nv1 : rv1;
      if (threadIdx.x < c2 * K) rl[o2 + threadIdx.x] = rv2;
      if (threadIdx.x < c3 * K) rl[o3 + threadIdx.x] = rv3;
      if (threadIdx.x < c4 * K) rl[o4 + threadIdx.x] = rv4;
    }
  };

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
    park_ride();
    __syncthreads();
    PER_MARK(1);
    if constexpr (RIDE) {
      PER_MARK(13);
      // the touched nodes height by height: sums of the staged groups, into the groups of the height above,
      // into the top copy where the height is part of it, and (last workgroup) aside for the stores
      const unsigned q = threadIdx.x % LPS;
      const uint32_t grp = threadIdx.x / LPS, ngrp = blockDim.x / LPS;
      // (a, c, o, top: the height's touched nodes; up_a, up_o: those of the height above, if it is patched too)
      auto sum_height = [&](uint32_t a, uint32_t cn, uint32_t o, uint32_t top, bool has_up, uint32_t up_a, uint32_t up_o) {
        for (uint32_t base = 0; base < cn; base += ngrp) {
          const uint32_t at = base + grp;
          const bool ok = at < cn;
          const float sum = group_sum<LOGK>(rl + o + (size_t)(ok ? at : 0u) * K, q);
          if (ok && q == 0) {
            const uint32_t nd = a + at;
            if (is_mover) rl[ride.val_off + (o >> LOGK) + at] = sum;
            if (has_up) rl[up_o + (nd - up_a * K)] = sum;
            if (top != kRideNone) lds[top + nd] = sum;
          }
        }
        __syncthreads();
      };
      const uint32_t hp = ride.hp;
      // One touched node per height (the rows lie under one height-1 node: the usual case of a few rows): one lane
      // group works its way up by itself, each sum patched into the staged group of the height above and read back
      // by the same wave, with no workgroup barrier between the heights.
      const bool chain = c1 == 1 && (hp < 2 || c2 == 1) && (hp < 3 || c3 == 1) && (hp < 4 || c4 == 1);
      if (chain) {
        if (threadIdx.x < (uint32_t)LPS) {
          auto one = [&](uint32_t a, uint32_t o, uint32_t top, bool has_up, uint32_t up_a, uint32_t up_o) {
            const float sum = group_sum<LOGK>(rl + o, q);
            if (q == 0) {
              if (is_mover) rl[ride.val_off + (o >> LOGK)] = sum;
              if (has_up) rl[up_o + (a - up_a * K)] = sum;
              if (top != kRideNone) lds[top + a] = sum;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          };
          one(a1, o1, t1, hp > 1, a2, o2);
          if (hp > 1) one(a2, o2, t2, hp > 2, a3, o3);
          if (hp > 2) one(a3, o3, t3, hp > 3, a4, o4);
          if (hp > 3) one(a4, o4, t4, false, 0, 0);
        }
        __syncthreads();
      } else {
        sum_height(a1, c1, o1, t1, hp > 1, a2, o2);
        if (hp > 1) sum_height(a2, c2, o2, t2, hp > 2, a3, o3);
        if (hp > 2) sum_height(a3, c3, o3, t3, hp > 3, a4, o4);
        if (hp > 3) sum_height(a4, c4, o4, t4, false, 0, 0);
      }
      if (is_mover) {   // the new leaves, the new sums of heights 1 .. hp, what the running maximum may rise to; the rows
        uint32_t mx = 0;
        bool bad = false;
        float* leaves = g.level[0] + (size_t)t * g.stride[0];
        for (uint32_t j = threadIdx.x; j < ride.n; j += blockDim.x) {
          const uint32_t slot = ride.cursor + j;
          leaves[slot] = rl[o1 + (slot - a1 * K)];   // (the old value again where the new one was invalid)
          if (ride.prio) {
            const float v = ride.prio[(size_t)t * ride.n + j];
            if (!valid_priority(v)) bad = true;
            else if (v > 0.0f) mx = __float_as_uint(v) > mx ? __float_as_uint(v) : mx;
          }
        }
        auto store_height = [&](uint32_t a, uint32_t cn, uint32_t o, int height) {
          float* lvl = g.level[height] + (size_t)t * g.stride[height];
          for (uint32_t at = threadIdx.x; at < cn; at += blockDim.x) lvl[a + at] = rl[ride.val_off + (o >> LOGK) + at];
        };
        store_height(a1, c1, o1, 1);
        if (hp > 1) store_height(a2, c2, o2, 2);
        if (hp > 2) store_height(a3, c3, o3, 3);
        if (hp > 3) store_height(a4, c4, o4, 4);
        if (ride.prio) {
          mx = wave_max_u32(mx);
          if (lane == 0 && mx) atomicMax(&g.max_pend[t], mx);
          if (bad) atomicOr(&g.status[t], 2u);
        }
        PER_MARK(14);
        ride_rows(ride, t, g.N, 0, movers);
        PER_MARK(12);
        PER_FLUSH_TAG(1);
        return;
      }
    }
    PER_MARK(14);
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
    // (a carried insertion: the group of a touched node is read from the patched copy)
    const float* patched = nullptr;
    if constexpr (RIDE) {
      // touched nodes of height l + 1 (l + 1 <= hp: the copy reaches down to hp)
      const uint32_t pa = l == 0 ? a1 : l == 1 ? a2 : l == 2 ? a3 : a4;
      const uint32_t pc = l == 0 ? c1 : l == 1 ? c2 : l == 2 ? c3 : c4;
      const uint32_t po = l == 0 ? o1 : l == 1 ? o2 : l == 2 ? o3 : o4;
      if (node - pa < pc) patched = rl + po + (size_t)(node - pa) * K;
    }
    if constexpr (LOGK <= 2) {
      if (RIDE && patched) descend_lane<LOGK>(patched, r, child, val);
      else descend_lane<LOGK>(lvl + (size_t)node * K, r, child, val);
    } else {
      stage_groups<LOGK, 0>(lvl, node, lane, stage);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      descend_lane<LOGK>(RIDE && patched ? patched : stage + lane * ROW, r, child, val);
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
  PER_FLUSH_TAG(1);
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
    if constexpr (RIDE) {
      mx = wave_max_u32(mx);
      if (lane == 0 && mx > max_seen) atomicMax(&g.max_pend[t], mx);
    } else {
      raise_max(g, t, mx, max_seen);
    }
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

// Workgroup size and top copy of a sampling launch for batch B (stale_hb: the height the stale top is rebuilt
// from, or 0).  The copy: at most kTopSlots of the topmost heights (below the root), within the LDS budget, and
// only while a height is small next to what the workgroup's samples would fetch from it one by one.
struct SampleShape {
  TopCopy tc;
  uint32_t waves, wave_bytes, top_bytes;
};
static SampleShape sample_shape(const Geom& g, const Tuning& tn, uint32_t B, uint32_t stale_hb, bool carries_insert = false) {
  constexpr uint32_t kLdsCap = 128 * 1024;
  SampleShape sh{};
  const uint32_t K = g.K;
  sh.wave_bytes = g.logK >= 3 ? 64u * (K + 4) * 4u : 0u;   // staging per wave
  // workgroup size: the whole batch in one workgroup when it is small (the weights are then finished
  // in-kernel), else the configured size; bounded by the LDS the staging rows need
  uint32_t max_waves = sh.wave_bytes ? (uint32_t)(kLdsCap / 2 / sh.wave_bytes) : 16u;
  if (max_waves > 16) max_waves = 16;
  if (max_waves < 1) max_waves = 1;
  uint32_t waves = tn.sample_block / 64;
  // Every sampling workgroup of a launch that carries an insertion works that insertion out for itself: on many trees
  // fewer, larger workgroups pay (64 trees, 1024 samples and 16 rows each: 29.3 -> 28.5 us per step with 512 lanes;
  // on one tree the small ones stay ahead).  Only when the size was not asked for.
  if (carries_insert && tn.sample_block_auto && g.T >= 8 && waves < 8) waves = 8;
  const uint32_t need = (B + 63) / 64;
  if (need <= max_waves) waves = need;
  if (waves > max_waves) waves = max_waves;
  sh.waves = waves;
  const uint32_t block = waves * 64;
  TopCopy& tc = sh.tc;
  uint64_t top = 0;
  for (int l = (int)g.H - 1; l >= 0 && tc.nslots < (uint32_t)kTopSlots; --l) {
    const uint64_t cnt = (uint64_t)g.n[l + 1] * K;
    const uint64_t add = cnt * 4;
    if (top + add > tn.lds_budget_bytes || top + add + (uint64_t)waves * sh.wave_bytes > kLdsCap) break;
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
  sh.top_bytes = (uint32_t)top;
  return sh;
}

// A carried insertion: the touched nodes of heights 1 .. hp (two ranges per height, narrowed by K from one height
// to the next) and where their child groups, their new sums and the new leaves sit in LDS.
constexpr uint32_t kRideRows = 1024;          // most rows a sampling kernel carries
constexpr uint32_t kRideLdsBytes = 16 * 1024; // most LDS its patch may take
// False when the insertion runs past the ring's end or a run of child groups is longer than the workgroup (`block`
// lanes): the insertion then goes by itself.
static bool plan_ride(const Geom& g, const TopCopy& tc, uint32_t block, uint32_t hp, InsertRide* rd) {
  const uint32_t L = g.logK;
  if ((uint64_t)rd->cursor + rd->n > g.N || hp > (uint32_t)kRideHeights) return false;
  uint32_t a = rd->cursor, b = rd->cursor + rd->n;   // touched nodes [a, b)
  uint32_t floats = 0, vals = 0;
  for (int i = 0; i < kRideHeights; ++i) rd->h[i] = RideHeight{0, 0, 0, kRideNone};
  for (uint32_t h = 1; h <= hp; ++h) {
    a >>= L;
    b = ((b - 1) >> L) + 1;
    RideHeight& P = rd->h[h - 1];
    P.a0 = a;
    P.cnt = b - a;
    P.off = floats;
    if ((uint64_t)P.cnt * g.K > block) return false;
    uint32_t top = 0;   // where the sampling kernel's top copy holds this height
    for (uint32_t i = 0; i < tc.nslots; ++i) {
      if (g.H - 1 - i == h) P.top_at = top;
      top += tc.cnt[i];
    }
    floats += P.cnt * g.K;
    vals += P.cnt;
  }
  rd->hp = hp;
  rd->val_off = floats;
  rd->floats = floats + vals;
  return true;
}

bool sample_can_carry_insert(const Geom& g, const Tuning& tn, uint32_t B, const FieldTable* ft, uint32_t n, uint32_t cursor) {
  const uint32_t hb = lazy_top_height(g, tn);
  if (!hb || hb > (uint32_t)kRideHeights || n == 0 || n > kRideRows || n > g.N) return false;
  uint64_t bytes = 0;
  if (ft)
    for (uint32_t f = 0; f < ft->n_fields; ++f)
      if (ft->io[f]) bytes += (uint64_t)n * ft->bytes[f];
  if (bytes > 256 * 1024) return false;
  // the top copy must reach down to the height the top is rebuilt from
  const SampleShape sh = sample_shape(g, tn, B, hb, true);
  if (sh.tc.nslots == 0 || g.H - sh.tc.nslots > hb) return false;
  // the runs of the patch must fit the workgroup, and the patch its share of the LDS
  InsertRide rd{};
  rd.n = n;
  rd.cursor = cursor;
  return plan_ride(g, sh.tc, sh.waves * 64, hb, &rd) && (uint64_t)rd.floats * 4 <= kRideLdsBytes;
}

// Sampling call with whatever is fused into it.  rows: gather of the sampled rows.  claim: a priority
// update whose claim phase runs where claim_mode says (CLAIM_INLINE / CLAIM_BLOCKS: in the sampling
// kernel, the tree pass then shares the second kernel with the weights and row jobs; CLAIM_FINISH: in
// the second kernel, the tree pass is a third).  ride: an insertion carried by the sampling kernel (the caller
// has checked sample_can_carry_insert and passes the lazily rebuilt height as stale_hb).
template <int LOGK>
static hipError_t launch_sample_k(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, float beta,
                                  const float* u, const RngArgs& rng, uint32_t* out_idx, float* out_w,
                                  float* out_prio, uint32_t weight_mode, uint32_t stale_hb, const FieldTable* rows,
                                  const ClaimArgs* claim, int claim_mode, const InsertRide* ride, hipStream_t s) {
  const SampleShape sh = sample_shape(g, tn, B, stale_hb, ride != nullptr);
  const TopCopy& tc = sh.tc;
  const uint32_t waves = sh.waves;
  const uint32_t block = waves * 64;
  const uint32_t gx = (B + block - 1) / block;
  size_t bytes = (size_t)sh.top_bytes + (size_t)waves * sh.wave_bytes;
  hipError_t e;
  int stale = -1;
  if (stale_hb) {
    // copied heights above stale_hb are rebuilt in LDS; the copy must reach down to stale_hb
    const int lowest_copied = (int)g.H - (int)tc.nslots;
    if (tc.nslots > 0 && lowest_copied <= (int)stale_hb) {
      stale = (int)g.H - 1 - (int)stale_hb;
    } else {
      if (ride) return hipErrorInvalidValue;
      e = launch_resum_top_k<LOGK>(g, tn, stale_hb, s);
      if (e != hipSuccess) return e;
    }
  }
  if (!claim) claim_mode = CLAIM_NONE;
  InsertRide rd{};
  if (ride) {
    if (stale < 0 || stale_hb != lazy_top_height(g, tn) || claim_mode == CLAIM_BLOCKS) return hipErrorInvalidValue;
    rd = *ride;
    if (!plan_ride(g, tc, block, stale_hb, &rd)) return hipErrorInvalidValue;
    // movers: as many as it takes to move every row element in one sweep (whole rows each; at most 32)
    uint64_t row_elements = 0;
    for (uint32_t f = 0; f < rd.rows.n_fields; ++f)
      if (rd.rows.io[f]) row_elements += (uint64_t)rd.n * (rd.rows.bytes[f] / rd.rows.vec[f]);
    rd.movers = (uint32_t)((row_elements + block - 1) / block);
    if (rd.movers > rd.n) rd.movers = rd.n;
    if (rd.movers > 32) rd.movers = 32;
    if (rd.movers < 1) rd.movers = 1;
    bytes += (size_t)rd.floats * 4;
  }
  if (bytes < tn.sample_min_lds) bytes = tn.sample_min_lds;   // asking for more LDS than needed spreads workgroups over more CUs
  const bool claim_here = claim_mode == CLAIM_INLINE || claim_mode == CLAIM_BLOCKS;
  uint32_t claim_blocks = 0;
  if (claim_mode == CLAIM_BLOCKS) {
    claim_blocks = (claim->B + block - 1) / block;
    if (claim_blocks > 4096) claim_blocks = 4096;   // the claim job strides
  }
  if (ride) {
    e = grant_lds<&k_sample<LOGK, true>>(tn, bytes);
    if (e != hipSuccess) return e;
    PER_LAUNCH(KID_SAMPLE, (k_sample<LOGK, true>), dim3(gx + claim_blocks + rd.movers, g.T), dim3(block), bytes, s, g, tc, B,
               size, beta, u, out_idx, out_prio, out_w, weight_mode, stale, claim_blocks, claim_here ? *claim : ClaimArgs{},
               claim_here ? claim_mode : (int)CLAIM_NONE, rng, rd);
  } else {
    e = grant_lds<&k_sample<LOGK, false>>(tn, bytes);
    if (e != hipSuccess) return e;
    PER_LAUNCH(KID_SAMPLE, (k_sample<LOGK, false>), dim3(gx + claim_blocks, g.T), dim3(block), bytes, s, g, tc, B, size,
               beta, u, out_idx, out_prio, out_w, weight_mode, stale, claim_blocks, claim_here ? *claim : ClaimArgs{},
               claim_here ? claim_mode : (int)CLAIM_NONE, rng, NoRide{});
  }
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
    ClaimArgs c2{};
    if (claim) {
      c2 = *claim;
      c2.fold_max = ride ? 1u : 0u;   // the tree pass folds what this kernel has left in max_pend
    }
    if (claim_here) {   // second kernel: tree pass beside the weights and the rows
      if (rows || finish_weights) return launch_tree_finish_k<LOGK>(g, tn, c2, rows, a, s);
      return launch_tree_k<LOGK>(g, tn, c2, s);
    }
    // second kernel: rows, weights and the claim phase; the tree pass follows
    a.has_claim = claim ? 1u : 0u;
    if (claim) a.claim = c2;
    e = launch_finish(g, tn, rows, a, s);
    if (e != hipSuccess || !claim) return e;
    return launch_tree_k<LOGK>(g, tn, c2, s);
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
                         hipStream_t s, const InsertRide* ride) {
#define CALL(L) launch_sample_k<L>(g, tn, B, size, beta, u, rng, out_idx, out_w, out_prio, weight_mode, stale_hb, rows, claim, claim_mode, ride, s)
  PER_DISPATCH_LOGK(g.logK, CALL)
#undef CALL
}
