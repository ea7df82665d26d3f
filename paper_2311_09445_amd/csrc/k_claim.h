// First half of a priority update: the claim of leaves by the last writer.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// priority update, first half: claim
// ---------------------------------------------------------------------------------
// Nothing about an update lives on the host (a captured update can be replayed).  The leaf stamps and the
// dirty bits are all zero between update batches: the tree pass that consumes a batch's claims clears
// exactly what the batch has set there (few leaves), so a leaf stamp only orders the elements of one
// batch.  The group entries are not cleared after every batch (that cost 0.5 us of write-back per
// step): their stamps come from a counter in device memory that grows from batch to batch, so an
// entry left by an earlier batch is recognised by its stamp lying below the batch's first.
//
// Leaf by leaf: element j raises the 64-bit stamp of its leaf to (base + j) << 32 | value bits by
// atomic max (base >= 1), and sets the leaf's bit in the dirty mask (one bit per leaf).  The largest j wins
// and carries its value with it.
__device__ __forceinline__ void claim_leaf(const Geom& g, uint32_t t, uint32_t i, uint32_t stamp, uint32_t vbits) {
  atomicMax(reinterpret_cast<unsigned long long*>(g.owner) + (size_t)t * g.owner_stride + i,
            ((unsigned long long)stamp << 32) | vbits);
  atomicOr(&g.dirty[(size_t)t * g.dirty_stride + (i >> 5)], 1u << (i & 31u));
}

// Through group entries: the per-leaf stamps of a large tree live in memory, and a batch spread over
// the tree pays a memory transaction per element to raise them and another to read them back.  A group
// of 32 leaves (64 for K = 64) therefore shares one entry, (stamp << 6 | leaf within the group, value
// bits), in an array small enough to stay in cache.  An element raises its group's entry by a
// returning atomic max.  Only when it meets an element of THIS batch (stamp at or above the batch's
// first) for ANOTHER leaf of the group, the earlier of the two is claimed leaf by leaf instead.
// At the end the entry holds the latest element of the whole group, which is the last writer of
// its leaf; every other leaf's last writer has gone to that leaf's own stamp, where the largest
// stamp wins as before: when it met the entry it either found a later element of another leaf, or
// it was stored and whatever displaced it later (necessarily of another leaf) passed it on.
// Elements for one leaf never need the detour: the later of them dominates the earlier.
// (The stamp has 26 bits here: see kGroupStampTurn.)
__device__ __forceinline__ void claim_in_group(const Geom& g, uint32_t t, uint32_t base, uint32_t j, uint32_t i,
                                               uint32_t vbits) {
  const uint32_t lg = g.logK == 6 ? 6u : 5u;
  const uint32_t slot = i & ((1u << lg) - 1u);
  const uint32_t mine_hi = ((base + j) << 6) | slot;
  const unsigned long long mine = ((unsigned long long)mine_hi << 32) | vbits;
  const unsigned long long old =
      atomicMax(reinterpret_cast<unsigned long long*>(g.nclaim) + (size_t)t * g.nclaim_stride + (i >> lg), mine);
  const uint32_t old_hi = (uint32_t)(old >> 32);
  if ((old_hi >> 6) >= base && (old_hi & 63u) != slot) {
    const bool stays = mine > old;
    const uint32_t out_hi = stays ? old_hi : mine_hi;
    claim_leaf(g, t, (i & ~((1u << lg) - 1u)) | (out_hi & 63u), out_hi >> 6, stays ? (uint32_t)old : vbits);
  }
}

// base: the batch's first stamp (group_mode: from the device counter, see claim_base; else 1).
__device__ __forceinline__ void claim_element(const Geom& g, uint32_t t, uint32_t size, uint32_t group_mode,
                                              uint32_t base, uint32_t j, uint32_t i, float v, uint32_t& mx,
                                              uint32_t& flags) {
  if (!(i < size)) flags |= 1u;
  else if (!valid_priority(v)) flags |= 2u;
  else {
    if (group_mode) claim_in_group(g, t, base, j, i, __float_as_uint(v));
    else claim_leaf(g, t, i, base + j, __float_as_uint(v));
    const uint32_t vb = v > 0.0f ? __float_as_uint(v) : 0u;
    mx = vb > mx ? vb : mx;
  }
}

// First stamp of the batch being claimed.  Through group entries it is the device counter (stable while the
// claim phase runs: only a tree pass writes it); one lane of the phase (`leader`) leaves it for the
// batch's tree pass.
__device__ __forceinline__ uint32_t claim_base(const Geom& g, uint32_t t, uint32_t group_mode) {
  return group_mode ? read_word_with_the_loads(g.sbase + t) : 1u;
}
// (stores last: the leader's store would otherwise make its wave wait for `base` before it issues its loads)
__device__ __forceinline__ void leave_claim_base(const Geom& g, uint32_t t, uint32_t group_mode, bool leader, uint32_t base) {
  if (group_mode && leader) g.sfloor[t] = base;
}

// Claims elements of the batch, strided over the job's workgroups.  Called by whole workgroups.
// TD: the batch may hold temporal-difference errors to be turned into priorities first (only the
// stand-alone claim kernel carries that code).
template <bool TD = false>
__device__ __forceinline__ void claim_job(const Geom& g, uint32_t t, const ClaimArgs& c, uint32_t job_block,
                                          uint32_t job_blocks) {
  if (job_block * blockDim.x >= c.B) return;   // nothing to do for this workgroup
  const uint32_t first = claim_base(g, t, c.group_mode);
  const uint32_t max_seen = read_max_bits(g, t);
  uint32_t mx = 0;
  uint32_t flags = 0;
  for (uint32_t base = job_block * blockDim.x; base < c.B; base += job_blocks * blockDim.x) {
    const uint32_t j = base + threadIdx.x;
    if (j < c.B) {
      float v = c.prio[(size_t)t * c.B + j];
      if constexpr (TD) {
        if (c.from_td)   // priority of a temporal-difference error; a non-finite error stays non-finite and is rejected
          v = (float)pow(fabs((double)v) + c.td_eps, c.td_alpha);
      }
      uint32_t at = j;
      if (c.pos) at = c.pos[(size_t)t * c.B + j];
      const uint32_t i = at < c.B ? c.idx[(size_t)t * c.B + at] : 0xFFFFFFFFu;
      claim_element(g, t, c.size, c.group_mode, first, j, i, v, mx, flags);
    }
  }
  raise_max(g, t, mx, max_seen);
  if (flags) atomicOr(&g.status[t], flags);
  leave_claim_base(g, t, c.group_mode, job_block == 0 && threadIdx.x == 0, first);
}

__global__ void k_update_claim(Geom g, ClaimArgs c) {
  claim_job<true>(g, blockIdx.y, c, blockIdx.x, gridDim.x);
}
