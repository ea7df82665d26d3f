// First half of a priority update: the claim of leaves by the last writer.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// priority update, first half: claim
// ---------------------------------------------------------------------------------
// Element j raises the 64-bit stamp of its leaf to (stamp_base + j) << 32 | value bits by
// atomic max, and sets the leaf's bit in the dirty mask (one bit per leaf).  The largest j wins
// and carries its value with it.  Stamps grow from call to call, so stale stamps never win
// and the stamp array needs no clearing between calls.
__device__ __forceinline__ void claim_element(const Geom& g, uint32_t t, uint32_t size, uint32_t stamp_base, uint32_t j,
                                              uint32_t i, float v, uint32_t& mx, uint32_t& flags) {
  if (!(i < size)) flags |= 1u;
  else if (!valid_priority(v)) flags |= 2u;
  else {
    const unsigned long long stamp = ((unsigned long long)(stamp_base + j) << 32) | __float_as_uint(v);
    atomicMax(reinterpret_cast<unsigned long long*>(g.owner) + (size_t)t * g.owner_stride + i, stamp);
    atomicOr(&g.dirty[(size_t)t * g.dirty_stride + (i >> 5)], 1u << (i & 31u));
    const uint32_t vb = v > 0.0f ? __float_as_uint(v) : 0u;
    mx = vb > mx ? vb : mx;
  }
}

// Claims elements of the batch, strided over the job's workgroups.  Called by whole workgroups.
// TD: the batch may hold temporal-difference errors to be turned into priorities first (only the
// stand-alone claim kernel carries that code).
template <bool TD = false>
__device__ __forceinline__ void claim_job(const Geom& g, uint32_t t, const ClaimArgs& c, uint32_t job_block,
                                          uint32_t job_blocks) {
  if (job_block * blockDim.x >= c.B) return;   // nothing to do for this workgroup
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
      claim_element(g, t, c.size, c.stamp_base, j, c.idx[(size_t)t * c.B + j], v, mx, flags);
    }
  }
  raise_max(g, t, mx, max_seen);
  if (flags) atomicOr(&g.status[t], flags);
}

__global__ void k_update_claim(Geom g, ClaimArgs c) { claim_job<true>(g, blockIdx.y, c, blockIdx.x, gridDim.x); }
