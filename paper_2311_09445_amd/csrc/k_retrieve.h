// Priority retrieval.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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

hipError_t launch_get_priority(const Geom& g, const Tuning& tn, uint32_t n, const uint32_t* idx, float* out,
                               hipStream_t s) {
  PER_LAUNCH(KID_GET_PRIORITY, k_get_priority, dim3((n + 255) / 256, g.T), dim3(256), 0, s, g, n, idx, out);
  return hipGetLastError();
}
