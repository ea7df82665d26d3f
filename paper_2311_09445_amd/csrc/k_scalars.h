// Fill kernel and the kernels that read or reset per-tree scalars.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

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

hipError_t launch_fill_u32(const Tuning& tn, uint32_t* p, uint64_t count, uint32_t value, hipStream_t s) {
  if (count == 0) return hipSuccess;
  uint64_t blocks = (count / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 16384) blocks = 16384;
  PER_LAUNCH(KID_FILL, k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, count, value);
  return hipGetLastError();
}

__global__ void k_init_scalars(Geom g, float init_max) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= g.T) return;
  g.max_v[t] = init_max;
  g.status[t] = 0;
  g.max_pend[t] = 0;
  for (uint32_t k = 0; k < 2 * kVminSlots; ++k) g.vmin[((size_t)(k / kVminSlots) * g.T + t) * kVminSlots + k % kVminSlots] = kNoMin;
  g.vnext[t] = 0;
  g.vcur[t] = 0;
  g.sbase[t] = 1;
  g.sfloor[t] = 1;
  if (g.step_ho) {
    for (uint32_t k = 0; k < kStepGroups; ++k) g.step_cnt[(size_t)t * kStepGroups + k] = 0ull;
    g.step_cnt2[t] = 0ull;
    g.step_rel[t] = 0u;
    for (uint32_t k = 0; k < 2 * kStepDoneSlots; ++k) g.step_done[(size_t)t * 2 * kStepDoneSlots + k] = 0u;
    for (uint32_t k = 0; k < 2 * kVminSlots; ++k) g.step_vmin[(size_t)t * 2 * kVminSlots + k] = kNoMin;
  }
}

hipError_t launch_init_scalars(const Geom& g, float init_max, hipStream_t s) {
  k_init_scalars<<<dim3((g.T + 63) / 64), dim3(64), 0, s>>>(g, init_max);
  return hipGetLastError();
}

// which: 0 = root of every tree, 1 = running max priority, 2 = smallest positive leaf from the partial
// minima of k_min_reduce (weight_mode tells how many there are)
__global__ void k_read_scalars(Geom g, int which, uint32_t weight_mode, float* out) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= g.T) return;
  if (which == 2) {
    uint32_t m = kNoMin;
    for (uint32_t k = 0; k < (weight_mode >> kWeightPartsShift); ++k) {
      const uint32_t v = g.vmin_buf[(size_t)t * kMinParts + k];
      m = v < m ? v : m;
    }
    out[t] = __uint_as_float(m);
    return;
  }
  out[t] = which == 0 ? g.root[(size_t)t * g.root_stride] : g.max_v[t];
}

hipError_t launch_read_scalars(const Geom& g, int which, uint32_t weight_mode, float* out, hipStream_t s) {
  k_read_scalars<<<dim3((g.T + 63) / 64), dim3(64), 0, s>>>(g, which, weight_mode, out);
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
