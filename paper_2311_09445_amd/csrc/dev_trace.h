// Optional in-kernel time stamps (development builds with -DPER_TRACE only).
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// optional in-kernel time stamps (development builds with -DPER_TRACE only)
// ---------------------------------------------------------------------------------
#ifdef PER_TRACE
// Time stamps are kept in registers and stored when the kernel ends, so that taking them does
// not add memory traffic (or waits for it) to the phases being timed.
constexpr int kTraceMarks = 16, kTraceBlocks = 2048;
__device__ unsigned long long g_trace[kTraceBlocks * kTraceMarks];
#define PER_TRACE_DECL unsigned long long tm_[kTraceMarks] = {}
#define PER_MARK(i) do { tm_[(i)] = wall_clock64(); } while (0)
#define PER_MARK_HWID(i) /* XCC id and HW_ID (SE, CU, SIMD, wave slot) of the calling wave */    \
  do {                                                                                         \
    tm_[(i)] = ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |        \
               (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);                            \
  } while (0)
#define PER_MARK_DYN(i)                                                                        \
  do {                                                                                         \
    const unsigned long long now_ = wall_clock64();                                            \
    _Pragma("unroll") for (int k_ = 0; k_ < kTraceMarks; ++k_) if (k_ == (int)(i)) tm_[k_] = now_; \
  } while (0)
// Kernels flush under tag 0, or under a tag of their own; only the selected tag's flushes are kept.
__device__ int g_trace_tag = 0;
#define PER_FLUSH() PER_FLUSH_TAG(0)
// Which workgroups are kept: those of tree 0 (g_trace_every == 0), or every g_trace_every-th of the whole grid,
// numbered tree after tree.
__device__ unsigned g_trace_every = 0;
#define PER_FLUSH_TAG(tag)                                                                     \
  do {                                                                                         \
    const unsigned every_ = g_trace_every;                                                     \
    const unsigned long long lin_ = (unsigned long long)blockIdx.y * gridDim.x + blockIdx.x;   \
    const bool keep_ = every_ ? lin_ % every_ == 0 && lin_ / every_ < kTraceBlocks             \
                              : blockIdx.y == 0 && blockIdx.x < kTraceBlocks;                  \
    if (threadIdx.x == 0 && keep_ && g_trace_tag == (tag)) {                                   \
      const unsigned slot_ = every_ ? (unsigned)(lin_ / every_) : blockIdx.x;                  \
      _Pragma("unroll") for (int k_ = 0; k_ < kTraceMarks; ++k_)                               \
        g_trace[slot_ * kTraceMarks + k_] = tm_[k_];                                           \
    }                                                                                          \
  } while (0)
extern "C" int per_trace_select(int tag) {
  return hipMemcpyToSymbol(HIP_SYMBOL(g_trace_tag), &tag, sizeof(tag)) == hipSuccess ? 0 : -1;
}
extern "C" int per_trace_every(unsigned every) {
  return hipMemcpyToSymbol(HIP_SYMBOL(g_trace_every), &every, sizeof(every)) == hipSuccess ? 0 : -1;
}
extern "C" int per_trace_read(unsigned long long* host, int clear) {
  if (hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), sizeof(g_trace)) != hipSuccess) return -1;
  if (clear) {
    static unsigned long long zeros[kTraceBlocks * kTraceMarks];
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_trace), zeros, sizeof(zeros)) != hipSuccess) return -1;
  }
  return kTraceBlocks * kTraceMarks;
}
#else
#define PER_TRACE_DECL do { } while (0)
#define PER_MARK(i) do { } while (0)
#define PER_MARK_HWID(i) do { } while (0)
#define PER_MARK_DYN(i) do { } while (0)
#define PER_FLUSH() do { } while (0)
#define PER_FLUSH_TAG(tag) do { } while (0)
#endif
