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

#include <hip/hip_ext.h>

#include <atomic>
#include <mutex>
#include <type_traits>

namespace per {

// ---------------------------------------------------------------------------------
// per-kernel timing
// ---------------------------------------------------------------------------------
const char* kernel_name(int kid) {
  static const char* const names[KID_COUNT] = {
      "k_fill_u32", "k_sample", "k_weights", "k_rows_gather", "k_finish", "k_rows_scatter", "k_insert_leaves",
      "k_resum_dense", "k_resum_tail", "k_update_claim", "k_update_tree", "k_tree_finish", "k_update_delta",
      "k_get_priority", "k_insert_small", "k_run_steps", "k_run_requests", "k_min_rebuild", "k_min_reduce", "k_step",
      "k_step_tables", "k_step_epilogue"};
  return kid >= 0 && kid < KID_COUNT ? names[kid] : "?";
}

void Profiler::reset() {
  for (Rec& r : recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  recs.clear();
  for (int k = 0; k < KID_COUNT; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
}

hipError_t Profiler::collect() {
  hipError_t first = hipSuccess;
  for (Rec& r : recs) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e == hipSuccess) { total_ms[r.kid] += ms; launches[r.kid] += 1; }
    else if (first == hipSuccess) first = e;
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  recs.clear();
  return first;
}

// When profiling is on, the launch carries its own pair of events (hipExtLaunchKernelGGL stamps
// them at the start and at the end of the kernel's execution, not at enqueue time), so the
// durations are those of the kernels themselves.
bool Profiler::begin(int kid, hipEvent_t* start, hipEvent_t* stop) {
  if (!on) return false;
  Rec r;
  r.kid = kid;
  if (hipEventCreate(&r.start) != hipSuccess) return false;
  if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return false; }
  recs.push_back(r);
  *start = r.start;
  *stop = r.stop;
  return true;
}

#define PER_LAUNCH(KID, KERNEL, GRID, BLOCK, LDS, STREAM, ...)                                     \
  do {                                                                                             \
    hipEvent_t ev_start_, ev_stop_;                                                                \
    if (tn.prof && tn.prof->begin(KID, &ev_start_, &ev_stop_))                                     \
      hipExtLaunchKernelGGL((KERNEL), GRID, BLOCK, LDS, STREAM, ev_start_, ev_stop_, 0, __VA_ARGS__); \
    else                                                                                           \
      KERNEL<<<GRID, BLOCK, LDS, STREAM>>>(__VA_ARGS__);                                           \
  } while (0)

// Dynamic LDS beyond the default limit of 64 KB has to be granted per kernel and device by a host call.  The
// largest grant made so far is remembered per kernel (process-wide: the grant belongs to the kernel, not to a
// buffer), so the call is made when a kernel first needs a size, not once per launch.
constexpr int kMaxDevices = 64;
template <auto Kern>
static hipError_t grant_lds(const Tuning& tn, size_t bytes) {
  static std::atomic<uint32_t> granted[kMaxDevices];
  if (bytes <= 64 * 1024) return hipSuccess;
  const bool tracked = tn.device >= 0 && tn.device < kMaxDevices;
  if (tracked && granted[tn.device].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)bytes);
  if (e == hipSuccess && tracked) granted[tn.device].store((uint32_t)bytes, std::memory_order_relaxed);
  return e;
}

#include "dev_trace.h"
#include "dev_common.h"
#include "k_scalars.h"
#include "k_claim.h"
#include "k_sample.h"
#include "k_rows.h"
#include "k_resum.h"
#include "k_insert.h"
#include "k_tree.h"
#include "k_step.h"
#include "k_delta.h"
#include "k_stream.h"
#include "k_retrieve.h"
#include "k_min.h"

}  // namespace per
