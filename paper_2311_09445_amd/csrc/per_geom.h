// Internal: tree geometry shared by the C-ABI layer and the kernels.
//
// Height h counts from the leaves: n[0] = N, n[h+1] = ceil(n[h] / K), root at
// height H.  Each stored level is zero-padded to a multiple of K so every child
// group is K wide ("a parent node stores the sum of priorities of its
// children", Section V-A); one array per level, as in the paper's FPGA design
// where every pipeline stage owns one tree level.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/per.h"

namespace per {

constexpr int kMaxHeight = 32;   // K = 2, N = 2^31 gives H = 31
constexpr int kMaxFields = 8;
constexpr uint32_t kVminSlots = 256;   // partial batch minima per tree and buffer
constexpr uint32_t kStepGroups = 64;   // counters the owners of the one-kernel step are spread over (one wave reads them all)
constexpr uint32_t kStepDoneSlots = 8; // counters its builders are spread over
constexpr uint32_t kStepMaxOwners = 2048;   // most owner workgroups over all trees

struct Geom {
  uint32_t K, logK, H, T;
  uint32_t N;                       // leaves per tree (<= 2^31)
  uint32_t n[kMaxHeight + 1];       // real nodes per level
  uint32_t stride[kMaxHeight + 1];  // floats between consecutive trees of a level (multiple of 64)
  float*   level[kMaxHeight + 1];   // level h of tree 0
  float*   root;                    // == level[H]; at a fixed offset so kernels need no dependent load
  uint32_t root_stride;             // == stride[H]
  uint64_t* owner;                  // [T][owner_stride] last-writer stamps: (stamp << 32) | fp32 bits of the value; zero between batches
  uint32_t owner_stride;
  uint2*   nclaim;                  // [T][nclaim_stride] group entries of the claim phase: (value bits, stamp << 6 | slot)
  uint32_t* sbase;                  // [T] first stamp of the next batch that claims through the group entries (device-side counter)
  uint32_t* sfloor;                 // [T] first stamp of the batch being processed (left by its claim phase for its tree pass)
  uint32_t nclaim_stride;
  uint32_t* dirty;                  // [T][dirty_stride] words of one bit per leaf: the leaf was claimed by the current update
  uint32_t dirty_stride;
  uint32_t* arrive;                 // [T][arrive_stride] arrival counters of the nodes of heights >= 2
  uint32_t arrive_stride;
  uint32_t arrive_off[kMaxHeight + 1];   // offset of height h (>= 2) inside a tree's counters
  float*    max_v;                  // [T] running max priority
  uint32_t* max_pend;               // [T] fp32 bits raised by a sampling kernel that carries an insertion (which reads max_v while
                                    // its claim lanes would raise it); folded into max_v by the tree pass of the same call; else 0
  uint32_t* status;                 // [T] sticky flags
  uint32_t* vmin;                   // [2][T][kVminSlots] partial batch minima of sampled values (fp32 bits), two buffers
  uint32_t* vnext;                  // [T] which buffer the next sampling kernel fills (written by the weights job)
  uint32_t* vcur;                   // [T] which buffer the current call uses (written by its sampling kernel for its weights job)
  uint32_t* min1;                   // [T][min1_stride] smallest positive leaf under each height-1 node (fp32 bits; kNoMin: none)
  uint32_t min1_stride;
  uint32_t* vmin_buf;               // [T][kMinParts] partial minima of min1 (fp32 bits), one per workgroup of k_min_reduce
  uint32_t step_ho;                 // owner height of the one-kernel step (0: that kernel does not fit this tree)
  float*   step_side;               // [T][step_side_stride] where its owners leave the new nodes of height step_ho
  void*    step_tab;                // its per-owner tables
  uint32_t step_tab_static;         // 1: they sit in the kernels' static array (see k_step), not in the arena
  uint32_t step_side_stride;
  unsigned long long* step_cnt;     // [T][kStepGroups] owners of the one-kernel step that have finished, over all calls
  uint32_t* step_done;              // [T][2][kStepDoneSlots] its builders that have finished (by parity of the call)
  uint32_t* step_vmin;              // [T][2][kVminSlots] smallest sampled values of its call (by parity)
  unsigned long long* step_cnt2;    // [T] groups of owners that have all arrived at the end of their update, over all calls that
                                    // finish inside the one kernel
  uint32_t* step_rel;               // [T] number of the last call whose owners have all arrived (what its waiting workgroups poll)
};
uint32_t step_owner_height(const Geom& g);   // (needs K, logK, H, T, n[])
constexpr uint32_t kMinParts = 1024;     // most workgroups k_min_reduce is launched with
constexpr uint32_t kStaticMinTrees = 64; // most trees per_min_priority_static serves (its static array: 64 x 1024 words = 256 KiB per GPU)

constexpr uint32_t kNoMin = 0x7F800000u;   // fp32 bits of +inf: above every valid priority

// How a sampling call scales its importance weights, packed into one kernel argument: 0 = by the batch's
// smallest sampled value; else kWeightBufferNorm | (number of partial minima in vmin_buf << kWeightPartsShift) =
// by the smallest positive leaf of the whole tree.
constexpr uint32_t kWeightBufferNorm = 1u;
constexpr uint32_t kWeightPartsShift = 8u;

// Payload.  Stored row-major: the fields of a row lie side by side (a row of several fields is then one or
// two cache lines to fetch, not one per field); the caller's arrays are dense per field.
struct FieldTable {
  uint8_t* col[kMaxFields];         // field f of row 0 of tree 0
  uint8_t* io[kMaxFields];          // caller's dense [T][B][bytes] array (source or destination)
  uint64_t col_stride[kMaxFields];  // bytes between trees (the same for every field)
  uint32_t bytes[kMaxFields];       // bytes of the field
  uint32_t vec[kMaxFields];         // bytes moved per lane: 16, 8, 4, 2 or 1
  uint32_t n_fields;
  uint32_t row_stride;              // bytes between stored rows (multiple of 16)
};

// Stamps of the group entries: 26 bits, taken from a counter in device memory that starts at 1 and
// grows by the batch size; a batch starts at or below kGroupStampTurn and is no longer than that, so
// its stamps fit; the tree pass of a batch that ends beyond it clears all entries and restarts the
// counter (about every 500 steps of the headline workload).
constexpr uint32_t kGroupStampTurn = 1u << 25;

// An update may leave the heights above its tree pass's workgroup roots to their next reader while that
// height has at most this many nodes.
constexpr uint32_t kLazyTopNodes = 4096;
constexpr uint32_t kStepSideStride = kLazyTopNodes + 64;   // floats per tree of the one-kernel step's side array
constexpr uint32_t kGroupClaimMaxBatch = kGroupStampTurn;

// Claim phase of a priority update (first half of per_update).
struct ClaimArgs {
  uint32_t B, size;
  uint32_t group_mode;     // the batch claims through the group entries (else leaf by leaf)
  uint32_t track_min;      // the tree pass also renews min1 of the height-1 nodes it rebuilds
  uint32_t fold_max;       // the tree pass also folds max_pend into the running maximum
  const uint32_t* idx;     // [T][B]
  const uint32_t* pos;     // null, or [T][B] positions: element j targets idx[pos[j]] (the leaf drawn by sample pos[j] of the
                           // sampling call the update is fused with); a position >= B makes the element invalid
  const float* prio;       // [T][B] tree values, or temporal-difference errors when from_td is set
  uint32_t from_td;        // value = (|prio| + td_eps)^td_alpha, fp64, rounded once
  double td_eps, td_alpha;
};

// Source of the uniforms of a sampling call when the caller passes none: a counter-based generator,
// counter (sample, call low, call high, tree), key (seed low, seed high).
struct RngArgs {
  uint32_t on;
  uint32_t seed_lo, seed_hi, call_lo, call_hi;
};

// Where the claim phase of an update fused into a sampling call runs.
enum ClaimMode {
  CLAIM_NONE = 0,
  CLAIM_INLINE = 1,   // by the sampling lanes: the update batch is the sampled batch (same index array)
  CLAIM_BLOCKS = 2,   // by extra workgroups of the sampling kernel: the update batch lies in other memory
  CLAIM_FINISH = 3    // in the second kernel, after sampling: the update batch overlaps the sampling outputs
};

// Jobs of the second kernel of the fused calls (see k_finish).
struct FinishArgs {
  uint32_t B;              // sampled batch
  const uint32_t* idx;     // [T][B] sampled indices
  float* w;                // [T][B] sampled values in, weights out; nullptr: no weights job
  uint32_t size;
  float beta;
  uint32_t weight_mode;    // see kWeightBufferNorm
  uint32_t has_claim;
  ClaimArgs claim;
};

// A list of steps run by one workgroup per tree on an LDS copy of the tree (see k_run_steps).
struct StreamArgs {
  uint32_t n_steps, n_insert, B;
  uint32_t cursor, size;            // ring state before the first step
  uint32_t upd_is_sampled;          // a step updates the batch it has just sampled
  uint32_t buffer_norm;             // importance weights relative to the whole tree (else to the batch)
  const float* u;                   // [steps][T][B]
  const float* beta;                // [steps]
  uint32_t* out_idx;                // [steps][T][B]
  float* out_w;                     // [steps][T][B] or null
  float* out_prio;                  // [steps][T][B] or null
  const uint32_t* upd_idx;          // [steps][T][B] (unused when upd_is_sampled)
  const float* upd_prio;            // [steps][T][B] or null: no update
  const float* ins_prio;            // [steps][T][n_insert] or null: running maximum
  FieldTable ins, rows;             // io arrays hold [steps][T][n][bytes]; io all null: nothing to move
  uint32_t off[kMaxHeight + 2];     // where height h starts in LDS (floats); off[H + 1] = all floats
  uint32_t leaves_in_memory;        // the LDS copy holds heights 1 .. H only
};

// A queue of op-coded requests run by one workgroup per tree on an LDS copy of the tree (see k_run_requests).
struct QueueArgs {
  uint32_t n_requests;
  uint32_t cursor, size;            // ring state before the first request
  uint32_t buffer_norm;             // importance weights relative to the whole tree (else to the batch)
  const per_request* queue;         // device copy of the requests
  FieldTable fields;                // columns, row sizes and access widths; the io pointers come from the requests
  uint32_t off[kMaxHeight + 2];     // as in StreamArgs
  uint32_t leaves_in_memory;
};

// Workgroup ranges of the jobs sharing one launch: [first[j], first[j+1]) for job j, where job 0 is the
// weights, job 1 the claim and job 2 + f the rows of payload field f.
struct JobRanges {
  uint32_t first[3 + kMaxFields];
  // Rows gathered whole (see move_whole_rows): rows per workgroup pass (0: every field has its own job), the
  // bytes of a stored row that cover the asked-for fields (from a 16-byte boundary, a multiple of 16), the field
  // that comes first in the row (its job range holds the workgroups) and the bytes between that boundary and it.
  uint32_t whole_rows, whole_span, whole_field, whole_lead;
};
constexpr uint32_t kWholeRowsLds = 8192;   // staging bytes of a workgroup that gathers whole rows

struct Range2 { uint32_t a0, b0, a1, b1; };   // two half-open node ranges [a0,b0) u [a1,b1)

// An insertion of a few rows carried by the sampling kernel of the call that follows it (see k_sample).  The
// caller fills the first part; launch_sample plans the rest.  Only for insertions that do not run past the ring's
// end: the touched nodes of a height are then one range, and their child groups one run of consecutive floats.
constexpr int kRideHeights = 4;   // (no fanout whose sampling kernel reaches the lazily rebuilt height has it higher)
constexpr uint32_t kRideNone = 0xFFFFFFFFu;
struct RideHeight {                // the touched nodes of one height: [a0, a0 + cnt)
  uint32_t a0, cnt;
  uint32_t off;                    // where their child groups start in the patch (floats); their new sums: val_off + off / K
  uint32_t top_at;                 // where this height starts in the sampling kernel's top copy (floats), or kRideNone
};
struct InsertRideHead {            // what the sampling workgroups read (the kernel fetches these argument lines first)
  uint32_t n, cursor;              // rows per tree, first ring slot
  const float* prio;               // [T][n] or null: the running maximum
  uint32_t* out_idx;               // [T][n] or null
  // planned by the launcher
  uint32_t hp;                     // heights 1 .. hp are patched (hp = the height the stale top is rebuilt from)
  uint32_t floats;                 // LDS floats of the patch: child groups, then new sums
  uint32_t val_off;                // where the new sums start
  uint32_t movers;                 // workgroups at the end of the grid that move the rows; the first also stores the patch
  RideHeight h[kRideHeights];      // h[i]: height i + 1 (unused: cnt 0)
};
struct InsertRide : InsertRideHead {
  FieldTable rows;                 // io all null: no rows to move (read by the one workgroup that moves them)
};

// Optional per-kernel timing with HIP events attached to each launch (off by default).
enum KernelId {
  KID_FILL, KID_SAMPLE, KID_WEIGHTS, KID_GATHER, KID_FINISH, KID_SCATTER, KID_INSERT_LEAVES, KID_RESUM_DENSE,
  KID_RESUM_TAIL, KID_UPDATE_CLAIM, KID_UPDATE_TREE, KID_TREE_FINISH, KID_UPDATE_DELTA, KID_GET_PRIORITY,
  KID_INSERT_SMALL, KID_RUN_STEPS, KID_RUN_REQUESTS, KID_MIN_REBUILD, KID_MIN_REDUCE, KID_STEP, KID_STEP_TABLES, KID_STEP_EPILOGUE, KID_COUNT
};
const char* kernel_name(int kid);

struct Profiler {
  struct Rec { hipEvent_t start, stop; int kid; };
  bool on = false;
  std::vector<Rec> recs;
  double total_ms[KID_COUNT] = {};
  uint64_t launches[KID_COUNT] = {};
  bool begin(int kid, hipEvent_t* start, hipEvent_t* stop);   // a fresh event pair for one launch (false: not profiling)
  void reset();                 // drops pending events and zeroes the totals
  hipError_t collect();         // waits for pending events and folds them into the totals
};

struct Tuning {
  uint32_t lds_budget_bytes;
  uint32_t sample_block, update_block, gather_block, tree_block;
  uint32_t sample_min_lds;   // lower bound of the sampling kernel's LDS request, bytes
  uint32_t lazy_top;   // updates may leave the few topmost heights to their next reader
  uint32_t insert_small;      // small inserts run as one kernel (one workgroup per tree)
  uint32_t claim_in_sample;   // fused steps may run the claim phase in the sampling kernel (two kernels per step)
  uint32_t group_claim;       // update batches claim through the group entries whenever they are short enough
  uint32_t insert_ride;       // per_insert_step lets its sampling kernel carry the insertion where that is possible
  uint32_t sample_block_auto; // sample_block is the default, not a size that was asked for
  uint32_t whole_rows;        // gathers of several fields move whole rows through LDS where the rows are short enough
  uint32_t step_tail;         // the one-kernel step also ends inside that kernel (rows, weights, tables) where all its workgroups fit the GPU at once
  uint32_t step_kernel;       // per_step runs sampling and update as one kernel: 0 never, 1 where it fits and pays off, 2 wherever it fits
  Profiler* prof;
  int device;                 // the device the buffer lives on
};

// Launchers (per_kernels.hip).  All enqueue on `s` and return hipGetLastError().
hipError_t launch_fill_u32(const Tuning& tn, uint32_t* p, uint64_t count, uint32_t value, hipStream_t s);
hipError_t launch_init_scalars(const Geom& g, float init_max, hipStream_t s);
hipError_t launch_min_rebuild(const Geom& g, const Tuning& tn, hipStream_t s);
hipError_t launch_min_reduce(const Geom& g, const Tuning& tn, uint32_t* weight_mode, hipStream_t s);
hipError_t static_scratch_address(int device, uint32_t** out);   // the static array of per_min_priority_static on `device` (which must be current)
hipError_t launch_sample(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, float beta, const float* u,
                         const RngArgs& rng,
                         uint32_t* out_idx, float* out_w, float* out_prio, uint32_t weight_mode, uint32_t stale_hb,
                         const FieldTable* rows, const ClaimArgs* claim, int claim_mode, hipStream_t s,
                         const InsertRide* ride = nullptr);
// True when the sampling kernel of a call with batch B can carry an insertion of n rows at ring slot cursor (ft: their
// fields, or null).
bool sample_can_carry_insert(const Geom& g, const Tuning& tn, uint32_t B, const FieldTable* ft, uint32_t n, uint32_t cursor);
hipError_t launch_gather(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t B, const uint32_t* idx,
                         hipStream_t s);
hipError_t launch_scatter(const Geom& g, const Tuning& tn, const FieldTable& ft, uint32_t n, uint32_t cursor,
                          hipStream_t s);
hipError_t launch_insert_leaves(const Geom& g, const Tuning& tn, uint32_t n, uint32_t cursor, const float* prio,
                                uint32_t* out_idx, hipStream_t s);
bool insert_fits_one_workgroup(const Geom& g, const FieldTable* ft, uint32_t n);
hipError_t launch_insert_small(const Geom& g, const Tuning& tn, const FieldTable* ft, uint32_t n, uint32_t cursor,
                               const float* prio, uint32_t* out_idx, uint32_t stale_hb, const uint32_t* protect,
                               uint32_t n_protect, bool track_min, hipStream_t s);
hipError_t launch_resum_ranges(const Geom& g, const Tuning& tn, Range2 r0, hipStream_t s);
hipError_t launch_resum_top(const Geom& g, const Tuning& tn, uint32_t hb, hipStream_t s);
uint32_t lazy_top_height(const Geom& g, const Tuning& tn);
hipError_t launch_update(const Geom& g, const Tuning& tn, const ClaimArgs& c, hipStream_t s);
hipError_t launch_update_delta(const Geom& g, const Tuning& tn, uint32_t B, uint32_t size, const uint32_t* idx,
                               const float* delta, hipStream_t s);
uint32_t step_fits(const Geom& g, uint32_t B, bool always);
hipError_t launch_step(const Geom& g, const Tuning& tn, uint32_t block, bool tables_valid, uint32_t B, uint32_t size,
                       float beta, const float* u, const RngArgs& rng, uint32_t* out_idx, float* out_w, float* out_prio,
                       uint32_t weight_mode, const FieldTable* rows, const float* upd_prio, const uint32_t* upd_pos,
                       hipStream_t s);
size_t step_table_bytes();
// The static array that holds one buffer's tables per GPU (see k_step): taken for `holder` if free (null otherwise,
// or when `device` is not the current one), and given back.
void* step_static_claim(const void* holder, int device, hipStream_t s);
void step_static_release(const void* holder, int device);
uint32_t stream_tree_floats(const Geom& g, uint32_t* off, uint32_t* leaves_in_memory = nullptr);
hipError_t launch_run_steps(const Geom& g, const Tuning& tn, const StreamArgs& a, hipStream_t s);
hipError_t launch_run_requests(const Geom& g, const Tuning& tn, const QueueArgs& a, hipStream_t s);
hipError_t launch_get_priority(const Geom& g, const Tuning& tn, uint32_t n, const uint32_t* idx, float* out, hipStream_t s);
hipError_t launch_read_scalars(const Geom& g, int which, uint32_t weight_mode, float* out, hipStream_t s);
hipError_t launch_clear_status(const Geom& g, hipStream_t s);

}  // namespace per
