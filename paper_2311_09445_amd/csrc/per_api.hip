// C-ABI of the prioritized replay buffer: argument checks, arena layout and the host-side
// mirrors (ring cursor, fill count).  All device work is in per_kernels.hip.
#include <math.h>
#include <string.h>

#include <new>

#include "../../include/per.h"
#include "per_geom.h"

using namespace per;

struct per_buffer {
  per_config cfg;
  Geom g;
  Tuning tn;
  uint8_t* arena;
  size_t arena_bytes;
  uint8_t* col[kMaxFields];
  uint64_t col_stride[kMaxFields];
  uint32_t row_stride;
  uint64_t cursor, size;
  bool claims_left;          // a launch failed between a claim phase and its tree pass: the claim arrays are not all zero
  int weight_norm;           // PER_NORM_BATCH or PER_NORM_BUFFER
  bool min_stale;            // min1 does not describe the leaves (it is rebuilt when next needed)
  uint32_t stale_hb;         // != 0: the last update left the heights above this one to their next reader
  bool tables_valid;         // the per-owner tables of the one-kernel step describe the tree as it is
  unsigned long long capture_id;   // the stream capture the last call was recorded into (0: it ran eagerly)
  bool rng_on;               // per_set_rng was called: sampling calls without uniforms draw their own
  uint64_t rng_seed, rng_calls;   // key of the generator; number of sampling calls that drew from it
  int device;
  uint8_t* arena_tab;        // where the arena keeps the tables of the one-kernel step (they may sit in the kernels' static array instead)
  uint32_t* static_scratch;   // this device's copy of the static array of per_min_priority_static (null: its address could not be had)
  Profiler prof;
};

namespace {

constexpr size_t kAlign = 256;

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
  uint32_t logK, H;
  uint32_t n[kMaxHeight + 1];
  uint32_t stride[kMaxHeight + 1];
  size_t level_off[kMaxHeight + 1];
  size_t scalars_off, owner_off, nclaim_off, dirty_off, arrive_off, min1_off, side_off, tab_off, step_off, col_off[kMaxFields];
  uint32_t dirty_stride, arrive_stride, arrive_level_off[kMaxHeight + 1];
  uint64_t col_stride[kMaxFields];
  uint32_t row_stride;        // bytes between stored rows
  uint32_t owner_stride, nclaim_stride, min1_stride;
  size_t tree_end;            // bytes up to here are zero-filled as 32-bit words at create
  size_t total;
};

int check_config(const per_config* c) {
  if (!c || c->struct_size != sizeof(per_config)) return PER_EINVAL;
  const uint32_t K = c->fanout;
  if (K < 2 || K > 64 || (K & (K - 1))) return PER_EINVAL;
  if (c->capacity < 1 || c->capacity > (1ull << 31)) return PER_EINVAL;
  if (c->n_trees < 1 || c->n_trees > 65535) return PER_EINVAL;
  if (c->n_fields > PER_MAX_FIELDS) return PER_EINVAL;
  for (uint32_t f = 0; f < c->n_fields; ++f)
    if (c->field_bytes[f] == 0 || c->field_bytes[f] > (1u << 20)) return PER_EINVAL;
  if (!(c->init_max_priority > 0.0f) || !isfinite(c->init_max_priority)) return PER_EINVAL;
  return PER_OK;
}

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// widest power-of-two access (<= 16 bytes) that divides the row size and the pointer
uint32_t vec_width(uint32_t bytes, const void* io) {
  uint32_t v = 16;
  while (v > 1 && (bytes % v != 0 || misaligned(io, v))) v >>= 1;
  return v;
}

void make_layout(const per_config* c, Layout* L) {
  const uint32_t K = c->fanout, T = c->n_trees;
  L->logK = 0;
  while ((1u << L->logK) < K) L->logK++;
  uint64_t n = c->capacity;
  uint32_t h = 0;
  L->n[0] = (uint32_t)n;
  do {
    n = (n + K - 1) / K;
    L->n[++h] = (uint32_t)n;
  } while (n > 1);
  L->H = h;
  size_t off = 0;
  L->scalars_off = off;                         // max_v, status, vnext, vcur, sbase, sfloor, max_pend [T] each; vmin[2][T][kVminSlots], vmin_buf[T][kMinParts]
  off = round_up(off + (size_t)(7 + 2 * kVminSlots + kMinParts) * T * 4, kAlign);
  L->step_off = off;                            // the one-kernel step's words: cnt[T][kStepGroups] (64-bit), cnt2[T] (64-bit), done[T][2][kStepDoneSlots], vmin[T][2][kVminSlots], rel[T]
  off = round_up(off + (size_t)(2 * kStepGroups + 2 * kStepDoneSlots + 2 * kVminSlots + 4) * T * 4, kAlign);   // (+ cnt2 (64-bit), rel, a spare word)
  for (uint32_t l = 0; l <= L->H; ++l) {
    const uint64_t padded = ((uint64_t)L->n[l] + K - 1) / K * K;
    L->stride[l] = (uint32_t)round_up(padded, 64);
    L->level_off[l] = off;
    off = round_up(off + (size_t)L->stride[l] * T * 4, kAlign);
  }
  L->owner_stride = (uint32_t)round_up(c->capacity, 64);
  L->owner_off = off;
  off = round_up(off + (size_t)L->owner_stride * T * 8, kAlign);
  // one claim entry per 32 (padded) leaves, per 64 for K = 64
  L->nclaim_stride = (uint32_t)round_up(((size_t)L->n[1] * K + (K == 64 ? 63 : 31)) / (K == 64 ? 64 : 32), 64);
  L->nclaim_off = off;
  off = round_up(off + (size_t)L->nclaim_stride * T * 8, kAlign);
  L->dirty_stride = (uint32_t)round_up(((size_t)L->n[1] * K + 31) / 32, 64);   // one bit per (padded) leaf
  L->dirty_off = off;
  off = round_up(off + (size_t)L->dirty_stride * T * 4, kAlign);
  uint32_t counters = 0;
  for (uint32_t l = 0; l <= L->H; ++l) {
    L->arrive_level_off[l] = counters;
    if (l >= 2) counters += L->n[l];
  }
  L->arrive_stride = (uint32_t)round_up((size_t)counters + 1, 64);
  L->arrive_off = off;
  off = round_up(off + (size_t)L->arrive_stride * T * 4, kAlign);
  L->min1_stride = (uint32_t)round_up(L->n[1], 64);
  L->min1_off = off;
  off = round_up(off + (size_t)L->min1_stride * T * 4, kAlign);
  L->side_off = off;                            // where the owners of the one-kernel step leave their nodes of the owner height
  off = round_up(off + (size_t)kStepSideStride * T * 4, kAlign);
  L->tab_off = off;                             // its per-owner tables
  off = round_up(off + step_table_bytes(), kAlign);
  L->tree_end = off;
  // payload, row-major: every field at an offset aligned to the widest access its size allows, rows 16 bytes apart or a multiple
  uint32_t row = 0;
  uint32_t field_off[kMaxFields] = {};
  for (uint32_t f = 0; f < c->n_fields; ++f) {
    const uint32_t a = vec_width(c->field_bytes[f], nullptr);
    row = (uint32_t)round_up(row, a);
    field_off[f] = row;
    row += c->field_bytes[f];
  }
  L->row_stride = (uint32_t)round_up(row, 16);
  const size_t tree_rows = round_up((size_t)c->capacity * L->row_stride, kAlign);
  for (uint32_t f = 0; f < c->n_fields; ++f) {
    L->col_stride[f] = tree_rows;
    L->col_off[f] = off + field_off[f];
  }
  off += tree_rows * T;
  L->total = round_up(off, kAlign);
}

int fill_fields(per_t* p, void* const* io, FieldTable* ft) {
  memset(ft, 0, sizeof(*ft));
  ft->n_fields = p->cfg.n_fields;
  ft->row_stride = p->row_stride;
  bool any = false;
  for (uint32_t f = 0; f < ft->n_fields; ++f) {
    ft->col[f] = p->col[f];
    ft->col_stride[f] = p->col_stride[f];
    ft->bytes[f] = p->cfg.field_bytes[f];
    ft->io[f] = io ? static_cast<uint8_t*>(io[f]) : nullptr;
    ft->vec[f] = vec_width(ft->bytes[f], ft->io[f]);
    any = any || ft->io[f] != nullptr;
  }
  return any ? 1 : 0;
}

int hip_rc(hipError_t e) { return e == hipSuccess ? PER_OK : PER_EHIP; }

// True when min1 is being kept current, so that kernels rewriting leaves must renew it; a caller whose
// kernels cannot do that marks it stale instead.
bool tracks_min(const per_t* p) { return p->weight_norm == PER_NORM_BUFFER && !p->min_stale; }

// Brings vmin_buf up to date for a reader: min1 from the leaves if it is stale, then its reduction.  Returns the
// weight mode that tells the reader where the result is.
hipError_t reduce_min(per_t* p, hipStream_t s, uint32_t* weight_mode) {
  if (p->min_stale) {
    hipError_t e = launch_min_rebuild(p->g, p->tn, s);
    if (e != hipSuccess) return e;
    p->min_stale = false;
  }
  return launch_min_reduce(p->g, p->tn, weight_mode, s);
}

// Rebuilds the heights an update left stale, for readers that take them from memory.
hipError_t ensure_top(per_t* p, hipStream_t s) {
  if (!p->stale_hb) return hipSuccess;
  hipError_t e = launch_resum_top(p->g, p->tn, p->stale_hb, s);
  if (e == hipSuccess) p->stale_hb = 0;
  return e;
}

// A call made while its stream is being captured into a HIP graph does not run now and may run many times
// later, in between other work on the buffer.  What the host has noted about the device (are the topmost
// heights current, is the companion minimum current, are the step tables current) therefore says nothing
// about the state a replay starts from: it is all taken as "not current".  Rebuilding what is current is
// harmless, so a captured call is correct on every replay whatever ran before it.
void forget_device_notes(per_t* p) {
  const uint32_t hb = lazy_top_height(p->g, p->tn);
  if (hb) p->stale_hb = hb;
  p->min_stale = true;
  p->tables_valid = false;
}
// Before a tree pass: the heights it does not rewrite in full (up to its workgroup roots) must not be stale below
// those roots.
hipError_t prepare_tree_pass(per_t* p, hipStream_t s) {
  const uint32_t hb = lazy_top_height(p->g, p->tn);
  p->tables_valid = false;   // (the pass changes the tree)
  if (p->stale_hb && (!hb || p->stale_hb < hb)) return ensure_top(p, s);
  return hipSuccess;
}

// The notes are dropped when a call is the first of a capture (whatever ran before the graph's replays is not
// known) and when the first eager call follows captured ones (the graph may have been replayed any number of
// times, or never).  Between the calls of one capture they are kept: a replay runs those calls in that order.
struct CaptureGuard {
  CaptureGuard(per_t* p, hipStream_t s) {
    if (!p) return;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    unsigned long long id = 0;
    if (hipStreamGetCaptureInfo(s, &st, &id) != hipSuccess || st != hipStreamCaptureStatusActive) id = 0;
    else if (id == 0) id = ~0ull;
    if (id != p->capture_id) forget_device_notes(p);
    p->capture_id = id;
  }
};

// The tables of the one-kernel step in the kernels' static array (one buffer per GPU, single tree; see k_step): taken
// if free, never while `s` is being captured (changing hands may drain the device).
bool take_static_tables(per_t* p, hipStream_t s) {
  if (p->g.step_tab_static) return true;
  if (p->g.T != 1 || !p->g.step_ho) return false;
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone) return false;
  void* addr = step_static_claim(p, p->device, s);
  if (!addr) return false;
  p->g.step_tab = addr;
  p->g.step_tab_static = 1;
  p->tables_valid = false;
  return true;
}
void leave_static_tables(per_t* p) {
  if (!p->g.step_tab_static) return;
  step_static_release(p, p->device);
  p->g.step_tab = p->arena_tab;
  p->g.step_tab_static = 0;
  p->tables_valid = false;
}

}  // namespace

extern "C" {

int per_arena_bytes(const per_config* cfg, size_t* bytes, size_t* align) {
  int rc = check_config(cfg);
  if (rc != PER_OK) return rc;
  if (!bytes) return PER_EINVAL;
  Layout L;
  make_layout(cfg, &L);
  *bytes = L.total;
  if (align) *align = kAlign;
  return PER_OK;
}

int per_create(const per_config* cfg, void* d_arena, size_t arena_bytes, void* stream, per_t** out) {
  int rc = check_config(cfg);
  if (rc != PER_OK) return rc;
  if (!out || !d_arena || misaligned(d_arena, kAlign)) return PER_EINVAL;
  Layout L;
  make_layout(cfg, &L);
  if (arena_bytes < L.total) return PER_ENOMEM;

  per_t* p = new (std::nothrow) per_buffer();
  if (!p) return PER_ENOMEM;
  p->cfg = *cfg;
  p->arena = static_cast<uint8_t*>(d_arena);
  p->arena_bytes = arena_bytes;
  Geom& g = p->g;
  g.K = cfg->fanout;
  g.logK = L.logK;
  g.H = L.H;
  g.T = cfg->n_trees;
  g.N = (uint32_t)cfg->capacity;
  for (uint32_t l = 0; l <= L.H; ++l) {
    g.n[l] = L.n[l];
    g.stride[l] = L.stride[l];
    g.level[l] = reinterpret_cast<float*>(p->arena + L.level_off[l]);
  }
  g.root = g.level[L.H];
  g.root_stride = g.stride[L.H];
  g.owner = reinterpret_cast<uint64_t*>(p->arena + L.owner_off);
  g.owner_stride = L.owner_stride;
  g.nclaim = reinterpret_cast<uint2*>(p->arena + L.nclaim_off);
  g.nclaim_stride = L.nclaim_stride;
  g.dirty = reinterpret_cast<uint32_t*>(p->arena + L.dirty_off);
  g.dirty_stride = L.dirty_stride;
  g.arrive = reinterpret_cast<uint32_t*>(p->arena + L.arrive_off);
  g.arrive_stride = L.arrive_stride;
  for (uint32_t l = 0; l <= L.H; ++l) g.arrive_off[l] = L.arrive_level_off[l];
  g.max_v = reinterpret_cast<float*>(p->arena + L.scalars_off);
  g.status = reinterpret_cast<uint32_t*>(g.max_v + g.T);
  g.vnext = g.status + g.T;
  g.vcur = g.vnext + g.T;
  g.sbase = g.vcur + g.T;
  g.sfloor = g.sbase + g.T;
  g.max_pend = g.sfloor + g.T;
  g.vmin = g.max_pend + g.T;
  g.step_cnt = reinterpret_cast<unsigned long long*>(p->arena + L.step_off);
  g.step_cnt2 = g.step_cnt + (size_t)kStepGroups * g.T;
  g.step_done = reinterpret_cast<uint32_t*>(g.step_cnt2 + g.T);
  g.step_vmin = g.step_done + (size_t)2 * kStepDoneSlots * g.T;
  g.step_rel = g.step_vmin + (size_t)2 * kVminSlots * g.T;
  g.vmin_buf = g.vmin + (size_t)2 * kVminSlots * g.T;
  g.step_side = reinterpret_cast<float*>(p->arena + L.side_off);
  g.step_side_stride = kStepSideStride;
  p->arena_tab = p->arena + L.tab_off;
  g.step_tab = p->arena_tab;
  g.step_tab_static = 0;
  g.step_ho = step_owner_height(g);
  g.min1 = reinterpret_cast<uint32_t*>(p->arena + L.min1_off);
  g.min1_stride = L.min1_stride;
  for (uint32_t f = 0; f < cfg->n_fields; ++f) {
    p->col[f] = p->arena + L.col_off[f];
    p->col_stride[f] = L.col_stride[f];
  }
  p->row_stride = L.row_stride;
  p->tn.lds_budget_bytes = 64 * 1024;
  p->tn.sample_block = 128;   // (two waves: measured faster than four on large batches, 20.8 -> 20.1 us on the 65536-sample workload)
  p->tn.update_block = 256;
  p->tn.gather_block = 256;
  p->tn.tree_block = 0;   // chosen per launch
  p->tn.lazy_top = 1;
  p->tn.claim_in_sample = 1;
  p->tn.insert_small = 1;
  p->tn.group_claim = 1;
  p->tn.step_kernel = 1;
  p->tn.step_tail = 0;   // (measured slower than the second kernel: see k_step)
  p->tn.insert_ride = 1;
  p->tn.whole_rows = 1;
  p->tn.sample_block_auto = 1;
  p->tn.sample_min_lds = 0;
  p->tn.prof = &p->prof;
  p->claims_left = false;
  p->tables_valid = false;
  p->capture_id = 0;
  p->weight_norm = PER_NORM_BATCH;
  p->min_stale = true;
  if (hipGetDevice(&p->device) != hipSuccess) { delete p; return PER_EHIP; }
  p->tn.device = p->device;
  if (static_scratch_address(p->device, &p->static_scratch) != hipSuccess) p->static_scratch = nullptr;

  hipStream_t s = static_cast<hipStream_t>(stream);
  // zero everything (tree levels, stamps and payload), then the scalars
  hipError_t e = launch_fill_u32(p->tn, reinterpret_cast<uint32_t*>(p->arena), L.total / 4, 0u, s);
  if (e == hipSuccess) e = launch_init_scalars(g, cfg->init_max_priority, s);
  if (e != hipSuccess) { delete p; return PER_EHIP; }
  (void)take_static_tables(p, s);
  *out = p;
  return PER_OK;
}

int per_destroy(per_t* p) {
  if (!p) return PER_EINVAL;
  leave_static_tables(p);
  p->prof.reset();
  delete p;
  return PER_OK;
}

static int insert_impl(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_prio, uint32_t* d_out_idx,
                       uint32_t n_protect, const uint32_t* d_protect, void* stream) {
  if (!p) return PER_EINVAL;
  if (n > p->cfg.capacity) return PER_ERANGE;
  if (misaligned(d_prio, 4) || misaligned(d_out_idx, 4) || misaligned(d_protect, 4)) return PER_EINVAL;
  if (n == 0) return PER_OK;
  if (!d_protect) n_protect = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  p->tables_valid = false;   // (the insert changes the tree)
  const uint64_t N = p->cfg.capacity;
  const uint32_t cursor = (uint32_t)p->cursor;
  FieldTable ft;
  const bool has_rows = fill_fields(p, const_cast<void* const*>(reinterpret_cast<const void* const*>(d_field_src)), &ft);
  const bool one_workgroup = insert_fits_one_workgroup(p->g, has_rows ? &ft : nullptr, n);
  if (n_protect && !one_workgroup) return PER_ERANGE;   // the protected form exists for small inserts only
  if ((p->tn.insert_small || n_protect) && one_workgroup) {
    // one kernel: rows, leaves, ancestors, and the heights an update may have left stale
    hipError_t e1 = launch_insert_small(p->g, p->tn, has_rows ? &ft : nullptr, n, cursor, d_prio, d_out_idx, p->stale_hb,
                                        n_protect ? d_protect : nullptr, n_protect, tracks_min(p), s);
    if (e1 != hipSuccess) return PER_EHIP;   // nothing was enqueued: the mirrors stay
    p->stale_hb = 0;
    p->cursor = (p->cursor + n) % N;
    p->size = p->size + n > N ? N : p->size + n;
    return PER_OK;
  }
  p->min_stale = true;   // (the kernels of a large insert do not renew min1)
  hipError_t e = ensure_top(p, s);
  if (e == hipSuccess && has_rows) e = launch_scatter(p->g, p->tn, ft, n, cursor, s);
  if (e == hipSuccess) e = launch_insert_leaves(p->g, p->tn, n, cursor, d_prio, d_out_idx, s);
  if (e == hipSuccess) {
    Range2 r;
    const uint64_t end = p->cursor + n;
    r.a0 = cursor;
    r.b0 = (uint32_t)(end < N ? end : N);
    r.a1 = 0;
    r.b1 = (uint32_t)(end > N ? end - N : 0);
    e = launch_resum_ranges(p->g, p->tn, r, s);
  }
  // the mirrors advance even if a later launch failed: rows already enqueued have been placed
  p->cursor = (p->cursor + n) % N;
  p->size = p->size + n > N ? N : p->size + n;
  return hip_rc(e);
}

int per_insert(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_prio, uint32_t* d_out_idx,
               void* stream) {
  return insert_impl(p, n, d_field_src, d_prio, d_out_idx, 0, nullptr, stream);
}

int per_insert_protected(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_prio, uint32_t* d_out_idx,
                         uint32_t n_protect, const uint32_t* d_protect_idx, void* stream) {
  return insert_impl(p, n, d_field_src, d_prio, d_out_idx, n_protect, d_protect_idx, stream);
}

// Decides how an update batch claims its leaves.  The claim arrays are all zero between batches (the
// tree pass clears what its batch has set); should a launch have failed between a claim phase and its
// tree pass, they are cleared here first.
static int prepare_claim(per_t* p, uint32_t B, hipStream_t s, ClaimArgs* c) {
  const Geom& g = p->g;
  if (p->claims_left) {
    hipError_t e = launch_fill_u32(p->tn, reinterpret_cast<uint32_t*>(g.owner), 2ull * g.owner_stride * g.T, 0u, s);
    if (e == hipSuccess)
      e = launch_fill_u32(p->tn, reinterpret_cast<uint32_t*>(g.nclaim), 2ull * g.nclaim_stride * g.T, 0u, s);
    if (e == hipSuccess) e = launch_fill_u32(p->tn, g.dirty, (uint64_t)g.dirty_stride * g.T, 0u, s);
    if (e == hipSuccess) e = launch_fill_u32(p->tn, g.sbase, g.T, 1u, s);
    if (e != hipSuccess) return PER_EHIP;
    p->claims_left = false;
  }
  c->group_mode = B <= kGroupClaimMaxBatch && p->tn.group_claim ? 1u : 0u;
  c->track_min = tracks_min(p) ? 1u : 0u;   // (else min1 is, or now becomes, stale)
  if (!c->track_min) p->min_stale = true;
  return PER_OK;
}

static int check_update_args(per_t* p, uint32_t B, const uint32_t* d_idx, const float* d_prio) {
  if (!p) return PER_EINVAL;
  if (B == 0) return PER_OK;
  if (!d_idx || !d_prio || misaligned(d_idx, 4) || misaligned(d_prio, 4)) return PER_EINVAL;
  if ((uint64_t)B * 16 > 0x7FFFFFFFull) return PER_ERANGE;
  return PER_OK;
}

// true when byte ranges [a, a+na) and [b, b+nb) share a byte (null ranges share nothing)
static bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  if (!a || !b) return false;
  const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
  return x < y + nb && y < x + na;
}

static int sample_impl(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx, float* d_out_weight,
                       float* d_out_prio, void* const* d_field_dst, uint32_t upd_B, const uint32_t* d_upd_idx,
                       const float* d_upd_prio, void* stream, const uint32_t* d_upd_pos = nullptr,
                       const InsertRide* ride = nullptr) {
  // ride: an insertion that the sampling kernel of this call carries.  The caller (per_insert_step) has checked
  // the arguments and that the kernel can carry it, and has advanced the ring mirrors: p->size counts its rows.
  if (!p) return PER_EINVAL;
  if (B == 0) return PER_OK;
  if ((!d_u && !p->rng_on) || !d_out_idx || misaligned(d_u, 4) || misaligned(d_out_idx, 4) ||
      misaligned(d_out_weight, 4) || misaligned(d_out_prio, 4))
    return PER_EINVAL;
  if (!isfinite(beta) || beta < 0.0f) return PER_EINVAL;
  if ((uint64_t)B * 16 > 0x7FFFFFFFull) return PER_ERANGE;
  if (p->size == 0) return PER_EEMPTY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  FieldTable ft;
  const bool fused = d_field_dst && fill_fields(p, d_field_dst, &ft);
  // An update of exactly the batch drawn here (element for element, or through a position map), its values apart
  // from the outputs: sampling and update run as one kernel where that kernel fits the tree and the batch.
  uint32_t step_block = 0;
  if (upd_B == B && d_upd_idx == d_out_idx && p->tn.step_kernel && p->tn.lazy_top && !ride) {
    const size_t n_out = (size_t)p->g.T * B * 4;
    if (!ranges_overlap(d_upd_prio, n_out, d_out_idx, n_out) && !ranges_overlap(d_upd_prio, n_out, d_out_weight, n_out) &&
        !ranges_overlap(d_upd_prio, n_out, d_out_prio, n_out) && !ranges_overlap(d_upd_pos, n_out, d_out_idx, n_out) &&
        !ranges_overlap(d_upd_pos, n_out, d_out_weight, n_out) && !ranges_overlap(d_upd_pos, n_out, d_out_prio, n_out))
      step_block = step_fits(p->g, B, p->tn.step_kernel == 2);
  }
  if (step_block) {
    // the tables are built from the nodes of the owner height: when they are rebuilt, that height must not be stale
    if (!p->tables_valid && p->stale_hb && p->stale_hb < p->g.step_ho && ensure_top(p, s) != hipSuccess) return PER_EHIP;
    if (p->claims_left) {   // (the kernel's scratch words alias the leaf stamps, which must be zero)
      ClaimArgs none{};
      int rc = prepare_claim(p, B, s, &none);
      if (rc != PER_OK) return rc;
    }
  } else if (upd_B && prepare_tree_pass(p, s) != hipSuccess) {
    return PER_EHIP;
  }
  uint32_t weight_mode = 0;
  if (d_out_weight && p->weight_norm == PER_NORM_BUFFER &&   // the weights refer to the tree as it is before this call's update
      reduce_min(p, s, &weight_mode) != hipSuccess)
    return PER_EHIP;
  if (step_block) {
    RngArgs rng{};
    if (!d_u) {
      rng.on = 1;
      rng.seed_lo = (uint32_t)p->rng_seed;
      rng.seed_hi = (uint32_t)(p->rng_seed >> 32);
      rng.call_lo = (uint32_t)p->rng_calls;
      rng.call_hi = (uint32_t)(p->rng_calls >> 32);
      ++p->rng_calls;
    }
    hipError_t e = launch_step(p->g, p->tn, step_block, p->tables_valid, B, (uint32_t)p->size, beta, d_u, rng, d_out_idx,
                               d_out_weight, d_out_prio, weight_mode, fused ? &ft : nullptr, d_upd_prio, d_upd_pos, s);
    p->min_stale = true;   // (the kernel does not renew the companion minimum)
    if (e == hipSuccess) {
      p->stale_hb = 0;          // its epilogue has put every height in order
      p->tables_valid = true;   // and built the tables of the next step
    } else {
      p->tables_valid = false;
      p->stale_hb = lazy_top_height(p->g, p->tn);
      p->claims_left = true;
    }
    return hip_rc(e);
  }
  ClaimArgs claim{};
  int claim_mode = CLAIM_NONE;
  if (upd_B) {
    claim.B = upd_B;
    claim.size = (uint32_t)p->size;
    claim.idx = d_upd_idx;
    claim.pos = d_upd_pos;
    claim.prio = d_upd_prio;
    int rc = prepare_claim(p, upd_B, s, &claim);
    if (rc != PER_OK) return rc;
    // The claim phase reads the update batch.  It may run inside the sampling kernel when that
    // kernel does not write what it reads: the batch is either the sampled batch itself (same
    // index array, element for element) or lies apart from every output of the sampling kernel.
    const size_t n_out = (size_t)p->g.T * B * 4, n_upd = (size_t)p->g.T * upd_B * 4;
    const void* outs[3] = {d_out_idx, d_out_weight, d_out_prio};
    bool prio_apart = true, idx_apart = true;
    for (const void* o : outs) {
      prio_apart = prio_apart && !ranges_overlap(d_upd_prio, n_upd, o, n_out);
      idx_apart = idx_apart && !ranges_overlap(d_upd_idx, n_upd, o, n_out);
    }
    claim_mode = CLAIM_FINISH;
    if (p->tn.claim_in_sample && prio_apart && !d_upd_pos) {   // (through a position map an element needs another lane's sample)
      if (d_upd_idx == d_out_idx && upd_B == B) claim_mode = CLAIM_INLINE;
      else if (idx_apart) claim_mode = CLAIM_BLOCKS;
    }
  }
  RngArgs rng{};
  if (!d_u) {   // this call draws its own uniforms: call number rng_calls of the generator
    rng.on = 1;
    rng.seed_lo = (uint32_t)p->rng_seed;
    rng.seed_hi = (uint32_t)(p->rng_seed >> 32);
    rng.call_lo = (uint32_t)p->rng_calls;
    rng.call_hi = (uint32_t)(p->rng_calls >> 32);
    ++p->rng_calls;
  }
  // (a carried insertion changes the heights up to the lazily rebuilt one: the top is rebuilt from there whether
  // it was stale or not)
  const uint32_t stale = ride ? lazy_top_height(p->g, p->tn) : p->stale_hb;
  p->stale_hb = 0;   // the sampling kernel rebuilds and stores the stale heights
  hipError_t e = launch_sample(p->g, p->tn, B, (uint32_t)p->size, beta, d_u, rng, d_out_idx, d_out_weight, d_out_prio,
                               weight_mode, stale, fused ? &ft : nullptr, upd_B ? &claim : nullptr,
                               claim_mode, s, ride);
  if (e == hipSuccess && upd_B) p->stale_hb = lazy_top_height(p->g, p->tn);   // the tree pass ran
  if (e != hipSuccess && upd_B) p->claims_left = true;   // (the claim phase may have run without its tree pass)
  return hip_rc(e);
}

int per_sample(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx, float* d_out_weight,
               float* d_out_prio, void* stream) {
  return sample_impl(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, nullptr, 0, nullptr, nullptr, stream);
}

int per_sample_gather(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx, float* d_out_weight,
                      float* d_out_prio, void* const* d_field_dst, void* stream) {
  if (!d_field_dst) return PER_EINVAL;
  return sample_impl(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, d_field_dst, 0, nullptr, nullptr, stream);
}

int per_sample_gather_update(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx,
                             float* d_out_weight, float* d_out_prio, void* const* d_field_dst, uint32_t upd_B,
                             const uint32_t* d_upd_idx, const float* d_upd_prio, void* stream) {
  int rc = check_update_args(p, upd_B, d_upd_idx, d_upd_prio);
  if (rc != PER_OK) return rc;
  if (B == 0)   // nothing to sample: plain update
    return upd_B ? per_update(p, upd_B, d_upd_idx, d_upd_prio, stream) : PER_OK;
  return sample_impl(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, d_field_dst, upd_B, d_upd_idx, d_upd_prio,
                     stream);
}

int per_step(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx, float* d_out_weight,
             float* d_out_prio, void* const* d_field_dst, const float* d_upd_prio, const uint32_t* d_upd_pos,
             void* stream) {
  if (!p) return PER_EINVAL;
  if (B == 0) return PER_OK;
  if (!d_upd_prio || misaligned(d_upd_prio, 4) || misaligned(d_upd_pos, 4)) return PER_EINVAL;
  const size_t n = (size_t)p->g.T * B * 4;
  const void* outs[3] = {d_out_idx, d_out_weight, d_out_prio};
  for (const void* o : outs)   // the update's inputs are read after (and while) the outputs are written
    if (ranges_overlap(d_upd_prio, n, o, n) || ranges_overlap(d_upd_pos, n, o, n)) return PER_EINVAL;
  return sample_impl(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, d_field_dst, B, d_out_idx, d_upd_prio, stream,
                     d_upd_pos);
}

int per_insert_step(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_ins_prio, uint32_t* d_ins_out_idx,
                    uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx, float* d_out_weight, float* d_out_prio,
                    void* const* d_field_dst, const float* d_upd_prio, const uint32_t* d_upd_pos, void* stream) {
  if (!p) return PER_EINVAL;
  if (n == 0 || B == 0) {
    int rc = n ? per_insert(p, n, d_field_src, d_ins_prio, d_ins_out_idx, stream) : PER_OK;
    if (rc != PER_OK) return rc;
    return per_step(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, d_field_dst, d_upd_prio, d_upd_pos, stream);
  }
  // The step's arguments are checked before anything of the insertion is enqueued.
  if (n > p->cfg.capacity || (uint64_t)B * 16 > 0x7FFFFFFFull) return PER_ERANGE;
  if ((!d_u && !p->rng_on) || !d_out_idx || !d_upd_prio || !isfinite(beta) || beta < 0.0f) return PER_EINVAL;
  for (const void* a : {static_cast<const void*>(d_ins_prio), static_cast<const void*>(d_ins_out_idx),
                        static_cast<const void*>(d_u), static_cast<const void*>(d_out_idx),
                        static_cast<const void*>(d_out_weight), static_cast<const void*>(d_out_prio),
                        static_cast<const void*>(d_upd_prio), static_cast<const void*>(d_upd_pos)})
    if (misaligned(a, 4)) return PER_EINVAL;
  const size_t n_ins = (size_t)p->g.T * n * 4, n_out = (size_t)p->g.T * B * 4;
  const void* outs[3] = {d_out_idx, d_out_weight, d_out_prio};
  for (const void* o : outs)
    if (ranges_overlap(d_upd_prio, n_out, o, n_out) || ranges_overlap(d_upd_pos, n_out, o, n_out)) return PER_EINVAL;

  // The sampling kernel of the step carries the insertion where it can.  What the insertion reads and writes then
  // must lie apart from what the sampling kernel writes and reads, since the two run side by side.
  InsertRide ride{};
  const bool has_rows = fill_fields(p, const_cast<void* const*>(reinterpret_cast<const void* const*>(d_field_src)), &ride.rows);
  if (!has_rows) ride.rows = FieldTable{};
  bool carried = p->tn.insert_ride && p->weight_norm == PER_NORM_BATCH &&
                 sample_can_carry_insert(p->g, p->tn, B, has_rows ? &ride.rows : nullptr, n, (uint32_t)p->cursor);
  for (const void* o : outs) {
    carried = carried && !ranges_overlap(d_ins_prio, n_ins, o, n_out);
    if (has_rows)
      for (uint32_t f = 0; f < p->cfg.n_fields; ++f)
        carried = carried && !ranges_overlap(d_field_src[f], (size_t)p->g.T * n * p->cfg.field_bytes[f], o, n_out);
  }
  for (const void* a : {static_cast<const void*>(d_u), static_cast<const void*>(d_out_idx),
                        static_cast<const void*>(d_out_weight), static_cast<const void*>(d_out_prio),
                        static_cast<const void*>(d_upd_prio), static_cast<const void*>(d_upd_pos)})
    carried = carried && !ranges_overlap(d_ins_out_idx, n_ins, a, n_out);
  if (!carried) {
    int rc = per_insert(p, n, d_field_src, d_ins_prio, d_ins_out_idx, stream);
    if (rc != PER_OK) return rc;
    return per_step(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, d_field_dst, d_upd_prio, d_upd_pos, stream);
  }
  ride.n = n;
  ride.cursor = (uint32_t)p->cursor;
  ride.prio = d_ins_prio;
  ride.out_idx = d_ins_out_idx;
  const uint64_t N = p->cfg.capacity;
  const uint64_t cursor0 = p->cursor, size0 = p->size;
  p->cursor = (p->cursor + n) % N;                // (the step sees the ring as the insertion leaves it)
  p->size = p->size + n > N ? N : p->size + n;
  p->min_stale = true;                            // (the carried insertion does not renew the companion minimum)
  const int rc = sample_impl(p, B, beta, d_u, d_out_idx, d_out_weight, d_out_prio, d_field_dst, B, d_out_idx, d_upd_prio, stream,
                             d_upd_pos, &ride);
  if (rc != PER_OK && rc != PER_EHIP) {           // refused before anything was enqueued
    p->cursor = cursor0;
    p->size = size0;
  }
  return rc;
}

int per_gather(per_t* p, uint32_t B, const uint32_t* d_idx, void* const* d_field_dst, void* stream) {
  if (!p) return PER_EINVAL;
  if (B == 0) return PER_OK;
  if (!d_idx || misaligned(d_idx, 4) || !d_field_dst) return PER_EINVAL;
  FieldTable ft;
  if (!fill_fields(p, d_field_dst, &ft)) return PER_OK;
  return hip_rc(launch_gather(p->g, p->tn, ft, B, d_idx, static_cast<hipStream_t>(stream)));
}

int per_update(per_t* p, uint32_t B, const uint32_t* d_idx, const float* d_prio, void* stream) {
  int rc = check_update_args(p, B, d_idx, d_prio);
  if (rc != PER_OK || B == 0) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  if (prepare_tree_pass(p, s) != hipSuccess) return PER_EHIP;
  ClaimArgs claim{};
  claim.B = B;
  claim.size = (uint32_t)p->size;
  claim.idx = d_idx;
  claim.prio = d_prio;
  rc = prepare_claim(p, B, s, &claim);
  if (rc != PER_OK) return rc;
  hipError_t e = launch_update(p->g, p->tn, claim, s);
  if (e == hipSuccess) p->stale_hb = lazy_top_height(p->g, p->tn);
  else p->claims_left = true;   // (the claim phase may have run without its tree pass)
  return hip_rc(e);
}

int per_update_td(per_t* p, uint32_t B, const uint32_t* d_idx, const float* d_td, double eps, double alpha,
                  void* stream) {
  int rc = check_update_args(p, B, d_idx, d_td);
  if (rc != PER_OK || B == 0) return rc;
  if (!(eps >= 0.0) || !isfinite(eps) || !(alpha >= 0.0) || !isfinite(alpha)) return PER_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  if (prepare_tree_pass(p, s) != hipSuccess) return PER_EHIP;
  ClaimArgs claim{};
  claim.B = B;
  claim.size = (uint32_t)p->size;
  claim.idx = d_idx;
  claim.prio = d_td;
  claim.from_td = 1;
  claim.td_eps = eps;
  claim.td_alpha = alpha;
  rc = prepare_claim(p, B, s, &claim);
  if (rc != PER_OK) return rc;
  hipError_t e = launch_update(p->g, p->tn, claim, s);
  if (e == hipSuccess) p->stale_hb = lazy_top_height(p->g, p->tn);
  else p->claims_left = true;   // (the claim phase may have run without its tree pass)
  return hip_rc(e);
}

int per_update_delta(per_t* p, uint32_t B, const uint32_t* d_idx, const float* d_delta, void* stream) {
  int rc = check_update_args(p, B, d_idx, d_delta);
  if (rc != PER_OK || B == 0) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  p->min_stale = true;               // (changes added by atomics: min1 cannot follow them)
  p->tables_valid = false;
  hipError_t e = ensure_top(p, s);   // changes are added to whole nodes: the top heights must be current
  if (e == hipSuccess) e = launch_update_delta(p->g, p->tn, B, (uint32_t)p->size, d_idx, d_delta, s);
  return hip_rc(e);
}

int per_run_steps_fits(const per_t* p) { return p && stream_tree_floats(p->g, nullptr) ? 1 : 0; }

int per_run_steps(per_t* p, uint32_t n_steps, uint32_t n_insert, uint32_t B, const per_stream_io* io, void* stream) {
  if (!p || !io || io->struct_size != sizeof(per_stream_io)) return PER_EINVAL;
  if (n_steps == 0) return PER_OK;
  if (B == 0 || B > 1024 || n_insert > 1024 || n_insert > p->cfg.capacity) return PER_ERANGE;
  if (!stream_tree_floats(p->g, nullptr)) return PER_ERANGE;   // the tree does not fit the LDS of a compute unit
  if (!io->d_u || !io->d_beta || !io->d_out_idx || misaligned(io->d_u, 4) || misaligned(io->d_beta, 4) ||
      misaligned(io->d_out_idx, 4) || misaligned(io->d_out_weight, 4) || misaligned(io->d_out_prio, 4) ||
      misaligned(io->d_upd_idx, 4) || misaligned(io->d_upd_prio, 4) || misaligned(io->d_ins_prio, 4))
    return PER_EINVAL;
  if (io->d_upd_idx && !io->d_upd_prio) return PER_EINVAL;
  if (p->size == 0 && n_insert == 0) return PER_EEMPTY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  StreamArgs a{};
  a.n_steps = n_steps;
  a.n_insert = n_insert;
  a.B = B;
  a.cursor = (uint32_t)p->cursor;
  a.size = (uint32_t)p->size;
  a.upd_is_sampled = io->d_upd_prio && !io->d_upd_idx ? 1u : 0u;
  a.buffer_norm = p->weight_norm == PER_NORM_BUFFER ? 1u : 0u;
  p->min_stale = true;   // (the kernel works on an LDS copy of the leaves and does not keep min1)
  p->tables_valid = false;
  a.u = io->d_u;
  a.beta = io->d_beta;
  a.out_idx = io->d_out_idx;
  a.out_w = io->d_out_weight;
  a.out_prio = io->d_out_prio;
  a.upd_idx = io->d_upd_idx;
  a.upd_prio = io->d_upd_prio;
  a.ins_prio = io->d_ins_prio;
  if (n_insert) (void)fill_fields(p, const_cast<void* const*>(reinterpret_cast<const void* const*>(io->d_ins_rows)), &a.ins);
  (void)fill_fields(p, io->d_rows_out, &a.rows);
  hipError_t e = ensure_top(p, s);   // the kernel loads whole heights from memory
  if (e == hipSuccess) e = launch_run_steps(p->g, p->tn, a, s);
  const uint64_t N = p->cfg.capacity, added = (uint64_t)n_steps * n_insert;
  p->cursor = (p->cursor + added) % N;
  p->size = p->size + added > N ? N : p->size + added;
  return hip_rc(e);
}

int per_run_requests(per_t* p, uint32_t n_requests, const per_request* h_requests, const per_request* d_requests,
                     void* stream) {
  if (!p) return PER_EINVAL;
  if (n_requests == 0) return PER_OK;
  if (!h_requests || !d_requests || misaligned(d_requests, 8)) return PER_EINVAL;
  if (!stream_tree_floats(p->g, nullptr)) return PER_ERANGE;   // the tree does not fit the LDS of a compute unit
  QueueArgs a{};
  (void)fill_fields(p, nullptr, &a.fields);
  for (uint32_t f = 0; f < a.fields.n_fields; ++f) a.fields.vec[f] = vec_width(a.fields.bytes[f], nullptr);
  // a dry run over the host copy: argument checks and the ring state after every request
  const uint64_t N = p->cfg.capacity;
  uint64_t cursor = p->cursor, size = p->size;
  uint32_t sampled_n = 0;   // batch of the latest SAMPLE request (0: none yet)
  for (uint32_t r = 0; r < n_requests; ++r) {
    const per_request& q = h_requests[r];
    if (q.op != PER_OP_INSERT && q.op != PER_OP_SAMPLE && q.op != PER_OP_UPDATE) return PER_EINVAL;
    if (q.n == 0 || q.n > 1024) return PER_ERANGE;
    if (misaligned(q.prio, 4) || misaligned(q.u, 4) || misaligned(q.idx, 4) || misaligned(q.out_weight, 4) ||
        misaligned(q.out_prio, 4) || misaligned(q.protect, 4))
      return PER_EINVAL;
    if (q.op != PER_OP_UPDATE)
      for (uint32_t f = 0; f < a.fields.n_fields; ++f)
        if (misaligned(q.field[f], a.fields.vec[f])) return PER_EINVAL;
    if (q.op == PER_OP_INSERT) {
      if (q.n > N) return PER_ERANGE;
      cursor = (cursor + q.n) % N;
      size = size + q.n > N ? N : size + q.n;
    } else if (q.op == PER_OP_SAMPLE) {
      if (!q.u || !q.idx || !isfinite(q.beta) || q.beta < 0.0f) return PER_EINVAL;
      if (size == 0) return PER_EEMPTY;
      sampled_n = q.n;
    } else {
      if (!q.prio || (!q.idx && sampled_n != q.n)) return PER_EINVAL;
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  a.n_requests = n_requests;
  a.buffer_norm = p->weight_norm == PER_NORM_BUFFER ? 1u : 0u;
  p->min_stale = true;   // (as per_run_steps)
  p->tables_valid = false;
  a.cursor = (uint32_t)p->cursor;
  a.size = (uint32_t)p->size;
  a.queue = d_requests;
  hipError_t e = ensure_top(p, s);   // the kernel loads whole heights from memory
  if (e == hipSuccess) e = launch_run_requests(p->g, p->tn, a, s);
  p->cursor = cursor;
  p->size = size;
  return hip_rc(e);
}

int per_rebuild(per_t* p, void* stream) {
  if (!p) return PER_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  p->tables_valid = false;
  // all leaves count as touched: every height is recomputed in full, bottom-up
  hipError_t e = launch_resum_ranges(p->g, p->tn, Range2{0, p->g.N, 0, 0}, s);
  if (e != hipSuccess) return PER_EHIP;
  p->stale_hb = 0;
  return PER_OK;
}

int per_get_priority(per_t* p, uint32_t n, const uint32_t* d_idx, float* d_out, void* stream) {
  if (!p) return PER_EINVAL;
  if (n == 0) return PER_OK;
  if (!d_idx || !d_out || misaligned(d_idx, 4) || misaligned(d_out, 4)) return PER_EINVAL;
  return hip_rc(launch_get_priority(p->g, p->tn, n, d_idx, d_out, static_cast<hipStream_t>(stream)));
}

int per_read_level(per_t* p, uint32_t tree, uint32_t height, float* d_out, uint64_t* count, void* stream) {
  if (!p) return PER_EINVAL;
  if (tree >= p->g.T || height > p->g.H) return PER_ERANGE;
  if (count) *count = p->g.n[height];
  if (!d_out) return PER_OK;
  if (misaligned(d_out, 4)) return PER_EINVAL;
  CaptureGuard capture(p, static_cast<hipStream_t>(stream));
  if (p->stale_hb && height > p->stale_hb && ensure_top(p, static_cast<hipStream_t>(stream)) != hipSuccess)
    return PER_EHIP;
  const float* src = p->g.level[height] + (size_t)tree * p->g.stride[height];
  return hip_rc(hipMemcpyAsync(d_out, src, (size_t)p->g.n[height] * 4, hipMemcpyDeviceToDevice,
                               static_cast<hipStream_t>(stream)));
}

int per_total(per_t* p, float* d_out, void* stream) {
  if (!p || !d_out || misaligned(d_out, 4)) return PER_EINVAL;
  CaptureGuard capture(p, static_cast<hipStream_t>(stream));
  if (ensure_top(p, static_cast<hipStream_t>(stream)) != hipSuccess) return PER_EHIP;
  return hip_rc(launch_read_scalars(p->g, 0, 0, d_out, static_cast<hipStream_t>(stream)));
}

int per_max_priority(per_t* p, float* d_out, void* stream) {
  if (!p || !d_out || misaligned(d_out, 4)) return PER_EINVAL;
  return hip_rc(launch_read_scalars(p->g, 1, 0, d_out, static_cast<hipStream_t>(stream)));
}

int per_status(per_t* p, void* stream, uint32_t* flags) {
  if (!p || !flags) return PER_EINVAL;
  if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return PER_EHIP;
  uint32_t acc = 0;
  uint32_t buf[256];
  for (uint32_t t0 = 0; t0 < p->g.T; t0 += 256) {
    const uint32_t m = p->g.T - t0 < 256 ? p->g.T - t0 : 256;
    if (hipMemcpy(buf, p->g.status + t0, m * 4, hipMemcpyDeviceToHost) != hipSuccess) return PER_EHIP;
    for (uint32_t i = 0; i < m; ++i) acc |= buf[i];
  }
  *flags = acc;
  return PER_OK;
}

int per_clear_status(per_t* p, void* stream) {
  if (!p) return PER_EINVAL;
  return hip_rc(launch_clear_status(p->g, static_cast<hipStream_t>(stream)));
}

uint32_t per_height(const per_t* p) { return p ? p->g.H : 0; }
uint64_t per_size(const per_t* p) { return p ? p->size : 0; }
uint64_t per_cursor(const per_t* p) { return p ? p->cursor : 0; }

int per_set_ring(per_t* p, uint64_t cursor, uint64_t size) {
  if (!p) return PER_EINVAL;
  if (size > p->cfg.capacity || cursor >= p->cfg.capacity) return PER_ERANGE;
  p->cursor = cursor;
  p->size = size;
  p->stale_hb = lazy_top_height(p->g, p->tn);   // a saved arena may predate the rebuild of its top heights
  p->min_stale = true;
  p->tables_valid = false;
  return PER_OK;
}

int per_set_weight_norm(per_t* p, int mode) {
  if (!p || (mode != PER_NORM_BATCH && mode != PER_NORM_BUFFER)) return PER_EINVAL;
  p->weight_norm = mode;
  return PER_OK;
}

int per_min_priority(per_t* p, float* d_out, void* stream) {
  if (!p || !d_out || misaligned(d_out, 4)) return PER_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  uint32_t mode = 0;
  if (reduce_min(p, s, &mode) != hipSuccess) return PER_EHIP;
  return hip_rc(launch_read_scalars(p->g, 2, mode, d_out, s));
}

int per_min_priority_static(per_t* p, float* d_out, void* stream) {
  if (!p || !d_out || misaligned(d_out, 4)) return PER_EINVAL;
  if (p->g.T > kStaticMinTrees) return PER_ERANGE;   // more trees than the static array has room for
  if (!p->static_scratch) return PER_EHIP;           // the array's address on this device could not be had at create
  hipStream_t s = static_cast<hipStream_t>(stream);
  CaptureGuard capture(p, s);
  if (p->min_stale) {
    if (launch_min_rebuild(p->g, p->tn, s) != hipSuccess) return PER_EHIP;
    p->min_stale = false;
  }
  // the kernels of per_min_priority, with their partial minima in the static array instead of the arena; every
  // word the reader folds is written by the reduction first (plain stores), so nothing has to start at zero
  Geom g = p->g;
  g.vmin_buf = p->static_scratch;
  uint32_t mode = 0;
  if (launch_min_reduce(g, p->tn, &mode, s) != hipSuccess) return PER_EHIP;
  return hip_rc(launch_read_scalars(g, 2, mode, d_out, s));
}

int per_note_replay(per_t* p) {
  if (!p) return PER_EINVAL;
  forget_device_notes(p);   // a replayed update has left the topmost heights to their next reader, and so on
  return PER_OK;
}

int per_set_rng(per_t* p, uint64_t seed, uint64_t next_call) {
  if (!p) return PER_EINVAL;
  p->rng_on = true;
  p->rng_seed = seed;
  p->rng_calls = next_call;
  return PER_OK;
}

uint64_t per_rng_calls(const per_t* p) { return p ? p->rng_calls : 0; }

int per_set_tuning(per_t* p, const char* name, int64_t value) {
  if (!p || !name) return PER_EINVAL;
  if (!strcmp(name, "lds_budget_bytes")) {
    if (value < 0 || value > 160 * 1024) return PER_EINVAL;
    p->tn.lds_budget_bytes = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "group_stamp_next")) {   // test hook: move the device-side stamp counter of the group entries
    if (value < 1 || value > (int64_t)kGroupStampTurn) return PER_EINVAL;
    return hip_rc(launch_fill_u32(p->tn, p->g.sbase, p->g.T, (uint32_t)value, nullptr));
  }
  if (!strcmp(name, "sample_min_lds")) {
    if (value < 0 || value > 160 * 1024) return PER_EINVAL;
    p->tn.sample_min_lds = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "lazy_top")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    p->tn.lazy_top = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "insert_small")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    p->tn.insert_small = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "group_claim")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    p->tn.group_claim = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "step_tail")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    p->tn.step_tail = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "static_tables")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    if (value == 0) {
      leave_static_tables(p);
      return PER_OK;
    }
    return take_static_tables(p, nullptr) ? PER_OK : PER_ERANGE;
  }
  if (!strcmp(name, "whole_rows")) {
    if (value < 0 || value > 2) return PER_EINVAL;
    p->tn.whole_rows = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "insert_ride")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    p->tn.insert_ride = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "step_kernel")) {
    if (value < 0 || value > 2) return PER_EINVAL;
    p->tn.step_kernel = (uint32_t)value;
    return PER_OK;
  }
  if (!strcmp(name, "claim_in_sample")) {
    if (value != 0 && value != 1) return PER_EINVAL;
    p->tn.claim_in_sample = (uint32_t)value;
    return PER_OK;
  }
  uint32_t* blk = !strcmp(name, "sample_block") ? &p->tn.sample_block
                : !strcmp(name, "update_block") ? &p->tn.update_block
                : !strcmp(name, "gather_block") ? &p->tn.gather_block
                : !strcmp(name, "tree_block") ? &p->tn.tree_block : nullptr;
  if (!blk) return PER_EINVAL;
  if (blk == &p->tn.tree_block && value == 0) { *blk = 0; return PER_OK; }
  if (value < 64 || value > 1024 || value % 64) return PER_EINVAL;
  *blk = (uint32_t)value;
  if (blk == &p->tn.sample_block) p->tn.sample_block_auto = 0;
  return PER_OK;
}

int per_profile(per_t* p, int enable) {
  if (!p) return PER_EINVAL;
  p->prof.reset();
  p->prof.on = enable != 0;
  return PER_OK;
}

int per_profile_read(per_t* p, uint32_t max_entries, const char** names, double* total_ms, uint64_t* launches,
                     uint32_t* n_entries) {
  if (!p || !n_entries || (max_entries && (!names || !total_ms || !launches))) return PER_EINVAL;
  if (p->prof.collect() != hipSuccess) return PER_EHIP;
  uint32_t n = 0;
  for (int k = 0; k < KID_COUNT; ++k) {
    if (p->prof.launches[k] == 0) continue;
    if (n < max_entries) {
      names[n] = kernel_name(k);
      total_ms[n] = p->prof.total_ms[k];
      launches[n] = p->prof.launches[k];
    }
    ++n;
  }
  *n_entries = n;
  return PER_OK;
}

const char* per_strerror(int code) {
  switch (code) {
    case PER_OK: return "ok";
    case PER_EINVAL: return "invalid argument";
    case PER_ENOMEM: return "arena too small";
    case PER_EEMPTY: return "buffer holds no rows";
    case PER_ERANGE: return "size out of range";
    case PER_EHIP: return "HIP call or kernel launch failed";
    default: return "unknown error";
  }
}

}  // extern "C"
