/*
 * per.h -- C-ABI of the MI355X prioritized replay buffer (K-ary sum tree).
 *
 * The operations are the paper's Replay Manager requests (Section V-A:
 * priority sampling, priority retrieval, priority update, insertion) plus the
 * read of sampled rows from Data Storage (Section II-A "Learner"; Listing 2,
 * `sampled_data = D_storage[sampled_indices]`), batched over B requests and
 * over T independent buffers.
 *
 * Conventions
 *  - Pointers named d_* are DEVICE pointers owned by the caller; they must stay
 *    valid until the work enqueued by the call has finished.  All other
 *    pointers are HOST pointers.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Every
 *    call only enqueues work on `stream` and returns; nothing synchronises
 *    except per_status.  Calls on one buffer must be issued in order on one
 *    stream (or be ordered by the caller with events).
 *  - The library never allocates device memory: the caller provides one arena
 *    (per_arena_bytes tells how large) that holds the tree levels, the payload
 *    (stored row-major: the fields of a row side by side) and all scratch.
 *  - Arrays carry a leading tree dimension: "[T][B]" means T*B contiguous
 *    elements, tree-major.
 *  - Tree values are fp32.  The tree stores the value it is given (the caller
 *    applies any exponent alpha beforehand).  A K-child sum is the balanced
 *    pairwise fp32 sum over child positions, so results do not depend on the
 *    launch shape and equal those of a binary sum tree.
 *  - Return value: 0 on success; a negative PER_E* code on an error detected on
 *    the host, in which case no work was enqueued.  Conditions only the device
 *    can see set sticky bits (PER_FLAG_*) read by per_status.
 *  - A batch of size 0 is valid and enqueues nothing.
 *  - The ring cursor, the filled size and the call number of the generator of per_set_rng are kept
 *    on the host (they are pure functions of the call sequence) and enter the kernels as arguments.
 *    Calls may be captured into a HIP graph.  A captured insertion, or a captured sampling call that
 *    draws its own uniforms, stands for exactly the captured call: launch such a graph once, on the
 *    buffer state it was captured on.  Sampling with given uniforms, gather and the update forms carry
 *    no host state: a graph of them may be replayed any number of times with the inputs refilled in
 *    place, whatever ran on the buffer before the capture (what the host has noted about the device is
 *    not relied on while a stream is being captured).  Call per_note_replay after a replay and before
 *    the next call made outside the graph.
 */
#ifndef PER_H_
#define PER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PER_MAX_FIELDS 8

#define PER_OK       0
#define PER_EINVAL  (-1)  /* null/misaligned pointer, bad fanout, bad field table, bad beta ...   */
#define PER_ENOMEM  (-2)  /* arena too small                                                    */
#define PER_EEMPTY  (-3)  /* sample on a buffer that holds no rows                              */
#define PER_ERANGE  (-4)  /* insert of more rows than the capacity, height out of range ...     */
#define PER_EHIP    (-5)  /* a HIP call or kernel launch failed                                 */

#define PER_FLAG_BAD_INDEX    1u  /* index >= capacity (gather / get_priority) or >= size (update): element skipped;
                                     gather and get_priority write zeros for it                                   */
#define PER_FLAG_BAD_PRIORITY 2u  /* NaN, infinite or negative value: leaf write skipped                          */
#define PER_FLAG_ZERO_TOTAL   4u  /* sample on a tree whose root is not > 0: indices 0xFFFFFFFF, weights 0        */
#define PER_FLAG_GAVE_UP      8u  /* a bounded wait inside a kernel ran out (never seen; the call's update is then
                                     incomplete: rebuild the buffer from a saved state)                           */

typedef struct per_buffer per_t;   /* opaque host object */

typedef struct per_config {
  uint32_t struct_size;                 /* sizeof(per_config): ABI check                              */
  uint32_t fanout;                      /* K in {2,4,8,16,32,64} (the paper's "fanout", Listing 1)    */
  uint64_t capacity;                    /* N leaves per tree, 1 <= N <= 2^31 (the paper's "size")     */
  uint32_t n_trees;                     /* T >= 1 independent buffers                                 */
  uint32_t n_fields;                    /* payload fields per row, 0..PER_MAX_FIELDS; the caller's    */
                                        /* arrays are dense per field, the stored rows are row-major  */
  uint32_t field_bytes[PER_MAX_FIELDS]; /* bytes per row of each field, e.g. {68,24,4,68,1}           */
  float    init_max_priority;           /* value given to the first inserted rows; finite and > 0     */
} per_config;

/* Size and alignment the arena must have for this configuration. */
int per_arena_bytes(const per_config* cfg, size_t* bytes, size_t* align);

/* Lays the tree levels, payload columns and scratch out in `d_arena` (device memory,
 * at least per_arena_bytes large and aligned), zero-fills tree and scratch on `stream`
 * and returns a host handle.  The arena stays the caller's; it must outlive the handle.
 * Not for use while a stream is being captured.  A buffer with one tree may be given the library's static table
 * array (tuning "static_tables" below): the first time on a GPU that costs a small kernel and a wait for `stream`,
 * and when the array was held by another buffer before, a wait for the whole GPU. */
int per_create(const per_config* cfg, void* d_arena, size_t arena_bytes, void* stream, per_t** out);

/* Frees the host handle only. */
int per_destroy(per_t* p);

/* Insertion (Section V-A; Listing 2, "Populate Replay memory").  Row j of every tree goes
 * to ring slot (cursor + j) mod N; its leaf is set to d_prio[t][j], or, when d_prio is
 * NULL, to the running maximum of all valid values written so far (as it was when the
 * call started).  Ancestors are re-summed.  n <= N.
 *   d_field_src : HOST array of n_fields DEVICE pointers, each [T][n][field_bytes[f]];
 *                 may be NULL (or hold NULLs) to leave payload columns untouched.
 *   d_out_idx   : [T][n] slots written, or NULL.
 * An invalid explicit priority skips the leaf write (row is still stored) and sets
 * PER_FLAG_BAD_PRIORITY. */
int per_insert(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_prio,
               uint32_t* d_out_idx, void* stream);

/* Collision-free insertion (Section IV-B "Replay-Collision-Free Scheduling": insertions are scheduled
 * after sampling and the insertion index is compared against the sampled indices, so that rows the
 * Learner is still working on are not overwritten).  As per_insert, except that a row whose ring slot
 * is one of d_protect_idx[T][n_protect] (say, the batch sampled last and not yet updated) is deferred:
 * neither its payload nor its leaf is written, d_out_idx reports 0xFFFFFFFF for it, and the caller
 * keeps it for its next insertion.  The ring advances by n all the same.  What happens to a colliding
 * experience is not stated in the paper; this is the reading taken here.  Small inserts only
 * (at most 4096 rows and 256 KiB of payload per tree), else PER_ERANGE. */
int per_insert_protected(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_prio_or_null,
                         uint32_t* d_out_idx_or_null, uint32_t n_protect, const uint32_t* d_protect_idx,
                         void* stream);

/* Priority sampling (Eq. 1; Section V-A "traversing the tree performing prefix sum from
 * root to leaf"), stratified: sample i of a tree takes the target
 *   ((float)i + u[i]) * (total / (float)B)
 * and returns the leaf whose half-open prefix interval contains it.  Leaves with value 0
 * and slots never written are never returned.
 *   d_u          : [T][B] uniforms in [0,1); or NULL after per_set_rng: the call then draws its own
 *   d_out_idx    : [T][B]
 *   d_out_weight : [T][B] importance weights (size * P(i))^-beta divided by the batch
 *                  maximum, so the largest is 1; or NULL.  beta must be finite and >= 0.
 *   d_out_prio   : [T][B] value of each sampled leaf; or NULL. */
int per_sample(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx,
               float* d_out_weight, float* d_out_prio, void* stream);

/* Data Storage read: d_field_dst[f][t][i] = column f, row d_idx[t][i].
 *   d_field_dst : HOST array of n_fields DEVICE pointers, each [T][B][field_bytes[f]];
 *                 a NULL entry skips that column. */
int per_gather(per_t* p, uint32_t B, const uint32_t* d_idx, void* const* d_field_dst, void* stream);

/* per_sample followed by per_gather of the sampled indices, as one call (the paper's mode where
 * Replay Manager and consumer share a device, Section IV-A "setting 2"): the kernel that reads
 * the rows also finishes the importance weights, which saves a launch on the critical path.
 * Same arguments and results as the two separate calls. */
int per_sample_gather(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx,
                      float* d_out_weight, float* d_out_prio, void* const* d_field_dst, void* stream);

/* per_sample_gather followed by per_update(upd_B, d_upd_idx, d_upd_prio), as one call with the same
 * results (one iteration of Listing 2: draw a batch, read its rows, apply a priority update).  The
 * update's first phase (last-writer claim) touches nothing that sampling reads, so it runs inside
 * the sampling kernel, and the tree pass shares the second kernel with the row gather and the
 * importance weights: two launches for the whole step.  That holds when the update batch is the
 * sampled batch itself (d_upd_idx == d_out_idx and upd_B == B: update the rows just drawn, element i
 * gets d_upd_prio[i]) or lies in memory apart from d_out_idx / d_out_weight / d_out_prio (the
 * priorities computed for an earlier batch).  Any other overlap between the update batch and the
 * sampling outputs is still correct (the update then reads them after sampling has written them)
 * and costs a third launch.  d_field_dst may be NULL (no gather).  upd_B == 0 makes it
 * per_sample_gather. */
int per_sample_gather_update(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx,
                             float* d_out_weight, float* d_out_prio, void* const* d_field_dst,
                             uint32_t upd_B, const uint32_t* d_upd_idx, const float* d_upd_prio,
                             void* stream);

/* One whole iteration of the loop of Listing 2 (Section IV-D) in one call: draw a batch, read its rows, and
 * write back the priorities the Learner derived for that very batch.  Sampling, weights and rows as
 * per_sample_gather; then, as per_update, element j of the update sets the leaf drawn by sample
 * d_upd_pos[t][j] of this call to d_upd_prio[t][j] (d_upd_pos NULL: the leaf drawn by sample j), i.e. it is
 *   per_sample_gather(...);  upd_idx[t][j] = d_out_idx[t][d_upd_pos[t][j]];  per_update(B, upd_idx, d_upd_prio)
 * with the same results (last writer in order of j where several elements meet on a leaf).  A position
 * >= B makes its element invalid (PER_FLAG_BAD_INDEX), as does a sample that found nothing
 * (PER_FLAG_ZERO_TOTAL).  d_upd_prio and d_upd_pos are [T][B] and must not overlap the outputs
 * (PER_EINVAL).  d_field_dst and d_out_weight may be NULL. */
int per_step(per_t* p, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx, float* d_out_weight,
             float* d_out_prio, void* const* d_field_dst, const float* d_upd_prio, const uint32_t* d_upd_pos,
             void* stream);

/* per_insert(n, d_field_src, d_ins_prio, d_ins_out_idx) followed by per_step(...) as one call with the same results:
 * the iteration of Listing 2 (Section IV-D) with the Actors' new rows put in first (Section II-A: insertion at
 * the maximum priority, or at given values).  Where the insertion is small (at most 1024 rows per tree, few
 * touched nodes), the buffer's weights refer to the batch, and the tree's topmost heights are rebuilt lazily
 * (tuning "lazy_top"), the sampling kernel of the step carries the insertion: each of its workgroups works out
 * the few new nodes for itself and samples from the tree as the insertion leaves it, one of them stores them,
 * one extra workgroup moves the rows; the step then takes two kernel launches, insertion included.  For that the
 * insertion's arrays (d_field_src[f], d_ins_prio, d_ins_out_idx) must not overlap the step's outputs and
 * d_ins_out_idx none of the step's inputs either; otherwise, and for any other shape, the two calls are made one
 * after the other.  Arguments, flags and errors as for the two calls; an argument error of the step is
 * reported before the insertion is enqueued. */
int per_insert_step(per_t* p, uint32_t n, const void* const* d_field_src, const float* d_ins_prio,
                    uint32_t* d_ins_out_idx, uint32_t B, float beta, const float* d_u, uint32_t* d_out_idx,
                    float* d_out_weight, float* d_out_prio, void* const* d_field_dst, const float* d_upd_prio,
                    const uint32_t* d_upd_pos, void* stream);

/* Priority update (Section V-A), in the set-and-re-sum form: every valid element sets its
 * leaf; when an index occurs more than once the element latest in the batch wins;
 * afterwards every ancestor of a touched leaf equals the pairwise sum of its children.
 * Valid means d_idx < size and d_prio finite and >= 0. */
int per_update(per_t* p, uint32_t B, const uint32_t* d_idx, const float* d_prio, void* stream);

/* per_update from temporal-difference errors: the tree value of element j is
 * (|d_td[j]| + eps)^alpha, the priority of prioritized experience replay that the paper's sampling
 * follows (Section II-A: experiences are drawn in proportion to the policy loss), evaluated in fp64
 * on the device and rounded once to fp32; everything else as per_update.  A non-finite error is
 * skipped and flagged BAD_PRIORITY.  eps >= 0 and alpha >= 0, both finite, else PER_EINVAL. */
int per_update_td(per_t* p, uint32_t B, const uint32_t* d_idx /*[T][B]*/, const float* d_td /*[T][B]*/,
                  double eps, double alpha, void* stream);

/* Priority update in the paper's own form (Section V-A: "the inputs are the indices of the
 * experiences and the changes to their priorities"): d_delta[j] is added to the leaf d_idx[j] and to
 * every stored ancestor up to the root.  Together with per_get_priority it realises the paper's
 * "priority retrievals followed by priority updates": retrieve the old values, form
 * delta = new - old, apply.  Changes to the same node meet in no fixed order (hardware float
 * atomics), so a node equals the sequential result only up to fp32 rounding, no longer the
 * exact pairwise sum of its children; per_update restores that for the paths it touches.
 * Duplicated indices add up.  The running maximum priority is not touched (the call never sees a
 * priority).  Valid means d_idx < size and d_delta finite; other elements are skipped and flagged
 * (BAD_INDEX, BAD_PRIORITY).  The caller keeps leaves non-negative. */
int per_update_delta(per_t* p, uint32_t B, const uint32_t* d_idx /*[T][B]*/, const float* d_delta /*[T][B]*/,
                     void* stream);

/* A list of steps in one launch, for buffers small enough that a tree, or at least its heights above the
 * leaves, fits the LDS of one compute unit (about 150 KB: all of a tree of 32768 leaves at fanout 16; the
 * upper heights of one of 524288 leaves at fanout 16, of 2^20 at fanout 32, 2^21 at fanout 64).  The paper
 * keeps the sum tree of its Replay Manager in on-chip memory and lets a kernel that is started once work
 * through a stream of requests (Section V-A, "RM on FPGA": buffers of 10K to 100K entries); here one
 * workgroup per tree loads the tree, runs step after step against the LDS copy and stores it back at the
 * end; where only the upper heights fit, the leaves stay in memory and the workgroup, the only one that
 * touches the tree meanwhile, reads and writes them there.  Step s is, in this order,
 *   per_insert(n_insert rows)  ->  per_sample(B)  ->  per_gather  ->  per_update(B),
 * with the same results as those calls.  All arrays carry a leading step dimension:
 *   d_ins_rows   : [n_fields] device pointers, each [steps][T][n_insert][field_bytes]; NULL entries or a
 *                  NULL table skip the payload
 *   d_ins_prio   : [steps][T][n_insert] tree values of the new rows, or NULL: the running maximum
 *   d_u, d_beta  : [steps][T][B] uniforms in [0,1); [steps] exponents of the importance weights
 *   d_out_idx    : [steps][T][B];  d_out_weight, d_out_prio: same shape, or NULL
 *   d_rows_out   : [n_fields] device pointers, each [steps][T][B][field_bytes], or NULL
 *   d_upd_prio   : [steps][T][B] new tree values, or NULL: no update
 *   d_upd_idx    : [steps][T][B] indices to update; NULL with d_upd_prio given: step s updates the batch
 *                  it has just sampled
 * n_insert <= 1024 (0: no insertion), 1 <= B <= 1024.  PER_ERANGE when the tree does not fit
 * (per_run_steps_fits tells beforehand) or a count is out of range. */
typedef struct {
  uint32_t struct_size;            /* sizeof(per_stream_io) */
  const void* const* d_ins_rows;
  const float* d_ins_prio;
  const float* d_u;
  const float* d_beta;
  uint32_t* d_out_idx;
  float* d_out_weight;
  float* d_out_prio;
  void* const* d_rows_out;
  const uint32_t* d_upd_idx;
  const float* d_upd_prio;
} per_stream_io;
int per_run_steps(per_t* p, uint32_t n_steps, uint32_t n_insert, uint32_t B, const per_stream_io* io, void* stream);
int per_run_steps_fits(const per_t* p);   /* 1: the trees of this buffer fit (wholly, or above their leaves), 0: they do not */

/* A queue of op-coded requests in one launch (Section V-A, "RM on FPGA": the requests fed to the Replay
 * Manager carry a unified operation code and are decoded and executed as they stream in, by kernels
 * that are started once).  As per_run_steps: for buffers whose trees fit the LDS of a compute unit, one
 * workgroup per tree loads the tree, works through the queue in order against the LDS copy and stores
 * the tree back.  Request r is one of
 *   PER_OP_INSERT : per_insert of n rows (per_insert_protected when protect is given): field[f] are the
 *                   sources [T][n][bytes] (NULL entries skipped), prio [T][n] or NULL (running maximum),
 *                   idx receives the slots [T][n] (or NULL), protect [T][n_protect] or NULL
 *   PER_OP_SAMPLE : per_sample_gather of n samples: u [T][n] uniforms, beta, idx receives the indices
 *                   [T][n], out_weight / out_prio [T][n] or NULL, field[f] the destinations
 *                   [T][n][bytes] of the gathered rows (NULL entries skipped)
 *   PER_OP_UPDATE : per_update of n elements: idx [T][n] (NULL: the indices sampled by the latest SAMPLE
 *                   request of this queue, whose n must be the same), prio [T][n]
 * with the results of those calls issued one after the other.  1 <= n <= 1024.  All pointers are
 * device pointers; a field pointer must be aligned to the largest power of two (at most 16) that
 * divides the field's row size.
 *   h_requests : HOST array of n_requests requests: the call checks the arguments on it and derives the
 *                ring state (cursor, size) from it; read during the call only
 *   d_requests : the same queue in DEVICE memory (8-byte aligned), placed there by the caller: this is
 *                what the kernel decodes; it stays untouched until the work on `stream` is done
 * PER_ERANGE: a tree does not fit (per_run_steps_fits) or a count is out of range; PER_EINVAL:
 * unknown operation code, missing or misaligned pointer; PER_EEMPTY: a SAMPLE request would meet an
 * empty buffer.  Nothing is enqueued on an error. */
enum { PER_OP_INSERT = 1, PER_OP_SAMPLE = 2, PER_OP_UPDATE = 3 };
typedef struct per_request {
  uint32_t op;                   /* PER_OP_*                                                    */
  uint32_t n;                    /* rows, samples or elements per tree                          */
  float beta;                    /* SAMPLE: exponent of the importance weights                  */
  uint32_t n_protect;            /* INSERT: entries per tree of protect                         */
  const float* prio;             /* INSERT: values or NULL; UPDATE: new values                  */
  const float* u;                /* SAMPLE: uniforms in [0,1)                                   */
  uint32_t* idx;                 /* INSERT: slots out; SAMPLE: indices out; UPDATE: indices in  */
  float* out_weight;             /* SAMPLE, or NULL                                             */
  float* out_prio;               /* SAMPLE, or NULL                                             */
  const uint32_t* protect;       /* INSERT: slots not to be overwritten, or NULL                */
  void* field[PER_MAX_FIELDS];   /* INSERT: row sources; SAMPLE: row destinations               */
} per_request;
int per_run_requests(per_t* p, uint32_t n_requests, const per_request* h_requests, const per_request* d_requests,
                     void* stream);

/* Full bottom-up rebuild: every stored node above the leaves is recomputed from its children, level by
 * level, so that afterwards "a parent node stores the sum of priorities of its children" (Section V-A)
 * holds exactly (balanced pairwise fp32 sums), whatever was done to the tree before.  Needed after
 * per_update_delta, whose float atomics leave the upper levels equal to those sums only up to rounding;
 * also usable after the leaves of a restored arena were edited.  Streaming and coalesced: reads every
 * level once. */
int per_rebuild(per_t* p, void* stream);

/* Priority retrieval (Section V-A): d_out[t][i] = leaf d_idx[t][i]. */
int per_get_priority(per_t* p, uint32_t n, const uint32_t* d_idx, float* d_out, void* stream);

/* Copies the n_h real nodes of height `height` (0 = leaves, H = root) of one tree to d_out
 * (may be NULL to only query the count).  *count receives n_h. */
int per_read_level(per_t* p, uint32_t tree, uint32_t height, float* d_out, uint64_t* count,
                   void* stream);

/* d_out[t] = root of tree t. */
int per_total(per_t* p, float* d_out, void* stream);

/* d_out[t] = running maximum priority of tree t. */
int per_max_priority(per_t* p, float* d_out, void* stream);

/* Synchronises `stream` (the one the buffer's calls were issued on), then ORs the sticky device flags of all
 * trees into *flags.  The only call that waits for the device. */
int per_status(per_t* p, void* stream, uint32_t* flags);
int per_clear_status(per_t* p, void* stream);

/* Host-side mirrors (pure functions of the call sequence). */
uint32_t per_height(const per_t* p);     /* H                                   */
uint64_t per_size(const per_t* p);       /* filled rows per tree                */
uint64_t per_cursor(const per_t* p);     /* next ring slot                      */

/* Checkpoint / resume: a byte copy of the arena plus (cursor, size) is the whole state of a
 * buffer.  After the caller has copied a saved arena back, this sets the host mirrors to the
 * values saved with it.  cursor < N, size <= N.  Take the copy between calls (with the stream
 * idle): the scratch arrays of an update are all zero then, which the next update relies on. */
int per_set_ring(per_t* p, uint64_t cursor, uint64_t size);

/* What the importance weights of the sampling calls are relative to.  w_i = (size * P(i) / total)^-beta is
 * scaled by 1 / max w (prioritized experience replay, the method cited in Section II-A).
 *   PER_NORM_BATCH  (default): the maximum over the sampled batch, so the largest weight returned is 1;
 *   PER_NORM_BUFFER : the maximum over every stored row that can be sampled (priority > 0), the form
 *                     that implementations back with a min tree beside the sum tree.
 * Here the companion structure is the smallest positive leaf under every height-1 node, renewed by
 * per_update, the fused step and small inserts for the nodes they touch while this mode is on, rebuilt
 * from the leaves after calls that cannot (large inserts, per_update_delta, per_run_steps,
 * per_run_requests, per_set_ring), and reduced to one value per tree by a kernel in front of every
 * sampling call that returns weights.  per_run_steps and per_run_requests sweep the leaves (their LDS copy,
 * or memory) instead.  The mode applies to the calls made after it is set.
 * per_min_priority: d_out[t] = smallest positive leaf of tree t (+infinity if there is none). */
#define PER_NORM_BATCH  0
#define PER_NORM_BUFFER 1
int per_set_weight_norm(per_t* p, int mode);
int per_min_priority(per_t* p, float* d_out, void* stream);

/* per_min_priority for callers that must not allocate and cannot set memory aside for scratch (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the partial minima of the
 * reduction live in a static device array of the library (256 KiB on every GPU the library runs on, held
 * until the process ends) instead of the arena; no allocating call is made.  Same result as
 * per_min_priority.  At most 64 trees (PER_ERANGE beyond).  PER_EHIP if the array's device address could not
 * be obtained when the buffer was created.  All buffers on one GPU share the array, which keeps the last
 * call's contents (nothing in it has to start at zero: every word read is written by the call first):
 * calls that overlap in time on one GPU (different streams) race; issue them on one stream or order them. */
int per_min_priority_static(per_t* p, float* d_out, void* stream);

/* To be called after a captured graph holding calls on this buffer has been replayed and before the next
 * call made outside the graph: a replay changes the device without passing through the library, so
 * what the host has noted about the device (are the topmost heights current, is the companion minimum
 * current) is set to "no", and the next call rebuilds what it needs. */
int per_note_replay(per_t* p);

/* Uniforms drawn on the device ("uniformly generated random", Section II-A), for sampling calls that
 * pass d_u == NULL.  The generator is counter-based (Philox4x32-10), so the uniforms are a pure
 * function of (seed, number of the sampling call, tree, sample): sample i of tree t in call number c
 * uses the counter (i, c low word, c high word, t) under the key (seed low, seed high), and its
 * uniform is the first output word's top 24 bits times 2^-24.  next_call is the number the next such
 * call gets (0 at the start; the saved value when resuming).  per_rng_calls returns the current one. */
int per_set_rng(per_t* p, uint64_t seed, uint64_t next_call);
uint64_t per_rng_calls(const per_t* p);

/* Performance knobs; results never depend on them.
 *   "lds_budget_bytes" : upper tree levels are staged in LDS while they fit this many bytes
 *   "sample_block", "update_block", "gather_block" : workgroup sizes (multiples of 64, <= 1024).  Until "sample_block"
 *                  is set, a sampling launch that carries an insertion on 8 or more trees takes 512 lanes instead of
 *                  the default 128
 *   "tree_block" : workgroup size of the update's tree pass (multiple of 64, <= 1024; 0 = chosen per launch)
 *   "sample_min_lds" : lower bound in bytes of the sampling kernel's LDS request
 *   "group_stamp_next" : moves the device-side stamp counter of the claim group entries (1 .. 2^25; enqueued on
 *                  the default stream), e.g. close to the point where the entries are cleared and it starts over
 *   "group_claim" : how per_update and the fused step find the last writer of a leaf.  0: every element
 *                  raises the 64-bit stamp of its leaf; 1 (default): every element raises the entry shared
 *                  by a group of 32 leaves (64 for K = 64), an array small enough to stay in cache, and
 *                  goes to its leaf's own stamp only when two leaves of one group meet in a batch
 *                  (batches of more than 2^25 elements always use form 0)
 *   "lazy_top"   : 1 (default) lets per_update leave the few topmost heights to be rebuilt by
 *                  the next call that reads them; 0 makes per_update finish them itself
 *   "insert_small" : 1 (default) runs an insert of few rows as a single kernel, one workgroup per tree
 *   "step_tail"  : 1 lets the one-kernel step end inside that kernel (rows, weights and the next call's tables after a
 *                  wait of all its workgroups for each other) where all of them fit the GPU at once; 0 (default): a second
 *                  kernel does that, which was measured faster
 *   "insert_ride" : 1 (default) lets the sampling kernel of per_insert_step carry the insertion; 0: two calls
 *   "static_tables" : the per-owner tables of the one-kernel step live in the arena, or, for ONE buffer per GPU at a
 *                  time, in an array of the library's own at an address its kernels know without their arguments
 *                  (an owner then fetches its entry while the arguments are still on their way: about half a
 *                  microsecond per step).  per_create takes the array for a buffer with a single tree when nobody
 *                  holds it (per_destroy gives it back; when it changes hands the GPU is drained first, so that work
 *                  of the previous holder cannot meet the new one's).  0: give it back; 1: take it if it is free
 *                  (PER_ERANGE if another buffer holds it or the buffer has several trees).  Not while a stream is
 *                  being captured; graphs captured before the switch must not be replayed after it
 *   "whole_rows" : how a gather of two or more fields reads the stored rows.  0: one job per field; 1 (default):
 *                  from 16384 rows per call (all trees together), and where the asked-for fields lie within 512
 *                  bytes of a row, every sampled row is read once, as a whole, and each field's dense rows are
 *                  written from a copy in LDS; 2: that form wherever the rows fit (tests)
 *   "step_kernel" : how per_step (and per_sample_gather_update called with the sampled batch as its update batch)
 *                  runs.  1 (default): sampling and update as one kernel, one workgroup per subtree, with rows and
 *                  weights in a second, where the tree fits that kernel and the batch is large enough for it
 *                  to pay off (long runs of samples per subtree, few trees); 2: wherever the tree fits (tests);
 *                  0: always the separate kernels
 *   "claim_in_sample" : 1 (default) lets per_sample_gather_update run the first phase of its update
 *                  inside the sampling kernel (two kernels per step) whenever the update batch is the
 *                  sampled batch itself or lies apart from the sampling outputs; 0: always three kernels */
int per_set_tuning(per_t* p, const char* name, int64_t value);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch of this buffer carries a
 * pair of HIP events stamped at the start and end of the kernel's execution (this slows the
 * launches down, so whole-step times must be taken with profiling off).  per_profile(p, 1) clears the
 * totals and starts; per_profile(p, 0) stops.  per_profile_read waits for the recorded
 * events and fills, for each kernel launched since the totals were cleared, its name
 * (static string), summed duration in ms and launch count; *n_entries receives how many
 * kernels there are (entries beyond max_entries are not written). */
int per_profile(per_t* p, int enable);
int per_profile_read(per_t* p, uint32_t max_entries, const char** names, double* total_ms,
                     uint64_t* launches, uint32_t* n_entries);

const char* per_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PER_H_ */
