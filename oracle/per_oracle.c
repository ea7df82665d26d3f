/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * Plain, slow, single-threaded CPU reference for the prioritized replay
 * buffer's sum tree (the paper's "Replay Manager" operations of Section V-A:
 * priority sampling, priority retrieval, priority update, insertion) and the
 * row gather from "Data Storage" (Section II-A).  Only tests, the smoke check
 * and the bench's cpu_baseline leg may load it.  It shares no code, header,
 * table or helper with the HIP library.
 *
 * What it is: the textbook binary sum tree of prioritized experience replay
 * in a heap array, fp32, "a parent node stores the sum of priorities of its
 * children" (Section V-A), left operand first:
 *
 *     tree[1] root, children of i are 2i and 2i+1, leaf j at tree[P + j].
 *
 * A K-ary tree whose K-child sum is taken as the balanced pairwise sum over
 * child positions ((c0+c1)+(c2+c3))+... is this same binary tree with only
 * every log2(K)-th level kept.  The fanout therefore changes nothing in the
 * arithmetic here; it only decides which binary depths are "stored levels"
 * (oracle_read_level) and how many padded leaves P = K^H there are.
 *
 * Readings the paper leaves open (Eq. 1 and Section V-A), fixed here:
 *   - leaves are 0-based; sample i selects the leaf whose half-open prefix
 *     interval [prefix(i-1), prefix(i)) contains the target (go left iff
 *     r < L), and a subtree whose sum is 0 is never entered;
 *   - targets are stratified: t_i = ((float)i + u_i) * (total / (float)B);
 *   - update *sets* the leaf and re-sums its ancestors, batch order, so the last
 *     writer of a duplicated index wins (the paper's delta propagation is a
 *     separate operation, oracle_update_delta);
 *   - new rows get the running maximum of all values ever written;
 *   - importance weights are normalised by the batch maximum, in fp64; on request
 *     (oracle_set_weight_norm) by the maximum over the whole buffer instead, i.e. over
 *     every stored row that can be sampled at all (priority > 0).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_FIELDS 8
#define ORACLE_FLAG_BAD_INDEX    1u
#define ORACLE_FLAG_BAD_PRIORITY 2u
#define ORACLE_FLAG_ZERO_TOTAL   4u

typedef struct {
  uint32_t K, logK, H, HB;   /* fanout, log2 fanout, K-ary height, binary height */
  uint64_t N, P;             /* capacity, padded leaf count K^H                    */
  float*   tree;             /* 2P floats, heap order                              */
  uint32_t n_fields;
  uint32_t field_bytes[ORACLE_MAX_FIELDS];
  uint8_t* col[ORACLE_MAX_FIELDS];   /* N * field_bytes each, or NULL (no payload) */
  uint64_t cursor, size;
  float    max_v;
  uint32_t status;
  int      weight_norm;      /* 0: weights relative to the batch maximum, 1: to the buffer-wide one */
} oracle_t;

static int valid_priority(float v) { return isfinite(v) && v >= 0.0f; }

oracle_t* oracle_create(uint32_t K, uint64_t N, uint32_t n_fields,
                        const uint32_t* field_bytes, float init_max, int with_payload) {
  if (K < 2 || (K & (K - 1)) || N < 1 || n_fields > ORACLE_MAX_FIELDS) return NULL;
  oracle_t* o = (oracle_t*)calloc(1, sizeof(oracle_t));
  if (!o) return NULL;
  o->K = K;
  while ((1u << o->logK) < K) o->logK++;
  o->N = N;
  /* H = smallest h >= 1 with ceil(N / K^h) == 1 */
  uint64_t n = N;
  o->H = 0;
  do { n = (n + K - 1) / K; o->H++; } while (n > 1);
  o->HB = o->H * o->logK;
  o->P = (uint64_t)1 << o->HB;
  o->tree = (float*)calloc(2 * o->P, sizeof(float));
  if (!o->tree) { free(o); return NULL; }
  o->n_fields = n_fields;
  for (uint32_t f = 0; f < n_fields; ++f) {
    o->field_bytes[f] = field_bytes[f];
    if (with_payload) {
      o->col[f] = (uint8_t*)calloc(N, field_bytes[f]);
      if (!o->col[f]) return NULL;
    }
  }
  o->max_v = init_max;
  return o;
}

void oracle_destroy(oracle_t* o) {
  if (!o) return;
  for (uint32_t f = 0; f < ORACLE_MAX_FIELDS; ++f) free(o->col[f]);
  free(o->tree);
  free(o);
}

/* Set one leaf and re-sum every ancestor as left child + right child. */
static void set_leaf(oracle_t* o, uint64_t idx, float v) {
  float* t = o->tree;
  uint64_t i = o->P + idx;
  t[i] = v;
  for (i >>= 1; i >= 1; i >>= 1) t[i] = t[2 * i] + t[2 * i + 1];
}

/* Priority update (Section V-A), as set + re-sum; sequential batch order. */
void oracle_update(oracle_t* o, uint32_t B, const uint32_t* idx, const float* prio) {
  for (uint32_t j = 0; j < B; ++j) {
    if (!(idx[j] < o->size)) { o->status |= ORACLE_FLAG_BAD_INDEX; continue; }
    if (!valid_priority(prio[j])) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
    set_leaf(o, idx[j], prio[j]);
    if (prio[j] > o->max_v) o->max_v = prio[j];
  }
}

/* Priority update from temporal-difference errors: the priority of prioritized experience replay
 * (cited in Section II-A), value = (|td| + eps)^alpha, evaluated in fp64 and rounded once to fp32,
 * then the set-and-re-sum update above.  Valid means idx < size and td finite. */
void oracle_update_td(oracle_t* o, uint32_t B, const uint32_t* idx, const float* td, double eps, double alpha) {
  for (uint32_t j = 0; j < B; ++j) {
    if (!(idx[j] < o->size)) { o->status |= ORACLE_FLAG_BAD_INDEX; continue; }
    if (!isfinite(td[j])) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
    const float v = (float)pow(fabs((double)td[j]) + eps, alpha);
    if (!valid_priority(v)) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
    set_leaf(o, idx[j], v);
    if (v > o->max_v) o->max_v = v;
  }
}

/* Priority update in the paper's own form (Section V-A): the inputs are indices and changes
 * delta; every node on the path from the root down to the leaf gets the change added, level by
 * level.  Sequential batch order; duplicated indices simply add up.  Unlike the set-and-re-sum
 * form above, a node is then no longer the rounded sum of its children but the running result of
 * its own additions, so two orders of the same batch may differ in the last bits.  The running
 * maximum is left alone (the operation never sees a priority, only its change).  Valid means
 * idx < size and delta finite. */
void oracle_update_delta(oracle_t* o, uint32_t B, const uint32_t* idx, const float* delta) {
  float* t = o->tree;
  for (uint32_t j = 0; j < B; ++j) {
    if (!(idx[j] < o->size)) { o->status |= ORACLE_FLAG_BAD_INDEX; continue; }
    if (!isfinite(delta[j])) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
    const uint64_t leaf = o->P + idx[j];
    for (uint32_t depth = 0; depth <= o->HB; ++depth) {   /* root (depth 0) first, leaf last */
      const uint64_t node = leaf >> (o->HB - depth);
      t[node] = t[node] + delta[j];
    }
  }
}

/* Insertion (Section V-A; Listing 2 "Populate Replay memory"): ring slots,
 * rows into Data Storage, leaf = explicit value or the running max on entry. */
int oracle_insert(oracle_t* o, uint32_t n, const void* const* field_src,
                  const float* prio_or_null, uint32_t* out_idx_or_null) {
  if (n > o->N) return -4;
  const float m = o->max_v;
  for (uint32_t j = 0; j < n; ++j) {
    uint64_t slot = (o->cursor + j) % o->N;
    for (uint32_t f = 0; f < o->n_fields; ++f)
      if (o->col[f] && field_src && field_src[f])
        memcpy(o->col[f] + slot * o->field_bytes[f],
               (const uint8_t*)field_src[f] + (uint64_t)j * o->field_bytes[f], o->field_bytes[f]);
    if (out_idx_or_null) out_idx_or_null[j] = (uint32_t)slot;
    if (prio_or_null) {
      if (!valid_priority(prio_or_null[j])) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
      set_leaf(o, slot, prio_or_null[j]);
    } else {
      set_leaf(o, slot, m);
    }
  }
  if (prio_or_null)
    for (uint32_t j = 0; j < n; ++j)
      if (valid_priority(prio_or_null[j]) && prio_or_null[j] > o->max_v) o->max_v = prio_or_null[j];
  o->cursor = (o->cursor + n) % o->N;
  o->size = (o->size + n > o->N) ? o->N : o->size + n;
  return 0;
}

/* Collision-free insertion (Section IV-B, "Replay-Collision-Free Scheduling": the insertion index is
 * compared against the sampled indices so that rows the Learner is still working on are not
 * overwritten).  The paper does not say what happens to a colliding experience; the reading here:
 * row j targets ring slot (cursor + j) mod N as always; if that slot is one of the protected
 * indices the row is deferred (nothing is written, out_idx[j] = 0xFFFFFFFF, the caller keeps it
 * for the next insertion), and the ring advances by n all the same. */
int oracle_insert_protected(oracle_t* o, uint32_t n, const void* const* field_src, const float* prio_or_null,
                            uint32_t* out_idx_or_null, uint32_t n_protect, const uint32_t* protect) {
  if (n > o->N) return -4;
  const float m = o->max_v;
  for (uint32_t j = 0; j < n; ++j) {
    uint64_t slot = (o->cursor + j) % o->N;
    int deferred = 0;
    for (uint32_t k = 0; k < n_protect && !deferred; ++k) deferred = protect[k] == slot;
    if (deferred) {
      if (out_idx_or_null) out_idx_or_null[j] = 0xFFFFFFFFu;
      continue;
    }
    for (uint32_t f = 0; f < o->n_fields; ++f)
      if (o->col[f] && field_src && field_src[f])
        memcpy(o->col[f] + slot * o->field_bytes[f],
               (const uint8_t*)field_src[f] + (uint64_t)j * o->field_bytes[f], o->field_bytes[f]);
    if (out_idx_or_null) out_idx_or_null[j] = (uint32_t)slot;
    if (prio_or_null) {
      if (!valid_priority(prio_or_null[j])) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
      set_leaf(o, slot, prio_or_null[j]);
      if (prio_or_null[j] > o->max_v) o->max_v = prio_or_null[j];
    } else {
      set_leaf(o, slot, m);
    }
  }
  o->cursor = (o->cursor + n) % o->N;
  o->size = (o->size + n > o->N) ? o->N : o->size + n;
  return 0;
}

/* Priority sampling (Eq. 1 via root-to-leaf prefix-sum traversal, Section V-A),
 * stratified targets, plus importance weights. */
int oracle_sample(oracle_t* o, uint32_t B, float beta, const float* u, uint32_t* out_idx,
                  float* out_weight_or_null, float* out_prio_or_null) {
  const float* t = o->tree;
  const float total = t[1];
  if (!(total > 0.0f)) {
    o->status |= ORACLE_FLAG_ZERO_TOTAL;
    for (uint32_t i = 0; i < B; ++i) {
      out_idx[i] = 0xFFFFFFFFu;
      if (out_weight_or_null) out_weight_or_null[i] = 0.0f;
      if (out_prio_or_null) out_prio_or_null[i] = 0.0f;
    }
    return 0;
  }
  const float seg = total / (float)B;
  double* wt = out_weight_or_null ? (double*)malloc(sizeof(double) * B) : NULL;
  double wmax = 0.0;
  for (uint32_t i = 0; i < B; ++i) {
    float pos = (float)i + u[i];
    float r = pos * seg;
    uint64_t node = 1;
    while (node < o->P) {
      float L = t[2 * node], R = t[2 * node + 1];
      if (R == 0.0f) node = 2 * node;
      else if (r < L) node = 2 * node;
      else { r = r - L; node = 2 * node + 1; }
    }
    float v = t[node];
    out_idx[i] = (uint32_t)(node - o->P);
    if (out_prio_or_null) out_prio_or_null[i] = v;
    if (wt) {
      wt[i] = pow((double)o->size * (double)v / (double)total, -(double)beta);
      if (wt[i] > wmax) wmax = wt[i];
    }
  }
  if (wt && o->weight_norm == 1) {
    /* the largest weight any stored row could get: rows that cannot be sampled (priority 0) have none */
    wmax = 0.0;
    for (uint64_t j = 0; j < o->size; ++j) {
      const float v = t[o->P + j];
      if (v > 0.0f) {
        const double w = pow((double)o->size * (double)v / (double)total, -(double)beta);
        if (w > wmax) wmax = w;
      }
    }
  }
  if (wt) {
    for (uint32_t i = 0; i < B; ++i) out_weight_or_null[i] = (float)(wt[i] / wmax);
    free(wt);
  }
  return 0;
}

/* Importance weights w_i = (size * P(i) / total)^-beta are scaled by 1 / max w "for stability" (prioritized
 * experience replay, the method cited in Section II-A); mode 0 takes the maximum over the sampled
 * batch, mode 1 over all stored rows with a positive priority. */
int oracle_set_weight_norm(oracle_t* o, int mode) {
  if (mode != 0 && mode != 1) return -1;
  o->weight_norm = mode;
  return 0;
}

/* Uniforms from a counter-based generator instead of an input array ("uniformly generated random",
 * Section II-A).  Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
 * 1, 2, 3", SC 2011): ten rounds of two 32x32->64 multiplications on a 4-word counter, the 2-word
 * key bumped by Weyl constants between rounds.  Sample i of tree t in sampling call number `call`
 * uses the counter (i, call low, call high, t) and the key (seed low, seed high); its uniform is
 * the first output word, (x >> 8) * 2^-24. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void oracle_uniforms(uint64_t seed, uint64_t call, uint32_t tree, uint32_t B, float* u) {
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  for (uint32_t i = 0; i < B; ++i) {
    const uint32_t ctr[4] = {i, (uint32_t)call, (uint32_t)(call >> 32), tree};
    uint32_t x[4];
    oracle_philox4x32_10(ctr, key, x);
    u[i] = (float)(x[0] >> 8) * (1.0f / 16777216.0f);
  }
}

/* Data Storage read: sampled_data = D_storage[sampled_indices] (Listing 2). */
void oracle_gather(oracle_t* o, uint32_t B, const uint32_t* idx, void* const* field_dst) {
  for (uint32_t f = 0; f < o->n_fields; ++f) {
    if (!o->col[f] || !field_dst[f]) continue;
    const uint32_t E = o->field_bytes[f];
    for (uint32_t i = 0; i < B; ++i) {
      uint8_t* d = (uint8_t*)field_dst[f] + (uint64_t)i * E;
      if (idx[i] < o->N) memcpy(d, o->col[f] + (uint64_t)idx[i] * E, E);
      else { memset(d, 0, E); o->status |= ORACLE_FLAG_BAD_INDEX; }
    }
  }
}

/* Priority retrieval (Section V-A). */
void oracle_get_priority(oracle_t* o, uint32_t n, const uint32_t* idx, float* out) {
  for (uint32_t i = 0; i < n; ++i) {
    if (idx[i] < o->N) out[i] = o->tree[o->P + idx[i]];
    else { out[i] = 0.0f; o->status |= ORACLE_FLAG_BAD_INDEX; }
  }
}

/* Number of real nodes of K-ary height h: n_0 = N, n_{h+1} = ceil(n_h / K). */
uint64_t oracle_level_count(const oracle_t* o, uint32_t height) {
  uint64_t n = o->N;
  for (uint32_t h = 0; h < height; ++h) n = (n + o->K - 1) / o->K;
  return n;
}

/* K-ary height h, position j  <->  tree[2^(HB - h*log2K) + j]. */
int oracle_read_level(const oracle_t* o, uint32_t height, float* out, uint64_t* count) {
  if (height > o->H) return -1;
  uint64_t n = oracle_level_count(o, height);
  uint64_t base = (uint64_t)1 << (o->HB - height * o->logK);
  if (out) memcpy(out, o->tree + base, n * sizeof(float));
  if (count) *count = n;
  return 0;
}

float    oracle_total(const oracle_t* o)        { return o->tree[1]; }
float    oracle_max_priority(const oracle_t* o) { return o->max_v; }
uint64_t oracle_size(const oracle_t* o)         { return o->size; }
uint64_t oracle_cursor(const oracle_t* o)       { return o->cursor; }
uint32_t oracle_height(const oracle_t* o)       { return o->H; }
uint32_t oracle_binary_height(const oracle_t* o){ return o->HB; }
uint32_t oracle_status(const oracle_t* o)       { return o->status; }
void     oracle_clear_status(oracle_t* o)       { o->status = 0; }

/* Raw binary-heap node, for tests that compare trees of different fanout at
 * shared binary depths. depth 0 = root. */
int oracle_read_binary_depth(const oracle_t* o, uint32_t depth, float* out, uint64_t count) {
  if (depth > o->HB) return -1;
  uint64_t base = (uint64_t)1 << depth;
  if (count > base) count = base;
  memcpy(out, o->tree + base, count * sizeof(float));
  return 0;
}
