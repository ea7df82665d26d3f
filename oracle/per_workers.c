/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * A second CPU baseline beside the plain oracle: the same arithmetic on W worker threads,
 * in the spirit of the paper's CPU kernel for the replay operations (Section V-A: the batch
 * of requests is split over workers, each handling its share).  It works on the oracle's own
 * state (the heap array of per_oracle.c, whose definitions this file includes), must leave
 * that state and every output bit-identical to what the sequential oracle produces, and is
 * checked against it in the CPU tests.  Only tests and the bench's CPU leg may load it.
 *
 *   sampling   every sample's root-to-leaf walk is independent: workers take slices of the batch.
 *   gather     row copies are independent: workers take slices of the batch.
 *   update     a sequential pass fixes validity, the running maximum and the last writer of
 *              every index (batch order); the winners' leaves are written in parallel; then the
 *              touched nodes are re-summed one binary level at a time, bottom-up, the distinct
 *              parents of a level shared among the workers.  Every node ends up as the fp32 sum
 *              of its two children, which is what the sequential set-and-re-sum leaves behind.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC.
 */
#include "per_oracle.c"

#include <omp.h>

int workers_max_threads(void) { return omp_get_max_threads(); }

int workers_sample(oracle_t* o, uint32_t B, float beta, const float* u, uint32_t* out_idx,
                   float* out_weight_or_null, float* out_prio_or_null, int nthreads) {
  const float* t = o->tree;
  const float total = t[1];
  if (!(total > 0.0f)) return oracle_sample(o, B, beta, u, out_idx, out_weight_or_null, out_prio_or_null);
  const float seg = total / (float)B;
  double* wt = out_weight_or_null ? (double*)malloc(sizeof(double) * B) : NULL;
  double wmax = 0.0;
#pragma omp parallel num_threads(nthreads)
  {
    double local_max = 0.0;
#pragma omp for schedule(static)
    for (int64_t i = 0; i < (int64_t)B; ++i) {
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
        if (wt[i] > local_max) local_max = wt[i];
      }
    }
#pragma omp critical
    if (local_max > wmax) wmax = local_max;
  }
  if (wt) {
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t i = 0; i < (int64_t)B; ++i) out_weight_or_null[i] = (float)(wt[i] / wmax);
    free(wt);
  }
  return 0;
}

void workers_gather(oracle_t* o, uint32_t B, const uint32_t* idx, void* const* field_dst, int nthreads) {
  for (uint32_t f = 0; f < o->n_fields; ++f) {
    if (!o->col[f] || !field_dst[f]) continue;
    const uint32_t E = o->field_bytes[f];
    int bad = 0;
#pragma omp parallel for schedule(static) num_threads(nthreads) reduction(| : bad)
    for (int64_t i = 0; i < (int64_t)B; ++i) {
      uint8_t* d = (uint8_t*)field_dst[f] + (uint64_t)i * E;
      if (idx[i] < o->N) memcpy(d, o->col[f] + (uint64_t)idx[i] * E, E);
      else { memset(d, 0, E); bad |= 1; }
    }
    if (bad) o->status |= ORACLE_FLAG_BAD_INDEX;
  }
}

static int cmp_u64(const void* a, const void* b) {
  const uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
  return x < y ? -1 : x > y ? 1 : 0;
}

/* Per-tree work array kept between calls: last[leaf] = (call << 32) | (1 + position of the latest valid
 * element of that call that names the leaf), so it never needs clearing. */
#define WORKERS_MAX_TREES 256
static struct { const oracle_t* o; uint64_t* last; uint64_t calls, n; } g_side[WORKERS_MAX_TREES];

static int side_slot(const oracle_t* o) {
  int free_slot = -1;
  for (int k = 0; k < WORKERS_MAX_TREES; ++k) {
    if (g_side[k].o == o && g_side[k].n == o->N) return k;
    if (g_side[k].o == o) {   /* an earlier tree at this address that was never released */
      free(g_side[k].last);
      g_side[k].o = NULL;
      g_side[k].last = NULL;
    }
    if (!g_side[k].o && free_slot < 0) free_slot = k;
  }
  if (free_slot < 0) return -1;
  g_side[free_slot].last = (uint64_t*)calloc(o->N, sizeof(uint64_t));
  if (!g_side[free_slot].last) return -1;
  g_side[free_slot].o = o;
  g_side[free_slot].n = o->N;
  g_side[free_slot].calls = 0;
  return free_slot;
}

/* Forget the work array of a tree (call before destroying the oracle it belongs to). */
void workers_release(const oracle_t* o) {
  for (int k = 0; k < WORKERS_MAX_TREES; ++k)
    if (g_side[k].o == o) { free(g_side[k].last); g_side[k].o = NULL; g_side[k].last = NULL; }
}

/* Returns 0, or -1 when the work arrays cannot be allocated (nothing is changed then). */
int workers_update(oracle_t* o, uint32_t B, const uint32_t* idx, const float* prio, int nthreads) {
  if (B == 0) return 0;
  const int slot = side_slot(o);
  uint64_t* cur = (uint64_t*)malloc(sizeof(uint64_t) * B);    /* touched nodes of the current level */
  uint64_t* nxt = (uint64_t*)malloc(sizeof(uint64_t) * B);
  if (slot < 0 || !cur || !nxt) { free(cur); free(nxt); return -1; }
  uint64_t* last = g_side[slot].last;
  const uint64_t call = ++g_side[slot].calls << 32;
  for (uint32_t j = 0; j < B; ++j) {   /* sequential: validity, running maximum, last writer in batch order */
    if (!(idx[j] < o->size)) { o->status |= ORACLE_FLAG_BAD_INDEX; continue; }
    if (!valid_priority(prio[j])) { o->status |= ORACLE_FLAG_BAD_PRIORITY; continue; }
    last[idx[j]] = call | (j + 1);
    if (prio[j] > o->max_v) o->max_v = prio[j];
  }
  uint64_t n = 0;
  for (uint32_t j = 0; j < B; ++j)
    if (idx[j] < o->size && last[idx[j]] == (call | (j + 1))) cur[n++] = o->P + idx[j];
  float* t = o->tree;
#pragma omp parallel for schedule(static) num_threads(nthreads)
  for (int64_t k = 0; k < (int64_t)n; ++k) {
    const uint32_t leaf = (uint32_t)(cur[k] - o->P);
    t[cur[k]] = prio[(uint32_t)last[leaf] - 1];
  }
  /* winners were collected in batch order; in index order equal parents are neighbours on every level */
  int sorted = 1;
  for (uint64_t k = 1; k < n && sorted; ++k) sorted = cur[k - 1] <= cur[k];
  if (!sorted) qsort(cur, n, sizeof(uint64_t), cmp_u64);
  while (n > 0 && cur[0] > 1) {   /* all touched nodes sit on one level; level of the root: done */
    uint64_t m = 0;
    for (uint64_t k = 0; k < n; ++k) {
      const uint64_t p = cur[k] >> 1;
      if (m == 0 || nxt[m - 1] != p) nxt[m++] = p;
    }
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t k = 0; k < (int64_t)m; ++k) t[nxt[k]] = t[2 * nxt[k]] + t[2 * nxt[k] + 1];
    uint64_t* sw = cur; cur = nxt; nxt = sw;
    n = m;
  }
  free(cur); free(nxt);
  return 0;
}
