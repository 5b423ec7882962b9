/*
 * CPU oracle for the sparse hot path of Distributed Equivalent Substitution (DES) training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP library is
 * checked against.  It shares no code with the HIP path and must never be called from it;
 * only tests, the smoke check and the CPU-baseline leg of the benchmark may use it.
 *
 * All floating-point accumulation is done in double from fp32 inputs.  Where a result is
 * stored in the table (weights, optimizer state) it is rounded to fp32 once.
 *
 * What each function follows in the paper (arXiv 1909.04823):
 *   table insert / find / update ....... Section 5, "Dynamic Hash Table" (lookup, insert of an
 *                                        initialized weight for a new feature ID, update)
 *   shard routing ...................... Section 5, "Large-scale Sparse Features" (i = f mod N)
 *                                        and Section 4.2 (any balanced partition of V)
 *   LR partial M1 ...................... Section 4.1, Eq. (lr_m1)
 *   FM partials M1, M2 and F ........... Section 4.2, Eq. (fm_m1m2), Eq. (des_fm2)
 *   per-field pooling .................. Section 4.3 (latent vectors aggregated by field)
 *   aggregation (+) .................... Section 3.2.1, Eq. (1); Algorithm 1
 *   DNN first layer partial M1 ......... Section 4.3, Eq. (dnn_bmm), Eq. (dnn_des)
 *   backward ........................... Section 3.2.2, "Back-propagation Phase": the gradient
 *                                        of the aggregate reaches every sub-operator unchanged
 *
 * Conventions the paper leaves open and this build fixes (the HIP library implements the same
 * text independently): the 64-bit mixer, the row initialiser, the row-assignment order (that of
 * a sequential insert loop), the merged-key order and the placement of eps in Adagrad.  These are "parity unpinned": nothing
 * in the paper can confirm them, the two implementations merely have to agree.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* The default build is single-threaded.  Compiled with -fopenmp (the all-cores leg of the benchmark's CPU
 * baseline) the loops marked below are split over threads: lookups over entries, the forward pass over samples,
 * merge + update over distinct rows.  Every iteration of those loops writes only its own outputs, so both
 * builds compute the same values in the same order per output. */
int oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

#define ORACLE_OK 0
#define ORACLE_ERR_INVALID_ARG 1
#define ORACLE_ERR_INVALID_KEY 2
#define ORACLE_ERR_FULL 3

#define ORACLE_EMPTY_KEY 0xFFFFFFFFFFFFFFFFull
#define ORACLE_MAX_DIM 4096    /* widest row the merge keeps a gradient for */

enum { SHARD_KEY_HASH = 0, SHARD_FIELD_MOD = 1 };
enum { OPT_NONE = 0, OPT_SGD = 1, OPT_ADAGRAD = 2, OPT_ADAM = 3, OPT_FTRL = 4 };

/* ------------------------------------------------------------------ conventions ---------- */

/* 64-bit finalizer of the SplitMix64 generator (Steele, Lea, Flood 2014). */
uint64_t oracle_mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* Which of the K logical shards owns an entry. */
int oracle_shard(uint64_t key, int32_t field, int K, int policy) {
  if (policy == SHARD_FIELD_MOD) return (int)(field % K);
  return (int)((uint32_t)(oracle_mix64(key) >> 32) % (uint32_t)K);
}

/* Initial value of column c (c < D: latent, c == D: LR weight) of a row inserted without
 * host values: uniform on [-sqrt(3) s, sqrt(3) s) (standard deviation s), a pure function of
 * (key, column, seed).  The 24-bit fraction and the subtraction are exact in fp32, so the
 * value is one correctly rounded fp32 product. */
float oracle_init_value(uint64_t key, int c, uint64_t seed, float init_scale) {
  uint64_t h = oracle_mix64(key ^ oracle_mix64(seed + (uint64_t)c));
  float u = (float)(h >> 40) * (1.0f / 16777216.0f);
  float width = (float)(2.0 * sqrt(3.0) * (double)init_scale);
  volatile float centred = u - 0.5f;
  return centred * width;
}

/* ------------------------------------------------------------------ table ---------------- */

typedef struct oracle_table {
  int D;
  int64_t capacity, n_rows;
  uint64_t seed;
  float init_scale;
  uint64_t *row_keys;           /* [capacity] row -> key                                   */
  float *emb, *w, *acc_emb, *acc_w;
  float *acc2_emb, *acc2_w;      /* second optimizer state (Adam v; FTRL z)                  */
  uint64_t *skeys;              /* keys in ascending order                                  */
  int32_t *srows;               /* row of skeys[i]                                          */
} oracle_table;

oracle_table *oracle_table_create(int D, int64_t capacity, uint64_t seed, float init_scale) {
  if (D <= 0 || D > ORACLE_MAX_DIM || capacity <= 0 || capacity > 2147483646ll) return NULL;
  oracle_table *t = (oracle_table *)calloc(1, sizeof(*t));
  if (!t) return NULL;
  t->D = D; t->capacity = capacity; t->seed = seed; t->init_scale = init_scale;
  t->row_keys = (uint64_t *)calloc((size_t)capacity, sizeof(uint64_t));
  t->emb = (float *)calloc((size_t)capacity * D, sizeof(float));
  t->w = (float *)calloc((size_t)capacity, sizeof(float));
  t->acc_emb = (float *)calloc((size_t)capacity * D, sizeof(float));
  t->acc_w = (float *)calloc((size_t)capacity, sizeof(float));
  t->acc2_emb = (float *)calloc((size_t)capacity * D, sizeof(float));
  t->acc2_w = (float *)calloc((size_t)capacity, sizeof(float));
  t->skeys = (uint64_t *)calloc((size_t)capacity, sizeof(uint64_t));
  t->srows = (int32_t *)calloc((size_t)capacity, sizeof(int32_t));
  if (!t->row_keys || !t->emb || !t->w || !t->acc_emb || !t->acc_w || !t->acc2_emb || !t->acc2_w || !t->skeys ||
      !t->srows) return NULL;
  return t;
}

void oracle_table_destroy(oracle_table *t) {
  if (!t) return;
  free(t->row_keys); free(t->emb); free(t->w); free(t->acc_emb); free(t->acc_w); free(t->acc2_emb); free(t->acc2_w);
  free(t->skeys); free(t->srows); free(t);
}

int64_t oracle_table_size(const oracle_table *t) { return t->n_rows; }
uint64_t *oracle_table_row_keys(oracle_table *t) { return t->row_keys; }
float *oracle_table_emb(oracle_table *t) { return t->emb; }
float *oracle_table_w(oracle_table *t) { return t->w; }
float *oracle_table_acc_emb(oracle_table *t) { return t->acc_emb; }
float *oracle_table_acc_w(oracle_table *t) { return t->acc_w; }
float *oracle_table_acc2_emb(oracle_table *t) { return t->acc2_emb; }
float *oracle_table_acc2_w(oracle_table *t) { return t->acc2_w; }

/* Row of a key, or -1: binary search in the ascending key list. */
static int32_t lookup(const oracle_table *t, uint64_t key) {
  int64_t lo = 0, hi = t->n_rows;
  while (lo < hi) {
    int64_t mid = lo + (hi - lo) / 2;
    if (t->skeys[mid] < key) lo = mid + 1; else hi = mid;
  }
  return (lo < t->n_rows && t->skeys[lo] == key) ? t->srows[lo] : -1;
}

typedef struct { uint64_t key; int64_t first; } newkey_t;

static int cmp_newkey(const void *a, const void *b) {
  const newkey_t *x = (const newkey_t *)a, *y = (const newkey_t *)b;
  if (x->key != y->key) return x->key < y->key ? -1 : 1;
  return x->first < y->first ? -1 : (x->first > y->first);
}

static int cmp_first(const void *a, const void *b) {
  const newkey_t *x = (const newkey_t *)a, *y = (const newkey_t *)b;
  return x->first < y->first ? -1 : (x->first > y->first);
}

/* Insert-if-absent, with the result of the plain sequential loop
 *     for i in 0..n-1: if keys[i] not in table: table[keys[i]] = n_rows++
 * i.e. the distinct keys of this call that the table does not hold yet receive the next
 * consecutive rows in the order of their first occurrence in the call.  Their weights are the
 * host values of that first occurrence, or the initialiser; optimizer state is zero.  Keys
 * already present are left untouched.  rows_out[i] = row of keys[i]. */
int oracle_table_insert(oracle_table *t, const uint64_t *keys, int64_t n, const float *values,
                        int32_t *rows_out) {
  if (!t || n < 0 || (n > 0 && !keys)) return ORACLE_ERR_INVALID_ARG;
  for (int64_t i = 0; i < n; ++i) if (keys[i] == ORACLE_EMPTY_KEY) return ORACLE_ERR_INVALID_KEY;
  newkey_t *cand = (newkey_t *)malloc(sizeof(newkey_t) * (size_t)(n > 0 ? n : 1));
  int64_t m = 0;
  for (int64_t i = 0; i < n; ++i)
    if (lookup(t, keys[i]) < 0) { cand[m].key = keys[i]; cand[m].first = i; ++m; }
  qsort(cand, (size_t)m, sizeof(newkey_t), cmp_newkey);
  int64_t u = 0;                                   /* distinct new keys, first occurrence kept */
  for (int64_t i = 0; i < m; ++i)
    if (i == 0 || cand[i].key != cand[i - 1].key) cand[u++] = cand[i];
  if (t->n_rows + u > t->capacity) { free(cand); return ORACLE_ERR_FULL; }
  qsort(cand, (size_t)u, sizeof(newkey_t), cmp_first);   /* row order = order of first occurrence */
  const int D = t->D;
  for (int64_t j = 0; j < u; ++j) {
    int64_t row = t->n_rows + j;
    uint64_t k = cand[j].key;
    t->row_keys[row] = k;
    for (int c = 0; c < D; ++c)
      t->emb[row * D + c] = values ? values[cand[j].first * (D + 1) + c]
                                   : oracle_init_value(k, c, t->seed, t->init_scale);
    t->w[row] = values ? values[cand[j].first * (D + 1) + D]
                       : oracle_init_value(k, D, t->seed, t->init_scale);
    for (int c = 0; c < D; ++c) t->acc_emb[row * D + c] = t->acc2_emb[row * D + c] = 0.0f;
    t->acc_w[row] = t->acc2_w[row] = 0.0f;
    cand[j].first = row;                           /* reuse the field: the key's row */
  }
  /* merge the new keys, ascending by key, into the ascending key list, back to front */
  qsort(cand, (size_t)u, sizeof(newkey_t), cmp_newkey);
  int64_t a = t->n_rows - 1, b = u - 1, o = t->n_rows + u - 1;
  while (b >= 0) {
    if (a >= 0 && t->skeys[a] > cand[b].key) { t->skeys[o] = t->skeys[a]; t->srows[o] = t->srows[a]; --a; }
    else { t->skeys[o] = cand[b].key; t->srows[o] = (int32_t)cand[b].first; --b; }
    --o;
  }
  t->n_rows += u;
  free(cand);
  if (rows_out) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < n; ++i) rows_out[i] = lookup(t, keys[i]);
  }
  return ORACLE_OK;
}

/* Lookup; with insert_missing the absent keys are inserted first (initialiser weights), so one
 * call both looks up and grows the table.  Absent keys otherwise map to -1. */
int oracle_table_find(oracle_table *t, const uint64_t *keys, int64_t n, int insert_missing,
                      int32_t *rows_out) {
  if (!t || n < 0 || (n > 0 && (!keys || !rows_out))) return ORACLE_ERR_INVALID_ARG;
  if (insert_missing) return oracle_table_insert(t, keys, n, NULL, rows_out);
  for (int64_t i = 0; i < n; ++i) if (keys[i] == ORACLE_EMPTY_KEY) return ORACLE_ERR_INVALID_KEY;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int64_t i = 0; i < n; ++i) rows_out[i] = lookup(t, keys[i]);
  return ORACLE_OK;
}

/* ------------------------------------------------------------------ forward -------------- */

/* Per-shard partial results of every sample.  Each CSR entry is one feature term, also when
 * a key repeats inside a sample.  Entries whose row is -1 contribute nothing.
 *   P_lr  [K,B]      sum of x*w over the shard's entries of the sample        (LR  M1)
 *   P_sum [K,B,D]    sum of x*v                                               (FM  M1)
 *   P_sq  [K,B]      sum of <x*v, x*v>                                        (FM  M2)
 *   P_pool[K,B,F,D]  sum of x*v over the shard's entries of bag (b,f)         (pooling)
 * Any output pointer may be NULL. */
void oracle_partial_forward(const oracle_table *t, int64_t B, int32_t F, const uint64_t *keys,
                            const int32_t *offsets, const float *vals, const int32_t *rows,
                            int K, int policy, double *P_lr, double *P_sum, double *P_sq,
                            double *P_pool) {
  const int D = t->D;
  if (P_lr) memset(P_lr, 0, sizeof(double) * (size_t)K * B);
  if (P_sum) memset(P_sum, 0, sizeof(double) * (size_t)K * B * D);
  if (P_sq) memset(P_sq, 0, sizeof(double) * (size_t)K * B);
  if (P_pool) memset(P_pool, 0, sizeof(double) * (size_t)K * B * F * D);
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int64_t b = 0; b < B; ++b)
    for (int32_t f = 0; f < F; ++f)
      for (int32_t e = offsets[b * F + f]; e < offsets[b * F + f + 1]; ++e) {
        int32_t r = rows[e];
        if (r < 0) continue;
        int s = oracle_shard(keys[e], f, K, policy);
        double x = vals ? (double)vals[e] : 1.0;
        if (P_lr) P_lr[(int64_t)s * B + b] += x * (double)t->w[r];
        for (int d = 0; d < D; ++d) {
          double xv = x * (double)t->emb[(int64_t)r * D + d];
          if (P_sum) P_sum[((int64_t)s * B + b) * D + d] += xv;
          if (P_sq) P_sq[(int64_t)s * B + b] += xv * xv;
          if (P_pool) P_pool[(((int64_t)s * B + b) * F + f) * D + d] += xv;
        }
      }
}

/* Aggregation over the K shards: out[i] = sum_s P[s][i]. */
void oracle_aggregate(const double *P, int K, int64_t n, double *out) {
  for (int64_t i = 0; i < n; ++i) {
    double a = 0.0;
    for (int s = 0; s < K; ++s) a += P[(int64_t)s * n + i];
    out[i] = a;
  }
}

/* Substitution operator of FM order 2: half of (<A_sum, A_sum> - A_sq) per sample. */
void oracle_fm_finalize(const double *A_sum, const double *A_sq, int64_t B, int D, double *fm2) {
  for (int64_t b = 0; b < B; ++b) {
    double q = 0.0;
    for (int d = 0; d < D; ++d) q += A_sum[b * D + d] * A_sum[b * D + d];
    fm2[b] = 0.5 * (q - A_sq[b]);
  }
}

/* ------------------------------------------------------------------ backward ------------- */

typedef struct { int32_t row; int32_t e; } rowent_t;

static int cmp_rowent(const void *a, const void *b) {
  const rowent_t *x = (const rowent_t *)a, *y = (const rowent_t *)b;
  if (x->row != y->row) return x->row < y->row ? -1 : 1;
  return x->e < y->e ? -1 : (x->e > y->e);
}

typedef struct {
  int32_t opt_emb, opt_w;          /* latent vectors: SGD, ADAGRAD, ADAM; LR weight: those or FTRL */
  float lr, eps;
  float beta1, beta2;              /* Adam */
  int64_t step;                    /* Adam: global step t >= 1 */
  float ftrl_alpha, ftrl_beta, ftrl_l1, ftrl_l2;
} oracle_optimizer;

/* One optimizer step on one coordinate with merged gradient G (double); state and weight are
 * stored in fp32.  SGD and Adagrad as in the comment of oracle_backward_update_opt; Adam and
 * FTRL-Proximal are the published algorithms:
 *   Adam (Kingma & Ba 2015, Algorithm 1), applied lazily to touched rows with the global step t:
 *     m = b1 m + (1-b1) G;  v = b2 v + (1-b2) G^2;  theta -= lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)
 *   FTRL-Proximal (McMahan et al. 2013, Algorithm 1), per coordinate with state (z, n):
 *     sigma = (sqrt(n+G^2) - sqrt(n))/alpha;  z += G - sigma w;  n += G^2;
 *     w = 0 if |z| <= l1 else -(z - sign(z) l1) / ((beta + sqrt(n))/alpha + l2)               */
static void optimizer_step(int opt, const oracle_optimizer *o, double G, float *theta, float *s1, float *s2) {
  if (opt == OPT_SGD) {
    *theta = (float)((double)*theta - (double)o->lr * G);
  } else if (opt == OPT_ADAGRAD) {
    double a = (double)*s1 + G * G;
    *theta = (float)((double)*theta - (double)o->lr * G / (sqrt(a) + (double)o->eps));
    *s1 = (float)a;
  } else if (opt == OPT_ADAM) {
    double b1 = (double)o->beta1, b2 = (double)o->beta2, t = (double)o->step;
    double m = b1 * (double)*s1 + (1.0 - b1) * G;
    double v = b2 * (double)*s2 + (1.0 - b2) * G * G;
    double mhat = m / (1.0 - pow(b1, t)), vhat = v / (1.0 - pow(b2, t));
    *theta = (float)((double)*theta - (double)o->lr * mhat / (sqrt(vhat) + (double)o->eps));
    *s1 = (float)m;
    *s2 = (float)v;
  } else if (opt == OPT_FTRL) {
    double n0 = (double)*s1, z0 = (double)*s2, alpha = (double)o->ftrl_alpha, l1 = (double)o->ftrl_l1;
    double n1 = n0 + G * G;
    double sigma = (sqrt(n1) - sqrt(n0)) / alpha;
    double z = z0 + G - sigma * (double)*theta;
    double w = fabs(z) <= l1 ? 0.0 : -(z - (z > 0 ? l1 : -l1)) / (((double)o->ftrl_beta + sqrt(n1)) / alpha + (double)o->ftrl_l2);
    *theta = (float)w;
    *s1 = (float)n1;
    *s2 = (float)z;
  }
}

/* Backward of the three sparse operators, duplicate-key merge and optimizer update.
 *
 * With upstream gradients g_lr[B] (of the aggregated LR sum), g_fm[B] (of the FM order-2
 * value), g_pool[B,F,D] (of the pooled embeddings) and the aggregated FM vector A_sum[B,D]
 * that the forward pass returned (fp32), entry e of bag (b,f) with value x and row r gets
 *     d/dw_r   : x * g_lr[b]
 *     d/dv_r,d : x * ( g_fm[b] * (A_sum[b,d] - x * v[r,d]) + g_pool[b,f,d] )
 * (the FM term is the derivative of Eq. (des_fm2)).  Gradients of entries that share a row
 * are summed; distinct rows are emitted in ascending row order.  The update then touches
 * exactly those rows, reading the pre-update weights:
 *     SGD      theta <- theta - lr*G
 *     Adagrad  a <- a + G^2 ;  theta <- theta - lr*G / (sqrt(a) + eps)   (a already updated)
 *     Adam, FTRL-Proximal: see optimizer_step
 * with one optimizer for the latent columns and one for the LR weight.  Any of g_lr, g_fm (with
 * A_sum), g_pool may be NULL (term absent).  OPT_NONE for both only merges.  Returns the number U of distinct rows; outputs (all nullable) hold U entries:
 * uniq_rows, uniq_keys, counts, merged[U, D+1] (D latent columns then the LR weight). */
int64_t oracle_backward_update_opt(oracle_table *t, int64_t B, int32_t F, const int32_t *offsets,
                                   const float *vals, const int32_t *rows, const float *g_lr,
                                   const float *g_fm, const float *A_sum, const float *g_pool,
                                   const oracle_optimizer *o, int32_t *uniq_rows,
                                   uint64_t *uniq_keys, int32_t *counts, double *merged) {
  const int D = t->D;
  const int64_t nnz = offsets[B * F];
  rowent_t *ent = (rowent_t *)malloc(sizeof(rowent_t) * (size_t)(nnz > 0 ? nnz : 1));
  int32_t *bag_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
  int64_t m = 0;
  for (int64_t bag = 0; bag < B * F; ++bag)
    for (int32_t e = offsets[bag]; e < offsets[bag + 1]; ++e) {
      bag_of[e] = (int32_t)bag;
      if (rows[e] >= 0) { ent[m].row = rows[e]; ent[m].e = e; ++m; }
    }
  qsort(ent, (size_t)m, sizeof(rowent_t), cmp_rowent);
  /* one segment of the sorted list per distinct row: seg[u] .. seg[u+1] */
  int64_t *seg = (int64_t *)malloc(sizeof(int64_t) * (size_t)(m + 1));
  int64_t U = 0;
  for (int64_t i = 0; i < m; ++i)
    if (i == 0 || ent[i].row != ent[i - 1].row) seg[U++] = i;
  seg[U] = m;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 256)
#endif
  for (int64_t u = 0; u < U; ++u) {
    double G[ORACLE_MAX_DIM + 1];
    const int64_t i = seg[u], j = seg[u + 1];
    const int32_t r = ent[i].row;
    for (int c = 0; c <= D; ++c) G[c] = 0.0;
    for (int64_t k = i; k < j; ++k) {
      const int32_t e = ent[k].e;
      const int64_t bag = bag_of[e], b = bag / F;
      const double x = vals ? (double)vals[e] : 1.0;
      if (g_lr) G[D] += x * (double)g_lr[b];
      for (int d = 0; d < D; ++d) {
        double g = 0.0;
        if (g_fm) g += (double)g_fm[b] * ((double)A_sum[b * D + d] - x * (double)t->emb[(int64_t)r * D + d]);
        if (g_pool) g += (double)g_pool[bag * D + d];
        G[d] += x * g;
      }
    }
    if (uniq_rows) uniq_rows[u] = r;
    if (uniq_keys) uniq_keys[u] = t->row_keys[r];
    if (counts) counts[u] = (int32_t)(j - i);
    if (merged) for (int c = 0; c <= D; ++c) merged[u * (D + 1) + c] = G[c];
    for (int c = 0; c <= D; ++c) {
      if (c < D)
        optimizer_step(o->opt_emb, o, G[c], &t->emb[(int64_t)r * D + c], &t->acc_emb[(int64_t)r * D + c],
                       &t->acc2_emb[(int64_t)r * D + c]);
      else
        optimizer_step(o->opt_w, o, G[c], &t->w[r], &t->acc_w[r], &t->acc2_w[r]);
    }
  }
  free(seg);
  free(bag_of); free(ent);
  return U;
}

/* Same optimizer (SGD, Adagrad or none) for latent vectors and LR weights. */
int64_t oracle_backward_update(oracle_table *t, int64_t B, int32_t F, const int32_t *offsets,
                               const float *vals, const int32_t *rows, const float *g_lr,
                               const float *g_fm, const float *A_sum, const float *g_pool,
                               int opt, float lr, float eps, int32_t *uniq_rows,
                               uint64_t *uniq_keys, int32_t *counts, double *merged) {
  oracle_optimizer o;
  memset(&o, 0, sizeof(o));
  o.opt_emb = o.opt_w = opt; o.lr = lr; o.eps = eps; o.step = 1;
  return oracle_backward_update_opt(t, B, F, offsets, vals, rows, g_lr, g_fm, A_sum, g_pool, &o, uniq_rows,
                                    uniq_keys, counts, merged);
}

/* ------------------------------------------------------------------ DNN first layer ------ */

/* Section 4.3, Eq. (dnn_bmm) / (dnn_des): V is the per-sample concatenation of the F pooled
 * field vectors, pool[B][F][D] (so V^T is [B, F*D]), and W is [F*D][H].  Both are cut along the
 * field dimension; the shard that holds field f (f mod K, the placement of Section 5) forms
 * M1(V_s, W_s) = V_s^T W_s:  Y_partial[s][b][h] = sum over its fields f and d of
 * pool[b][f][d] * W[f*D+d][h].  The aggregation sums the K partials. */
void oracle_dnn_partial_forward(const float *pool, const float *W, int64_t B, int32_t F, int D, int H, int K,
                                double *Y_partial) {
  memset(Y_partial, 0, sizeof(double) * (size_t)K * (size_t)B * (size_t)H);
  for (int64_t b = 0; b < B; ++b)
    for (int32_t f = 0; f < F; ++f) {
      const int s = f % K;
      for (int d = 0; d < D; ++d) {
        const double v = (double)pool[(b * F + f) * D + d];
        const float *wrow = W + ((int64_t)f * D + d) * H;
        for (int h = 0; h < H; ++h) Y_partial[((int64_t)s * B + b) * H + h] += v * (double)wrow[h];
      }
    }
}

/* Backward of the same layer (Section 3.2.2): the gradient dY[B][H] of the aggregate reaches every
 * shard unchanged; each shard differentiates its own product, so over all shards
 * g_pool[b][j] = sum_h dY[b][h] W[j][h]   and   dW[j][h] = sum_b pool[b][j] dY[b][h],  j = f*D+d. */
void oracle_dnn_backward(const float *pool, const float *W, const float *dY, int64_t B, int32_t F, int D, int H,
                         double *g_pool, double *dW) {
  const int64_t J = (int64_t)F * D;
  if (g_pool)
    for (int64_t b = 0; b < B; ++b)
      for (int64_t j = 0; j < J; ++j) {
        double a = 0.0;
        for (int h = 0; h < H; ++h) a += (double)dY[b * H + h] * (double)W[j * H + h];
        g_pool[b * J + j] = a;
      }
  if (dW)
    for (int64_t j = 0; j < J; ++j)
      for (int h = 0; h < H; ++h) {
        double a = 0.0;
        for (int64_t b = 0; b < B; ++b) a += (double)pool[b * J + j] * (double)dY[b * H + h];
        dW[j * H + h] = a;
      }
}

/* ------------------------------------------------------------------ DCN cross layer ------ */

/* Section 4, "DCN" paragraph (with the cross layer of the DCN paper it cites, its Section 2.2):
 *   x_{l+1} = x_0 (x_l^T w_l) + b_l + x_l,
 * all vectors of length d = F*D, x_0 the concatenated embedding output.  Under DES w_l is cut along d and
 * every process forms the dot product over its own part first, a scalar per sample; the aggregation sums
 * the scalars and the rest follows:  y = x_0 * (+)(x_local^T w_local) + b + x.
 * Columns are placed like the fields they belong to (f mod K, Section 5): column j = f*D + c goes with f.
 * P[s][b] = sum over the columns j of shard s of xl[b][j] * w[j]. */
void oracle_cross_partial(const float *xl, const float *w, int64_t B, int32_t F, int D, int K, double *P) {
  memset(P, 0, sizeof(double) * (size_t)K * (size_t)B);
  for (int64_t b = 0; b < B; ++b)
    for (int32_t f = 0; f < F; ++f)
      for (int c = 0; c < D; ++c) {
        const int64_t j = (int64_t)f * D + c;
        P[(int64_t)(f % K) * B + b] += (double)xl[b * (int64_t)F * D + j] * (double)w[j];
      }
}

/* Backward of that sub-operator for a gradient g_s[b] of its aggregated scalar (Section 3.2.2: every shard
 * receives it unchanged, so over all shards): g_xl[b][j] = g_s[b] w[j], dw[j] = sum_b g_s[b] xl[b][j]. */
void oracle_cross_partial_backward(const float *xl, const float *w, const float *g_s, int64_t B, int64_t d,
                                   double *g_xl, double *dw) {
  for (int64_t j = 0; j < d; ++j) dw[j] = 0.0;
  for (int64_t b = 0; b < B; ++b)
    for (int64_t j = 0; j < d; ++j) {
      g_xl[b * d + j] = (double)g_s[b] * (double)w[j];
      dw[j] += (double)g_s[b] * (double)xl[b * d + j];
    }
}

/* y[b][j] = x0[b][j] * s[b] + bias[j] + xl[b][j], s the aggregated scalar. */
void oracle_cross_apply(const float *x0, const float *xl, const float *s, const float *bias, int64_t B, int64_t d,
                        double *y) {
  for (int64_t b = 0; b < B; ++b)
    for (int64_t j = 0; j < d; ++j)
      y[b * d + j] = (double)x0[b * d + j] * (double)s[b] + (double)bias[j] + (double)xl[b * d + j];
}

/* Backward of one cross layer for the upstream gradient g_y[B][d] (Section 3.2.2: the gradient of the
 * aggregate reaches every sub-operator unchanged).  With s[b] = xl[b]^T w:
 *   g_s[b]     = sum_j g_y[b][j] x0[b][j]            (gradient of the aggregated scalar)
 *   g_xl[b][j] = g_y[b][j] + g_s[b] w[j]             (identity path + the sub-operators)
 *   g_x0[b][j] = g_y[b][j] s[b]                      (this layer's share; x_0 feeds every layer)
 *   dw[j] = sum_b g_s[b] xl[b][j],   db[j] = sum_b g_y[b][j]. */
void oracle_cross_backward(const float *x0, const float *xl, const float *w, const float *s, const float *g_y,
                           int64_t B, int64_t d, double *g_s, double *g_xl, double *g_x0, double *dw, double *db) {
  for (int64_t j = 0; j < d; ++j) { dw[j] = 0.0; db[j] = 0.0; }
  for (int64_t b = 0; b < B; ++b) {
    double gs = 0.0;
    for (int64_t j = 0; j < d; ++j) gs += (double)g_y[b * d + j] * (double)x0[b * d + j];
    g_s[b] = gs;
    for (int64_t j = 0; j < d; ++j) {
      const double g = (double)g_y[b * d + j];
      g_xl[b * d + j] = g + gs * (double)w[j];
      g_x0[b * d + j] = g * (double)s[b];
      dw[j] += gs * (double)xl[b * d + j];
      db[j] += g;
    }
  }
}

/* ------------------------------------------------------------------ dense tower and output unit ----
 * What follows the aggregated weights-rich operators (Section 3.2.1: the layers after them see the
 * same aggregated result on every process; Section 4, Table "common components": LR = first order,
 * FM = first + second order, W&D = first + high order, DeepFM = all three; Section 4.1 for the
 * sigmoid output).  The paper names these parts without formulas; they are the textbook ones:
 *   hidden layer     A = relu(Z + bias)           Z = aggregated product of the layer
 *   output unit      logit = b0 + A_lr + fm2 + <a, w_out>,  p = sigmoid(logit)
 *   loss             mean over the batch of  -y log p - (1-y) log(1-p)
 * "parity unpinned" for the choice of ReLU and of the mean log-loss: the paper reports log loss and
 * AUC (Section 6) but prints neither the activation nor the reduction. */

/* A[b,h] = Z[b,h] + bias[h], clamped at zero from below when relu != 0.  bias may be NULL. */
void oracle_bias_act(const double *Z, const float *bias, int64_t B, int H, int relu, double *A) {
  for (int64_t b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      double z = Z[b * H + h] + (bias ? (double)bias[h] : 0.0);
      A[b * H + h] = (relu && z < 0.0) ? 0.0 : z;
    }
}

/* Backward of the same: dZ[b,h] = dA[b,h] where the unit was active (A > 0; everywhere without
 * relu), else 0;  dbias[h] = sum_b dZ[b,h].  A is the forward output. */
void oracle_bias_act_backward(const float *A, const float *dA, int64_t B, int H, int relu, double *dZ,
                              double *dbias) {
  for (int h = 0; h < H; ++h) dbias[h] = 0.0;
  for (int64_t b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      double g = (!relu || A[b * H + h] > 0.0f) ? (double)dA[b * H + h] : 0.0;
      dZ[b * H + h] = g;
      dbias[h] += g;
    }
}

/* Output unit, loss and their gradients.  Any of A_lr, fm2, a (with w_out) may be NULL: the model
 * then has no such component.  Outputs (all but g_logit nullable):
 *   logit[B], p[B], *loss (mean log-loss), g_logit[b] = (p - y)/B = d loss / d logit[b] (which is
 *   also the upstream gradient of A_lr[b] and of fm2[b]),  da[b,h] = g_logit[b] w_out[h],
 *   dw_out[h] = sum_b g_logit[b] a[b,h],  *db0 = sum_b g_logit[b]. */
void oracle_head(const float *A_lr, const float *fm2, const float *a, const float *w_out, float b0,
                 const float *labels, int64_t B, int H, double *logit, double *p, double *loss,
                 double *g_logit, double *da, double *dw_out, double *db0) {
  double total = 0.0, gsum = 0.0;
  if (dw_out) for (int h = 0; h < H; ++h) dw_out[h] = 0.0;
  for (int64_t b = 0; b < B; ++b) {
    double z = (double)b0;
    if (A_lr) z += (double)A_lr[b];
    if (fm2) z += (double)fm2[b];
    if (a) for (int h = 0; h < H; ++h) z += (double)a[b * H + h] * (double)w_out[h];
    const double y = (double)labels[b];
    const double pb = 1.0 / (1.0 + exp(-z));
    /* -y log p - (1-y) log(1-p) = log(1 + e^z) - y z, written so that neither e^z nor the log overflows */
    total += (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z))) - y * z;
    const double g = (pb - y) / (double)B;
    if (logit) logit[b] = z;
    if (p) p[b] = pb;
    g_logit[b] = g;
    gsum += g;
    if (a && da) for (int h = 0; h < H; ++h) da[b * H + h] = g * (double)w_out[h];
    if (a && dw_out) for (int h = 0; h < H; ++h) dw_out[h] += g * (double)a[b * H + h];
  }
  if (loss) *loss = B > 0 ? total / (double)B : 0.0;
  if (db0) *db0 = gsum;
}

/* One optimizer step over a dense parameter array (every coordinate is touched every step):
 * optimizer o->opt_emb with the arithmetic of optimizer_step. */
void oracle_dense_update(float *theta, const float *grad, float *s1, float *s2, int64_t n,
                         const oracle_optimizer *o) {
  for (int64_t i = 0; i < n; ++i)
    optimizer_step(o->opt_emb, o, (double)grad[i], theta + i, s1 ? s1 + i : NULL, s2 ? s2 + i : NULL);
}

/* ------------------------------------------------------------------ growth and eviction ---
 * Section 1 ("Dynamic Features": the parameter set of a streaming recommender changes over time and
 * keeps growing) and Section 5 (dynamic hash table).  The paper states the requirement, not a
 * mechanism; this build's mechanism is a migration: the rows to keep move, in ascending row order,
 * into a new table of any capacity that holds them.  Row i of the result is the i-th kept row of the
 * source with its key, weights and optimizer state unchanged; keys of dropped rows are absent
 * afterwards (looking one up with insertion creates a fresh row with initialiser weights).
 * keep == NULL keeps every row (pure growth).  "parity unpinned" for the row order of the result
 * (stable), which nothing in the paper fixes.  Returns NULL if the kept rows exceed new_capacity. */
oracle_table *oracle_table_migrate(const oracle_table *src, const uint8_t *keep, int64_t new_capacity) {
  if (!src) return NULL;
  int64_t kept = 0;
  for (int64_t r = 0; r < src->n_rows; ++r) kept += (!keep || keep[r]) ? 1 : 0;
  if (kept > new_capacity) return NULL;
  oracle_table *dst = oracle_table_create(src->D, new_capacity, src->seed, src->init_scale);
  if (!dst) return NULL;
  const int D = src->D;
  int64_t n = 0;
  for (int64_t r = 0; r < src->n_rows; ++r) {
    if (keep && !keep[r]) continue;
    dst->row_keys[n] = src->row_keys[r];
    memcpy(dst->emb + n * D, src->emb + r * D, sizeof(float) * (size_t)D);
    memcpy(dst->acc_emb + n * D, src->acc_emb + r * D, sizeof(float) * (size_t)D);
    memcpy(dst->acc2_emb + n * D, src->acc2_emb + r * D, sizeof(float) * (size_t)D);
    dst->w[n] = src->w[r]; dst->acc_w[n] = src->acc_w[r]; dst->acc2_w[n] = src->acc2_w[r];
    ++n;
  }
  dst->n_rows = n;
  /* key -> row map of the result: (key, row) pairs in ascending key order (insertion sort by
   * repeated binary search would be quadratic; sort pairs instead) */
  newkey_t *pairs = (newkey_t *)malloc(sizeof(newkey_t) * (size_t)(n > 0 ? n : 1));
  for (int64_t i = 0; i < n; ++i) { pairs[i].key = dst->row_keys[i]; pairs[i].first = i; }
  qsort(pairs, (size_t)n, sizeof(newkey_t), cmp_newkey);
  for (int64_t i = 0; i < n; ++i) { dst->skeys[i] = pairs[i].key; dst->srows[i] = (int32_t)pairs[i].first; }
  free(pairs);
  return dst;
}
