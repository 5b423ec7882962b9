/*
 * One DES step driven from plain C: no Python, no PyTorch in the process.  Every buffer comes from hipMalloc
 * and is filled with hipMemcpy; the library is entered through include/des.h only:
 *   des_table_create -> des_table_insert -> des_table_find (inserting the unseen IDs)
 *   -> des_partial_forward -> des_aggregate_partials x3 -> des_fm_finalize
 *   -> des_backward_update_adagrad -> des_table_export_keys / des_table_size / des_table_status
 * and the results are compared with the CPU oracle (linked in from oracle/des_oracle.c: this program is test
 * infrastructure) to the library's bound: integers equal, |gpu - ref| <= max(1e-5 |ref|, 1e-6).
 * Prints one line per check, "des_host_step: PASS" at the end, and exits 0; any failure exits 1.
 *
 * Built by __graft_entry__.build() with the host C compiler (C11), linked against libdes.so and the HIP runtime.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "des.h"

/* the oracle's C interface (oracle/des_oracle.c) */
typedef struct oracle_table oracle_table;
oracle_table *oracle_table_create(int D, int64_t capacity, uint64_t seed, float init_scale);
void oracle_table_destroy(oracle_table *t);
int64_t oracle_table_size(const oracle_table *t);
uint64_t *oracle_table_row_keys(oracle_table *t);
float *oracle_table_emb(oracle_table *t);
float *oracle_table_w(oracle_table *t);
float *oracle_table_acc_emb(oracle_table *t);
float *oracle_table_acc_w(oracle_table *t);
int oracle_table_insert(oracle_table *t, const uint64_t *keys, int64_t n, const float *values, int32_t *rows_out);
int oracle_table_find(oracle_table *t, const uint64_t *keys, int64_t n, int insert_missing, int32_t *rows_out);
void oracle_partial_forward(const oracle_table *t, int64_t B, int32_t F, const uint64_t *keys, const int32_t *offsets,
                            const float *vals, const int32_t *rows, int K, int policy, double *P_lr, double *P_sum,
                            double *P_sq, double *P_pool);
void oracle_aggregate(const double *P, int K, int64_t n, double *out);
void oracle_fm_finalize(const double *A_sum, const double *A_sq, int64_t B, int D, double *fm2);
int64_t oracle_backward_update(oracle_table *t, int64_t B, int32_t F, const int32_t *offsets, const float *vals,
                               const int32_t *rows, const float *g_lr, const float *g_fm, const float *A_sum,
                               const float *g_pool, int opt, float lr, float eps, int32_t *uniq_rows,
                               uint64_t *uniq_keys, int32_t *counts, double *merged);

static int failures = 0;

#define HIP_OK(call)                                                                              \
  do {                                                                                            \
    hipError_t e_ = (call);                                                                       \
    if (e_ != hipSuccess) {                                                                       \
      fprintf(stderr, "des_host_step: %s failed: %s\n", #call, hipGetErrorString(e_));            \
      exit(1);                                                                                    \
    }                                                                                             \
  } while (0)
#define DES_OK_(call)                                                                             \
  do {                                                                                            \
    des_status_t s_ = (call);                                                                     \
    if (s_ != DES_OK) {                                                                           \
      fprintf(stderr, "des_host_step: %s returned %s\n", #call, des_status_string(s_));           \
      exit(1);                                                                                    \
    }                                                                                             \
  } while (0)

/* the program's own input generator: a 64-bit linear congruential step with an output xor-shift */
static uint64_t rng_state = 0x1909048231ull;
static uint64_t next_u64(void) {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  uint64_t x = rng_state;
  x ^= x >> 33;
  return x;
}
static double next_unit(void) { return (double)(next_u64() >> 11) / 9007199254740992.0; }
static float next_normalish(void) { /* sum of four uniforms, centred: inputs only need a spread of signs and sizes */
  return (float)((next_unit() + next_unit() + next_unit() + next_unit() - 2.0) * 1.7);
}

static void *dmalloc(size_t bytes) {
  void *p = NULL;
  HIP_OK(hipMalloc(&p, bytes ? bytes : 16));
  return p;
}
static void *to_device(const void *host, size_t bytes) {
  void *p = dmalloc(bytes);
  if (bytes) HIP_OK(hipMemcpy(p, host, bytes, hipMemcpyHostToDevice));
  return p;
}
static void *to_host(const void *dev, size_t bytes) {
  void *p = malloc(bytes ? bytes : 16);
  if (bytes) HIP_OK(hipMemcpy(p, dev, bytes, hipMemcpyDeviceToHost));
  return p;
}

static void check_close(const char *what, const float *gpu, const double *ref, size_t n) {
  size_t bad = 0, worst = 0;
  double worst_excess = 0.0;
  for (size_t i = 0; i < n; ++i) {
    const double err = fabs((double)gpu[i] - ref[i]);
    const double tol = fmax(1e-5 * fabs(ref[i]), 1e-6);
    if (!(err <= tol)) {
      ++bad;
      if (err - tol > worst_excess) { worst_excess = err - tol; worst = i; }
    }
  }
  if (bad) {
    printf("FAIL %s: %zu of %zu outside the bound; worst at %zu: gpu=%.9g ref=%.9g\n", what, bad, n, worst,
           (double)gpu[worst], ref[worst]);
    ++failures;
  } else {
    printf("ok   %s (%zu values)\n", what, n);
  }
}
static void check_close_f(const char *what, const float *gpu, const float *ref, size_t n) {
  double *r = (double *)malloc(sizeof(double) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) r[i] = (double)ref[i];
  check_close(what, gpu, r, n);
  free(r);
}
static void check_equal_bytes(const char *what, const void *gpu, const void *ref, size_t bytes) {
  if (memcmp(gpu, ref, bytes) != 0) {
    printf("FAIL %s: integer outputs differ\n", what);
    ++failures;
  } else {
    printf("ok   %s (%zu bytes equal)\n", what, bytes);
  }
}

int main(void) {
  enum { B = 300, F = 7, D = 16, K = 5, VOCAB = 4000, PRE = 2500, CAP = 6000 };
  const float lr = 0.05f, eps = 1e-8f, init_scale = 0.01f;
  const uint64_t seed = 77;
  int ndev = 0;
  HIP_OK(hipGetDeviceCount(&ndev));
  if (ndev < 1) { fprintf(stderr, "des_host_step: no GPU\n"); return 1; }
  HIP_OK(hipSetDevice(0));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  /* ---- inputs: a vocabulary of distinct odd IDs, ragged bags (0..6 entries) with a skewed popularity ---- */
  uint64_t *vocab = (uint64_t *)malloc(sizeof(uint64_t) * VOCAB);
  for (int i = 0; i < VOCAB; ++i) vocab[i] = ((uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull) | 1ull;   /* odd multiplier: distinct */
  int32_t *offsets = (int32_t *)malloc(sizeof(int32_t) * (B * F + 1));
  offsets[0] = 0;
  for (int i = 0; i < B * F; ++i) offsets[i + 1] = offsets[i] + (int32_t)(next_u64() % 7);
  const int64_t nnz = offsets[B * F];
  uint64_t *keys = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)nnz);
  for (int64_t e = 0; e < nnz; ++e) {
    const double u = next_unit();
    keys[e] = vocab[(int)(u * u * u * VOCAB)];          /* cube of a uniform: a few IDs occur hundreds of times */
  }
  float *values = (float *)malloc(sizeof(float) * PRE * (D + 1));
  for (int i = 0; i < PRE * (D + 1); ++i) values[i] = 0.05f * next_normalish();
  float *g_lr = (float *)malloc(sizeof(float) * B), *g_fm = (float *)malloc(sizeof(float) * B);
  float *g_pool = (float *)malloc(sizeof(float) * B * F * D);
  for (int i = 0; i < B; ++i) { g_lr[i] = next_normalish() / B; g_fm[i] = next_normalish() / B; }
  for (int i = 0; i < B * F * D; ++i) g_pool[i] = next_normalish() / B;

  /* ---- the oracle's step ---- */
  oracle_table *ot = oracle_table_create(D, CAP, seed, init_scale);
  int32_t *o_rows0 = (int32_t *)malloc(sizeof(int32_t) * PRE), *o_rows = (int32_t *)malloc(sizeof(int32_t) * (size_t)nnz);
  if (oracle_table_insert(ot, vocab, PRE, values, o_rows0) != 0 || oracle_table_find(ot, keys, nnz, 1, o_rows) != 0) {
    fprintf(stderr, "des_host_step: oracle refused the inputs\n");
    return 1;
  }
  const int64_t n_rows = oracle_table_size(ot);
  double *oP_lr = (double *)malloc(sizeof(double) * K * B), *oP_sum = (double *)malloc(sizeof(double) * K * B * D);
  double *oP_sq = (double *)malloc(sizeof(double) * K * B), *o_pool = (double *)malloc(sizeof(double) * B * F * D);
  oracle_partial_forward(ot, B, F, keys, offsets, NULL, o_rows, K, 0, oP_lr, oP_sum, oP_sq, NULL);
  oracle_partial_forward(ot, B, F, keys, offsets, NULL, o_rows, 1, 0, NULL, NULL, NULL, o_pool);
  double *oA_lr = (double *)malloc(sizeof(double) * B), *oA_sum = (double *)malloc(sizeof(double) * B * D);
  double *oA_sq = (double *)malloc(sizeof(double) * B), *o_fm2 = (double *)malloc(sizeof(double) * B);
  oracle_aggregate(oP_lr, K, B, oA_lr);
  oracle_aggregate(oP_sum, K, (int64_t)B * D, oA_sum);
  oracle_aggregate(oP_sq, K, B, oA_sq);
  oracle_fm_finalize(oA_sum, oA_sq, B, D, o_fm2);
  float *A_sum_in = (float *)malloc(sizeof(float) * B * D);      /* both sides take the oracle's rounded aggregate */
  for (int i = 0; i < B * D; ++i) A_sum_in[i] = (float)oA_sum[i];
  int32_t *o_uniq = (int32_t *)malloc(sizeof(int32_t) * (size_t)nnz), *o_counts = (int32_t *)malloc(sizeof(int32_t) * (size_t)nnz);
  uint64_t *o_ukeys = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)nnz);
  double *o_merged = (double *)malloc(sizeof(double) * (size_t)nnz * (D + 1));
  const int64_t U = oracle_backward_update(ot, B, F, offsets, NULL, o_rows, g_lr, g_fm, A_sum_in, g_pool, 2 /* Adagrad */,
                                           lr, eps, o_uniq, o_ukeys, o_counts, o_merged);

  /* ---- the library's step, hipMalloc'd memory only ---- */
  des_table_config_t cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.dim = D; cfg.capacity_rows = CAP; cfg.num_shards = K; cfg.shard_policy = DES_SHARD_KEY_HASH; cfg.opt = DES_OPT_ADAGRAD;
  cfg.init_seed = seed; cfg.init_scale = init_scale;
  const int64_t max_n = nnz > PRE ? nnz : PRE;
  DES_OK_(des_table_query_bytes(&cfg, max_n, &cfg.slots_bytes, &cfg.workspace_bytes));
  cfg.emb = (float *)dmalloc(sizeof(float) * CAP * D);
  cfg.w = (float *)dmalloc(sizeof(float) * CAP);
  cfg.acc_emb = (float *)dmalloc(sizeof(float) * CAP * D);
  cfg.acc_w = (float *)dmalloc(sizeof(float) * CAP);
  cfg.row_keys = (uint64_t *)dmalloc(sizeof(uint64_t) * CAP);
  cfg.slots = dmalloc(cfg.slots_bytes);
  cfg.workspace = dmalloc(cfg.workspace_bytes);
  des_table_t *t = NULL;
  DES_OK_(des_table_create(&cfg, &t));

  uint64_t *d_vocab = (uint64_t *)to_device(vocab, sizeof(uint64_t) * PRE);
  float *d_values = (float *)to_device(values, sizeof(float) * PRE * (D + 1));
  int32_t *d_rows0 = (int32_t *)dmalloc(sizeof(int32_t) * PRE);
  DES_OK_(des_table_insert(t, d_vocab, PRE, d_values, d_rows0, stream));

  des_batch_t batch;
  batch.B = B; batch.F = F; batch.nnz = nnz;
  batch.keys = (const uint64_t *)to_device(keys, sizeof(uint64_t) * (size_t)nnz);
  batch.offsets = (const int32_t *)to_device(offsets, sizeof(int32_t) * (B * F + 1));
  batch.vals = NULL;
  int32_t *d_rows = (int32_t *)dmalloc(sizeof(int32_t) * (size_t)nnz);
  DES_OK_(des_table_find(t, batch.keys, nnz, DES_MISS_INSERT, d_rows, stream));

  float *d_P_lr = (float *)dmalloc(sizeof(float) * K * B), *d_P_sum = (float *)dmalloc(sizeof(float) * K * B * D);
  float *d_P_sq = (float *)dmalloc(sizeof(float) * K * B), *d_pool = (float *)dmalloc(sizeof(float) * B * F * D);
  DES_OK_(des_partial_forward(t, &batch, d_rows, d_P_lr, d_P_sum, d_P_sq, d_pool, stream));
  float *d_A_lr = (float *)dmalloc(sizeof(float) * B), *d_A_sum = (float *)dmalloc(sizeof(float) * B * D);
  float *d_A_sq = (float *)dmalloc(sizeof(float) * B), *d_fm2 = (float *)dmalloc(sizeof(float) * B);
  DES_OK_(des_aggregate_partials(d_P_lr, K, B, d_A_lr, stream));
  DES_OK_(des_aggregate_partials(d_P_sum, K, (int64_t)B * D, d_A_sum, stream));
  DES_OK_(des_aggregate_partials(d_P_sq, K, B, d_A_sq, stream));
  DES_OK_(des_fm_finalize(d_A_sum, d_A_sq, B, D, d_fm2, stream));

  des_backward_io_t io;
  memset(&io, 0, sizeof(io));
  io.g_lr = (const float *)to_device(g_lr, sizeof(float) * B);
  io.g_fm = (const float *)to_device(g_fm, sizeof(float) * B);
  io.A_sum = (const float *)to_device(A_sum_in, sizeof(float) * B * D);
  io.g_pool = (const float *)to_device(g_pool, sizeof(float) * B * F * D);
  io.uniq_rows_out = (int32_t *)dmalloc(sizeof(int32_t) * (size_t)nnz);
  io.uniq_keys_out = (uint64_t *)dmalloc(sizeof(uint64_t) * (size_t)nnz);
  io.counts_out = (int32_t *)dmalloc(sizeof(int32_t) * (size_t)nnz);
  io.merged_out = (float *)dmalloc(sizeof(float) * (size_t)nnz * (D + 1));
  io.n_uniq_out = (int64_t *)dmalloc(sizeof(int64_t));
  DES_OK_(des_backward_update_adagrad(t, &batch, d_rows, &io, lr, eps, stream));
  uint64_t *d_keys_out = (uint64_t *)dmalloc(sizeof(uint64_t) * CAP);
  DES_OK_(des_table_export_keys(t, d_keys_out, CAP, stream));
  HIP_OK(hipStreamSynchronize(stream));

  /* ---- compare ---- */
  int64_t g_n_rows = -1, g_U = -1;
  DES_OK_(des_table_size(t, &g_n_rows));
  DES_OK_(des_table_status(t));
  HIP_OK(hipMemcpy(&g_U, io.n_uniq_out, sizeof(g_U), hipMemcpyDeviceToHost));
  printf("rows: library %lld, oracle %lld; distinct rows in the batch: library %lld, oracle %lld; entries %lld\n",
         (long long)g_n_rows, (long long)n_rows, (long long)g_U, (long long)U, (long long)nnz);
  if (g_n_rows != n_rows || g_U != U || n_rows <= PRE) { printf("FAIL counts\n"); ++failures; }
  void *h;
  h = to_host(d_rows0, sizeof(int32_t) * PRE); check_equal_bytes("rows of the pre-inserted IDs", h, o_rows0, sizeof(int32_t) * PRE); free(h);
  h = to_host(d_rows, sizeof(int32_t) * (size_t)nnz); check_equal_bytes("rows", h, o_rows, sizeof(int32_t) * (size_t)nnz); free(h);
  h = to_host(d_keys_out, sizeof(uint64_t) * (size_t)n_rows);
  check_equal_bytes("exported row -> key map", h, oracle_table_row_keys(ot), sizeof(uint64_t) * (size_t)n_rows); free(h);
  h = to_host(io.uniq_rows_out, sizeof(int32_t) * (size_t)U); check_equal_bytes("merged order (rows)", h, o_uniq, sizeof(int32_t) * (size_t)U); free(h);
  h = to_host(io.uniq_keys_out, sizeof(uint64_t) * (size_t)U); check_equal_bytes("merged order (keys)", h, o_ukeys, sizeof(uint64_t) * (size_t)U); free(h);
  h = to_host(io.counts_out, sizeof(int32_t) * (size_t)U); check_equal_bytes("merged counts", h, o_counts, sizeof(int32_t) * (size_t)U); free(h);
  h = to_host(d_P_lr, sizeof(float) * K * B); check_close("P_lr", (float *)h, oP_lr, (size_t)K * B); free(h);
  h = to_host(d_P_sum, sizeof(float) * K * B * D); check_close("P_sum", (float *)h, oP_sum, (size_t)K * B * D); free(h);
  h = to_host(d_P_sq, sizeof(float) * K * B); check_close("P_sq", (float *)h, oP_sq, (size_t)K * B); free(h);
  h = to_host(d_pool, sizeof(float) * B * F * D); check_close("pool", (float *)h, o_pool, (size_t)B * F * D); free(h);
  h = to_host(d_A_lr, sizeof(float) * B); check_close("A_lr", (float *)h, oA_lr, B); free(h);
  h = to_host(d_A_sum, sizeof(float) * B * D); check_close("A_sum", (float *)h, oA_sum, (size_t)B * D); free(h);
  h = to_host(d_fm2, sizeof(float) * B); check_close("fm2", (float *)h, o_fm2, B); free(h);
  h = to_host(io.merged_out, sizeof(float) * (size_t)U * (D + 1)); check_close("merged gradients", (float *)h, o_merged, (size_t)U * (D + 1)); free(h);
  h = to_host(cfg.emb, sizeof(float) * (size_t)n_rows * D); check_close_f("updated emb", (float *)h, oracle_table_emb(ot), (size_t)n_rows * D); free(h);
  h = to_host(cfg.w, sizeof(float) * (size_t)n_rows); check_close_f("updated w", (float *)h, oracle_table_w(ot), (size_t)n_rows); free(h);
  h = to_host(cfg.acc_emb, sizeof(float) * (size_t)n_rows * D); check_close_f("updated acc_emb", (float *)h, oracle_table_acc_emb(ot), (size_t)n_rows * D); free(h);
  h = to_host(cfg.acc_w, sizeof(float) * (size_t)n_rows); check_close_f("updated acc_w", (float *)h, oracle_table_acc_w(ot), (size_t)n_rows); free(h);

  DES_OK_(des_table_destroy(t));
  oracle_table_destroy(ot);
  HIP_OK(hipStreamDestroy(stream));
  if (failures) { printf("des_host_step: %d check(s) FAILED\n", failures); return 1; }
  printf("des_host_step: PASS\n");
  return 0;
}
