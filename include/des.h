/*
 * libdes -- the hot path of Distributed Equivalent Substitution (DES) training
 * (arXiv 1909.04823) for one AMD MI355X (gfx950): the sparse operators and their table, the first
 * fully-connected layer under DES, and the dense remainder of a model step.  Plain C interface.
 *
 * A DES worker owns one shard of the sparse weights of a CTR model and replaces each
 * weights-rich operator by a sub-operator on its shard whose small result is aggregated
 * across workers (Algorithm 1).  On one GPU the K workers are K logical partitions of one
 * table in HBM and the aggregation is an on-device sum over K.
 *
 * Conventions for every entry point
 *   - C linkage, returns des_status_t, never throws.
 *   - Every pointer named "device" is a device (HBM) pointer owned by the caller; it must
 *     stay valid until the stream the call was given has drained.  Pointers named "host"
 *     are ordinary host pointers.  The library allocates no device memory: all storage,
 *     including scratch, is handed over in des_table_config_t or in a workspace argument.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only
 *     enqueue work and return, except des_table_create/size/status/destroy/migrate and
 *     des_profile_read, which synchronise.
 *   - Errors the host can see (null pointers, bad sizes, buffers too small) return at once
 *     and enqueue nothing.  Errors only the device can see live in device memory and are read
 *     by des_table_status.  "Table full" is sticky: the call that would exceed the capacity
 *     inserts nothing, and every later insert on that table degrades to a lookup, until
 *     des_table_clear_status.  A reserved key is not: that entry is treated as absent (row -1),
 *     the rest of the call proceeds, and the table keeps a note that des_table_status reports.
 *   - Calls on one table must be ordered (same stream, or externally synchronised); two
 *     tables are independent.
 *   - Supported shapes: dim a power of two in [4, 256]; 1 <= num_shards <= 256;
 *     capacity_rows <= 2^31 - 2; nnz < 2^31; B*F < 2^31; for the forward calls
 *     8*num_shards*(dim+2) + 4*(F+1) + 4096 <= 65536 (bytes of on-chip memory per sample).
 *   - Not checked (the caller's contract): offsets are non-decreasing with offsets[0] = 0 and
 *     offsets[B*F] = nnz; `rows` passed to the forward / backward calls were produced by
 *     des_table_find / des_table_insert on the same table for the same keys.
 *
 * Conventions the paper leaves open, fixed here (the CPU oracle implements the same text):
 *   mix64(z)      finalizer of SplitMix64: z=(z^(z>>30))*0xBF58476D1CE4E5B9;
 *                 z=(z^(z>>27))*0x94D049BB133111EB; z^(z>>31).
 *   shard         DES_SHARD_KEY_HASH: (uint32)(mix64(key)>>32) mod K;
 *                 DES_SHARD_FIELD_MOD: field mod K (Section 5, "i = f mod N").
 *   row numbers   dense 0..n_rows-1; the distinct unseen keys of one insert/find call get
 *                 consecutive rows in the order of their first occurrence in the call, i.e.
 *                 the result of a sequential insert loop over the keys.
 *   initialiser   column c of a row inserted without values is
 *                 ((mix64(key ^ mix64(seed+c)) >> 40) * 2^-24 - 0.5) * (float)(2*sqrt(3)*init_scale)
 *                 (c < dim latent, c == dim the LR weight); optimizer state starts at 0.
 *   reserved key  0xFFFFFFFFFFFFFFFF marks an empty slot; as an ID it is never found and never inserted.
 */
#ifndef DES_H_
#define DES_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct des_table des_table_t;   /* opaque host handle */

typedef enum {
  DES_OK = 0,
  DES_ERR_INVALID_ARG = 1,   /* null / negative / unsupported shape / misaligned            */
  DES_ERR_INVALID_KEY = 2,   /* the reserved key was passed (device-detected, not blocking) */
  DES_ERR_FULL = 3,          /* capacity_rows or the slot array exhausted (sticky)          */
  DES_ERR_WORKSPACE = 4,     /* slots or workspace smaller than des_table_query_bytes says  */
  DES_ERR_DEVICE = 5         /* a HIP runtime call failed                                   */
} des_status_t;

typedef enum { DES_SHARD_KEY_HASH = 0, DES_SHARD_FIELD_MOD = 1 } des_shard_policy_t;
typedef enum { DES_OPT_NONE = 0, DES_OPT_SGD = 1, DES_OPT_ADAGRAD = 2, DES_OPT_ADAM = 3, DES_OPT_FTRL = 4 } des_opt_t;
typedef enum { DES_MISS_ZERO = 0, DES_MISS_INSERT = 1 } des_miss_t;

/* Table description.  The caller allocates every buffer (16-byte aligned). */
typedef struct {
  int32_t dim;                 /* D, latent dimension                                        */
  int64_t capacity_rows;       /* fixed for the table's life; to grow, des_table_migrate      */
  int32_t num_shards;          /* K logical DES workers                                      */
  int32_t shard_policy;        /* des_shard_policy_t                                         */
  int32_t opt;                 /* des_opt_t the table is meant for; only checked at creation: the state
                                  arrays that optimizer needs must be given (ADAGRAD acc_*, ADAM acc_* and
                                  acc2_*, FTRL acc_w and acc2_w).  DES_OPT_NONE skips the check.  The optimizer
                                  itself comes with every update call, which checks its own arrays again   */
  uint64_t init_seed;
  float init_scale;            /* standard deviation of the initialiser                      */
  float *emb;                  /* device [capacity, D]   latent vectors v                    */
  float *w;                    /* device [capacity]      LR (first-order) weights            */
  float *acc_emb;              /* device [capacity, D]   Adagrad accumulators (or NULL)      */
  float *acc_w;                /* device [capacity]                                          */
  uint64_t *row_keys;          /* device [capacity]      row -> key                          */
  void *slots;                 /* device, slots_bytes from des_table_query_bytes             */
  size_t slots_bytes;
  void *workspace;             /* device scratch for sort / scan / merge                     */
  size_t workspace_bytes;
  float *acc2_emb;             /* device [capacity, D]   second state array (Adam) or NULL   */
  float *acc2_w;               /* device [capacity]      second state (Adam, FTRL) or NULL   */
} des_table_config_t;

/* One batch in CSR form (Section 3.2.1: input X; variable-length multi-hot fields).
 * Bag (b,f) holds entries offsets[b*F+f] .. offsets[b*F+f+1]-1; every entry is one feature
 * term, also when a key repeats.  vals are the feature values x (NULL: all 1). */
typedef struct {
  int64_t B;
  int32_t F;
  int64_t nnz;
  const uint64_t *keys;        /* device [nnz]                                               */
  const int32_t *offsets;      /* device [B*F+1], offsets[0]=0, offsets[B*F]=nnz             */
  const float *vals;           /* device [nnz] or NULL                                       */
} des_batch_t;

/* Bytes needed for `slots` (depends on capacity_rows) and for `workspace` so that calls with
 * up to max_n keys per insert/find and up to max_n entries per batch fit. */
des_status_t des_table_query_bytes(const des_table_config_t *cfg, int64_t max_n,
                                   size_t *slots_bytes, size_t *workspace_bytes);

/* Dynamic hash table, Section 5 "Dynamic Hash Table": lookup, insert of an initialized
 * weight for a new feature ID (update is des_backward_update_*).
 * create: validates cfg, empties the slot array (synchronises the null stream). */
des_status_t des_table_create(const des_table_config_t *cfg, des_table_t **out);
des_status_t des_table_destroy(des_table_t *t);

/* Insert-if-absent of n keys (device).  values: device [n, D+1] (D latent then LR weight) or
 * NULL for the initialiser; a repeated new key takes the values of its first occurrence; keys
 * already present keep their weights.  rows_out: device [n] or NULL.  0 <= n <= max_n. */
des_status_t des_table_insert(des_table_t *t, const uint64_t *keys, int64_t n,
                              const float *values, int32_t *rows_out, void *stream);

/* rows_out[i] = row of keys[i]; absent keys give -1 (DES_MISS_ZERO) or are inserted with
 * initialiser weights first (DES_MISS_INSERT), so one call looks up and grows the table. */
des_status_t des_table_find(des_table_t *t, const uint64_t *keys, int64_t n, int32_t miss,
                            int32_t *rows_out, void *stream);

des_status_t des_table_size(des_table_t *t, int64_t *n_rows_host);   /* synchronises */

/* Device-side condition of the table (synchronises): DES_ERR_FULL (or DES_ERR_DEVICE) if the sticky status is
 * set, else DES_ERR_INVALID_KEY if a reserved key was passed since the last des_table_clear_status, else DES_OK. */
des_status_t des_table_status(des_table_t *t);

/* Starts the status over (synchronises).  After DES_ERR_FULL the table is exactly as before the failed call
 * except that the keys that call tried to add hold a hash slot without a row; they get their row the next time
 * they are inserted.  The table is still as full as it was: make room with des_table_compact, or move to a
 * larger table with des_table_migrate (both rebuild the slots and drop such leftovers), then insert again.
 * Also forgets the reserved keys seen so far. */
des_status_t des_table_clear_status(des_table_t *t);

/* Third table operation besides lookup and insert (Section 5, "Dynamic Hash Table"): the IDs the table holds.
 * Copies row_keys[0 .. min(n_rows, max_rows)) to row_keys_out (device, 8-byte aligned, max_rows entries);
 * entry r is the ID of row r.  The row count is read on the device, so no synchronisation; size the buffer from
 * des_table_size or the capacity.  (des_table_config_t.row_keys is the same map, owned by the caller.) */
des_status_t des_table_export_keys(des_table_t *t, uint64_t *row_keys_out, int64_t max_rows, void *stream);

/* ---- Growth and eviction (Section 1, "Dynamic Features": the parameter set of a streaming
 * recommender changes and grows over time; Section 5).  The paper gives the requirement, not a
 * mechanism; here rows migrate into a second table.
 *
 * des_table_migrate moves the rows r of `src` with keep[r] != 0 (keep: device, one byte per row of
 * src; null keeps all = pure growth) into `dst`, a table created with des_table_create that is still
 * empty, of the same dim and of any capacity that holds the kept rows.  Row i of dst is the i-th
 * kept row of src (ascending row order) with its key, weights and every optimizer-state array both
 * tables have; state arrays only dst has are zeroed for the moved rows.  dst's hash slots are built
 * from the moved keys; src is left untouched (destroy it, or keep it as a snapshot).  src_aux /
 * dst_aux (device, one uint32 per row, both or dst only or neither) is a caller array moved along
 * with the rows, e.g. the last_seen stamps below.  The arrays of the two tables must not overlap.
 * dst's workspace must hold des_table_migrate_bytes(rows of src) bytes, else DES_ERR_WORKSPACE.
 * If the kept rows exceed dst's capacity nothing is moved and DES_ERR_FULL is returned (dst stays
 * empty and usable).  A maintenance call: it synchronises with the stream and returns when the
 * migration is complete; *n_rows_out (host, may be null) = rows of dst. */
des_status_t des_table_migrate_bytes(int64_t n_rows, size_t *workspace_bytes);
des_status_t des_table_migrate(des_table_t *src, const uint8_t *keep, des_table_t *dst, const uint32_t *src_aux,
                               uint32_t *dst_aux, int64_t *n_rows_out, void *stream);

/* The same eviction inside one table, for tables too large for a second copy: the rows r with
 * keep[r] != 0 close up towards row 0 in ascending order (row i afterwards is the i-th kept row, with its
 * key, weights and every state array; `aux`, if not null, is moved along), the row count drops to the
 * number kept and the hash slots are rebuilt.  The result equals des_table_migrate into an empty table of
 * the same capacity.  The arrays are walked in chunks through `staging` (device, 16-byte aligned; any size
 * from 4096 * dim * 4 bytes up; larger means fewer launches), the row numbering uses the table's own
 * workspace (8 bytes per row; DES_ERR_WORKSPACE if it is smaller).  keep == NULL keeps everything and is
 * a no-op.  Synchronises with the host like des_table_migrate; n_rows_out (host, may be null) receives the
 * new row count.  Rows found before the call are stale afterwards. */
des_status_t des_table_compact(des_table_t *t, const uint8_t *keep, uint32_t *aux, void *staging, size_t staging_bytes,
                               int64_t *n_rows_out, void *stream);

/* Helpers for a least-recently-seen eviction policy.  last_seen: device, one uint32 per row, owned
 * and zero-initialised by the caller.  mark_seen: last_seen[rows[e]] = stamp for every e < n with
 * rows[e] >= 0 (rows as written by des_table_find).  select_recent: keep[r] = last_seen[r] >= min_stamp
 * for r < n_rows. */
des_status_t des_table_mark_seen(const int32_t *rows, int64_t n, uint32_t stamp, uint32_t *last_seen, void *stream);
des_status_t des_table_select_recent(const uint32_t *last_seen, int64_t n_rows, uint32_t min_stamp, uint8_t *keep,
                                     void *stream);
                       /* synchronises; sticky device status */

/* Sub-operators (Algorithm 1: M_j(w_i, x_i) for every shard i), rows from des_table_find.
 * Entries with row -1 contribute nothing.  Outputs are fully overwritten.
 *   lr   Eq. (lr_m1), Section 4.1:      P_lr [K,B]     sum of x*w over the shard's entries
 *   fm   Eq. (fm_m1m2), Section 4.2:    P_sum[K,B,D]   sum of x*v ;  P_sq[K,B] sum of <x*v,x*v>
 *   pool Section 4.3 (latent vectors aggregated by field before concatenation):
 *        dense_k=1: P_pool[K,B,F,D] per-shard bag sums;
 *        dense_k=0: P_pool[B,F,D], the K shards' bag sums already added on chip.
 * des_partial_forward computes all of them in one pass over the rows (any output NULL to
 * skip; pool in the dense_k=0 form). */
des_status_t des_partial_forward_lr(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                    float *P_lr, void *stream);
des_status_t des_partial_forward_fm(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                    float *P_sum, float *P_sq, void *stream);
des_status_t des_partial_forward_pool(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                      float *P_pool, int32_t dense_k, void *stream);
des_status_t des_partial_forward(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                 float *P_lr, float *P_sum, float *P_sq, float *pool, void *stream);

/* Aggregation over the K shards, Eq. (1) with AllReduce-sum: out[i] = sum_s P[s*n + i].
 * P device [K,n], out device [n]. */
des_status_t des_aggregate_partials(const float *P, int32_t K, int64_t n, float *out, void *stream);

/* The aggregations of one forward pass and the FM substitution operator in a single launch:
 * A_lr[B], A_sum[B,D], A_sq[B] = sums over the K shards of P_lr[K,B], P_sum[K,B,D], P_sq[K,B] (Eq. (1)) and
 * fm2[B] as below, formed from the double sums before they are rounded.  The LR group (P_lr, A_lr) or the
 * FM group (P_sum, P_sq, A_sum, A_sq, optional fm2) may be null, not both.  Same results as the separate
 * calls up to the last bit of fm2.  D a multiple of 4; P_sum and A_sum 16-byte aligned. */
des_status_t des_aggregate_forward(const float *P_lr, const float *P_sum, const float *P_sq, int32_t K, int64_t B,
                                   int32_t D, float *A_lr, float *A_sum, float *A_sq, float *fm2, void *stream);

/* Substitution operator of FM order 2, Eq. (des_fm2): fm2[b] = (<A_sum[b],A_sum[b]> - A_sq[b])/2. */
des_status_t des_fm_finalize(const float *A_sum, const float *A_sq, int64_t B, int32_t D,
                             float *fm2, void *stream);

/* First fully-connected layer of the DNN tower under DES, Section 4.3, Eq. (dnn_bmm) and Eq. (dnn_des).
 * V^T (the pooled embeddings concatenated over fields, pool[B,F,D] = [B, F*D]) and W[F*D, H] are
 * both cut along the field dimension; shard s = f mod K owns field f (the placement of Section 5)
 * and forms M1(V_s, W_s) = V_s^T W_s:
 *     Y_partial[s,b,h] = sum over fields f of shard s, d < D of  pool[b,f,d] * W[f*D+d, h].
 * des_aggregate_partials(Y_partial, K, B*H) then gives the layer output.  A shard with no field
 * (K > F) writes zeros.  fp32 in and out; products accumulate in fp32 on the matrix cores in
 * ascending k; a contraction deeper than 1024 products is summed in runs of 128 products that are
 * then added up (two-level fp32 summation), which keeps a sum over a whole batch within the
 * 1e-5 / 1e-6 bound of the rest of the library.
 * pool, W, Y_partial: device, 16-byte aligned, row-major as written; Y_partial [K,B,H] is owned by
 * the caller and fully overwritten.  D and H multiples of 4, 1 <= K <= 256, B < 2^31, F*D < 2^31,
 * else DES_ERR_INVALID_ARG.  B == 0 is a no-op (for the backward too: dW is then left untouched). */
des_status_t des_dnn_partial_forward(const float *pool, const float *W, int64_t B, int32_t F, int32_t D,
                                     int32_t H, int32_t K, float *Y_partial, void *stream);

/* Backward of that layer (Section 3.2.2: the gradient dY[B,H] of the aggregate reaches every shard
 * unchanged, each shard differentiates its own block, nothing is exchanged):
 *     g_pool[b, j] = sum_h dY[b,h] * W[j,h]        (the g_pool input of des_backward_update*)
 *     dW[j, h]     = sum_b pool[b,j] * dY[b,h]      j = f*D + d
 * Either output may be null (skipped), not both.  dW is computed in up to 16 slices of samples
 * that are summed in double; the slices live in `workspace` (device, 16-byte aligned, at least
 * des_dnn_backward_bytes() bytes; not needed, and may be null, when dW is not asked for or the
 * batch is so small that one slice is used).  Same shape rules as the forward; DES_ERR_WORKSPACE if
 * the workspace is too small.  W itself is updated by des_dense_update with dW.  A plain dense layer
 * Y = X W (X [B,Hin]) is the same pair of calls with F = 1, D = Hin, K = 1. */
des_status_t des_dnn_backward_bytes(int64_t B, int32_t F, int32_t D, int32_t H, size_t *workspace_bytes);
des_status_t des_dnn_backward(const float *pool, const float *W, const float *dY, int64_t B, int32_t F,
                              int32_t D, int32_t H, float *g_pool, float *dW, void *workspace,
                              size_t workspace_bytes, void *stream);

/* Backward (Section 3.2.2, back-propagation phase: the gradient of each aggregate goes
 * unchanged to every shard's sub-operator; no exchange), duplicate-key merge and optimizer
 * update (Section 5, "Dynamic Hash Table": a weight's gradient is applied where the weight lives).
 * Entry e of bag (b,f), value x, row r:   d/dw_r = x*g_lr[b]
 *     d/dv_r = x*( g_fm[b]*(A_sum[b,:] - x*v_r) + g_pool[b,f,:] )
 * summed over the entries of a row; rows are visited in ascending row order; the update reads
 * pre-update weights.   SGD: theta -= lr*G.   Adagrad: a += G*G; theta -= lr*G/(sqrt(a)+eps).
 * Inputs (device; NULL = term absent; g_fm and A_sum go together).  Optional outputs for
 * inspection (device; NULL to skip, then nothing is materialised): uniq_rows[<=nnz] ascending,
 * uniq_keys, counts, merged[U, D+1] (D latent then LR weight), n_uniq (int64 scalar). */
typedef struct {
  const float *g_lr;       /* [B]       */
  const float *g_fm;       /* [B]       */
  const float *A_sum;      /* [B,D]  aggregated FM vector returned by the forward pass */
  const float *g_pool;     /* [B,F,D]   */
  int32_t *uniq_rows_out;
  uint64_t *uniq_keys_out;
  int32_t *counts_out;
  float *merged_out;
  int64_t *n_uniq_out;
} des_backward_io_t;

/* Optional first half of the calls below, for overlap.  Sorting the batch's entries by row and cutting
 * the sorted list into segments needs the batch and `rows` only, not the gradients, so it can run on a
 * second stream while the forward pass and the loss head run on the first.  The sorted form stays in
 * the table's workspace; the next des_backward_update* / des_backward_merge call for the same batch
 * (same offsets, vals and rows pointers, same sizes) skips that half, any other call recomputes it.
 * Any des_table_insert or des_table_find on the table in between discards it (an insert reuses the
 * workspace; a lookup may be refilling the rows array).  The caller orders the streams: prepare after the find that wrote `rows`, the update
 * after prepare.  Results are identical with and without this call. */
des_status_t des_backward_prepare(des_table_t *t, const des_batch_t *batch, const int32_t *rows, void *stream);

des_status_t des_backward_update_sgd(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                     const des_backward_io_t *io, float lr, void *stream);
des_status_t des_backward_update_adagrad(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                         const des_backward_io_t *io, float lr, float eps, void *stream);
/* The optimizer setting of the paper's experiments (Section 6, "Parameter Settings": FTRL for
 * order-1 components, AdaGrad or Adam for the embeddings), with the same merge as above.  The
 * optimizers themselves are the published ones, restated:
 *   Adam (Kingma & Ba), lazily per touched row, global step t = `step` >= 1:
 *     m = b1*m + (1-b1)*G;  v = b2*v + (1-b2)*G*G;
 *     theta -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)          state: acc = m, acc2 = v
 *   FTRL-Proximal (McMahan et al.), order-1 weights only:
 *     sigma = (sqrt(n+G*G) - sqrt(n))/alpha;  z += G - sigma*w;  n += G*G;
 *     w = |z| <= l1 ? 0 : -(z - sign(z)*l1) / ((beta + sqrt(n))/alpha + l2)   state: acc_w = n, acc2_w = z
 * opt_emb is SGD, ADAGRAD or ADAM; opt_w is SGD, ADAGRAD, ADAM or FTRL.  The state arrays an
 * optimizer needs must have been given in des_table_config_t, else DES_ERR_INVALID_ARG. */
typedef struct {
  int32_t opt_emb, opt_w;       /* des_opt_t */
  float lr, eps;                /* SGD / Adagrad / Adam */
  float beta1, beta2;           /* Adam */
  int64_t step;                 /* Adam: t >= 1 */
  float ftrl_alpha, ftrl_beta, ftrl_l1, ftrl_l2;
} des_optimizer_t;
des_status_t des_backward_update(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                 const des_backward_io_t *io, const des_optimizer_t *optimizer, void *stream);

/* Merge only (no weight changes); fills the optional outputs. */
des_status_t des_backward_merge(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                const des_backward_io_t *io, void *stream);

/* ---- DCN cross layer under DES (Section 4, the paragraph on DCN; the layer is the cited DCN paper's
 *     x_{l+1} = x_0 (x_l^T w_l) + b_l + x_l,      all vectors of length d = F*D,
 * x_0 the concatenated embedding output [B,F,D] of des_partial_forward_pool).  The paper cuts w_l along
 * d, lets every process form the dot product over its own part first, a scalar per sample, and sums
 * the scalars:  y = x_0 * (+)(x_local^T w_local) + b + x.  Columns go with the field they belong to:
 * column j = f*D + c is held by shard f mod K (Section 5).
 *
 * des_cross_partial: the sub-operator.  P[s,b] = sum over the columns j of shard s of xl[b,j] * w[j]
 * (double sum in a fixed order, rounded once).  xl [B,F,D], w [F*D], P [K,B] fully overwritten.  The K
 * scalars of a sample are summed with des_aggregate_partials(P, K, B, s).  K = 1 gives the plain row
 * dot product xl w.
 * des_cross_apply: the remaining operator, the same on every process: y[b,j] = x0[b,j] * s[b] + bias[j]
 * + xl[b,j].  y may alias xl.
 * All pointers: device, 16-byte aligned, row-major, owned by the caller.  D and d multiples of 4,
 * F*D <= 2^30, K >= 1, else DES_ERR_INVALID_ARG.  B == 0 is a no-op. */
des_status_t des_cross_partial(const float *xl, const float *w, int64_t B, int32_t F, int32_t D, int32_t K, float *P,
                               void *stream);
des_status_t des_cross_apply(const float *x0, const float *xl, const float *s, const float *bias, int64_t B,
                             int64_t d, float *y, void *stream);

/* Backward of one cross layer for the gradient g_y[B,d] of its output (Section 3.2.2: the gradient of
 * the aggregated scalar reaches every sub-operator unchanged).  With s the aggregated scalar of the
 * forward pass and g_s[b] = <g_y[b,:], x0[b,:]>:
 *     g_xl[b,j] = g_y[b,j] + g_s[b] w[j]           dw[j] = sum_b g_s[b] xl[b,j]
 *     g_x0[b,j] (+)= g_y[b,j] s[b]                 db[j] = sum_b g_y[b,j]
 * x_0 feeds every layer, so the layers' shares of its gradient add up: accumulate_g_x0 != 0 adds to
 * what g_x0 holds, 0 overwrites it.  (The first layer's input is x_0 itself: its g_xl is one more
 * share: pass g_xl == NULL for that layer and it is added into g_x0 as well.)  Sums in double, the batch
 * sums as per-slice partials added in slice order.  g_xl may alias g_y.  workspace: device, 256-byte aligned, des_cross_backward_bytes(B, d)
 * bytes, else DES_ERR_WORKSPACE.  B == 0 writes dw = db = 0 and touches nothing else. */
des_status_t des_cross_backward_bytes(int64_t B, int64_t d, size_t *workspace_bytes);
des_status_t des_cross_backward(const float *x0, const float *xl, const float *w, const float *s, const float *g_y,
                                int64_t B, int64_t d, float *g_xl, float *g_x0, int32_t accumulate_g_x0, float *dw,
                                float *db, void *workspace, size_t workspace_bytes, void *stream);

/* Backward of the sub-operator alone, for a gradient g_s[B] of its aggregated scalar (e.g. when the
 * scalar is a term of the logit: the output unit's weights on the cross network's result):
 *     g_xl[b,j] = g_s[b] w[j]      dw[j] = sum_b g_s[b] xl[b,j].
 * g_xl may be null (only dw wanted).  Same workspace as des_cross_backward. */
des_status_t des_cross_partial_backward(const float *xl, const float *w, const float *g_s, int64_t B, int64_t d,
                                        float *g_xl, float *dw, void *workspace, size_t workspace_bytes, void *stream);

/* The whole cross network in two passes over x_0.  Every layer adds a multiple of x_0 and a bias to its
 * input, so x_l[b,:] = gamma_l[b] x_0[b,:] + c_l with gamma_0 = 1, gamma_{l+1} = gamma_l + s_l,
 * c_l = b_0 + ... + b_{l-1}, and s_l[b] = gamma_l[b] t_l[b] + <c_l, w_l> where t_k[b] = <x_0[b,:], u_k>.
 * U [m,d] holds the n layers' weights w_0 .. w_{n-1} and, as its last row, the weights u_n of the output
 * unit on the network's result x_n (m = n + 1 <= 8); bias is [n,d].  The dot products t_k are the
 * sub-operators (cut along d, one scalar per sample, shard and row of U; under DES one exchange of m
 * scalars per sample serves the whole network); the rest is arithmetic on scalars.  Results equal the
 * layer-by-layer calls above up to the rounding of the intermediate x_l, which are never formed.
 *
 * des_cross_net_partial: P[s,b,k] = sum over the columns j of shard s of x0[b,j] U[k,j]; P [K,B,m].  Sum the
 *   shards with des_aggregate_partials(P, K, B*m, t) to get t [B,m].
 * des_cross_net_forward: gamma [B,m] (gamma_0 .. gamma_n) and c[b] = <x_n[b,:], u_n>, the network's term of
 *   the logit.
 * des_cross_net_backward, for the gradient g[B] of that term: g_x0[b,:] (+)= sum_k beta_k[b] U[k,:] with
 *   beta_l = g_s_l gamma_l, beta_n = g gamma_n, g_s_l = g t_n + sum_{l'>l} g_s_l' t_l' (accumulate_g_x0 as above);
 *   dU[k,:] = sum_b beta_k[b] x0[b,:] + c_k sum_b g_s_k (k = n: sum_b g);  dbias[l,:] = the batch sum of the
 *   gradient of x_{l+1}.  Batch sums in double, per-slice partials added in slice order.
 * workspace: device, 256-byte aligned, des_cross_net_bytes(B, d, n) bytes, the same buffer for forward and
 * backward is fine.  Pointer, alignment and size rules as for the layer-by-layer calls. */
des_status_t des_cross_net_bytes(int64_t B, int64_t d, int32_t n_layers, size_t *workspace_bytes);
des_status_t des_cross_net_partial(const float *x0, const float *U, int64_t B, int32_t F, int32_t D, int32_t m,
                                   int32_t K, float *P, void *stream);
des_status_t des_cross_net_forward(const float *t, const float *U, const float *bias, int64_t B, int64_t d,
                                   int32_t n_layers, float *gamma, float *c, void *workspace, size_t workspace_bytes,
                                   void *stream);
des_status_t des_cross_net_backward(const float *x0, const float *U, const float *bias, const float *t,
                                    const float *gamma, const float *g, int64_t B, int64_t d, int32_t n_layers,
                                    float *g_x0, int32_t accumulate_g_x0, float *dU, float *dbias, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* ---- The dense remainder of a model step --------------------------------------------------------
 * After the aggregated weights-rich operators every process computes the same thing (Section 3.2.1);
 * Section 4's models differ in which components feed the output (LR: first order; FM: + second
 * order; W&D: first + high order; DeepFM: all three) and Section 4.1 gives the sigmoid output.  The
 * paper prints no formula for the tower's activation or the loss reduction; ReLU and the mean
 * log-loss (the quantity Section 6 reports) are used.  All pointers device, fp32, row-major. */

/* Hidden-layer epilogue fused into the aggregation of Eq. (1):
 *     out[r,h] = act( sum_s P[s,r,h] + bias[h] ),  act = max(.,0) when relu != 0, identity otherwise.
 * P [K,rows,H], bias [H] or null, out [rows,H]; H a multiple of 4, all 16-byte aligned.  Shard sum in
 * double, rounded once. */
des_status_t des_aggregate_bias_act(const float *P, int32_t K, int64_t rows, int32_t H, const float *bias,
                                    int32_t relu, float *out, void *stream);

/* Bytes of the workspace the three calls below take, for layers up to H_max wide. */
des_status_t des_dense_workspace_bytes(int32_t H_max, size_t *workspace_bytes);

/* Backward of that epilogue: dZ[r,h] = dA[r,h] where A[r,h] > 0 (everywhere when relu == 0), else 0;
 * dbias[h] = sum_r dZ[r,h] (double, fixed order).  A is the forward output.  dZ may alias dA. */
des_status_t des_bias_act_backward(const float *A, const float *dA, int64_t rows, int32_t H, int32_t relu,
                                   float *dZ, float *dbias, void *workspace, size_t workspace_bytes, void *stream);

/* des_bias_act_backward for callers that cannot allocate or hand over device memory: code under HIP graph
 * capture, serving loops and harnesses in which hipMalloc is forbidden.  Same arguments, kernels and results,
 * but the per-slice column partials live in a 2 MiB array inside the library's own device image instead of a
 * workspace; the call allocates nothing.  H <= 4096, else DES_ERR_WORKSPACE (nothing is enqueued).  The first
 * call on a GPU looks up that GPU's copy of the array (a host-side query, no allocation; make it outside a
 * capture).  All calls on one GPU share the array: two calls that overlap in time on one GPU (different
 * streams, no ordering) race; calls on one stream, or ordered by events, do not.  Nothing needs clearing
 * between calls: each call writes every partial it later reads. */
des_status_t des_bias_act_backward_static(const float *A, const float *dA, int64_t rows, int32_t H, int32_t relu,
                                          float *dZ, float *dbias, void *stream);

/* Output unit, loss and gradients for one batch:
 *     logit[b] = b0 + A_lr[b] + fm2[b] + <a[b,:], w_out>        (absent components: null pointers)
 *     p = 1/(1+exp(-logit));   loss = mean_b( -y log p - (1-y) log(1-p) ), evaluated as
 *     log(1+e^z) - y z in an overflow-free form;   g_logit[b] = (p[b]-y[b])/B,
 * which is d loss/d logit and therefore also the upstream gradient g_lr and g_fm of
 * des_backward_update*;  da[b,h] = g_logit[b] w_out[h];  dw_out[h] = sum_b g_logit[b] a[b,h];
 * db0 = sum_b g_logit[b].  Arithmetic in double, outputs fp32.  a [B,H] with w_out [H] (both or
 * neither); b0, loss_out, db0_out point to one float; labels [B] in {0,1}.  logit_out, p_out,
 * loss_out, da, dw_out, db0_out may be null.  B >= 1. */
des_status_t des_head(const float *A_lr, const float *fm2, const float *a, const float *w_out, const float *b0,
                      const float *labels, int64_t B, int32_t H, float *logit_out, float *p_out, float *loss_out,
                      float *g_logit, float *da, float *dw_out, float *db0_out, void *workspace,
                      size_t workspace_bytes, void *stream);

/* One optimizer step on a dense parameter array (every coordinate, every step): optimizer->opt_emb
 * (SGD, ADAGRAD, ADAM or FTRL) with the formulas given at des_optimizer_t; s1 = Adagrad accumulator /
 * Adam m / FTRL n, s2 = Adam v / FTRL z (null when the optimizer keeps no such state).  In place. */
des_status_t des_dense_update(float *theta, const float *grad, float *s1, float *s2, int64_t n,
                              const des_optimizer_t *optimizer, void *stream);

/* Checks the part of the contract the other calls take on trust, for callers that cannot vouch for
 * their batches (the kernels index memory with these values; a broken batch makes them fault):
 * offsets[0] == 0, offsets non-decreasing, offsets[B*F] == nnz, and, when `rows` is given, every
 * rows[e] in [-1, rows of the table).  Reads the whole batch on the device and synchronises.
 * Returns DES_OK, or DES_ERR_INVALID_ARG with *first_bad (host, may be null) = index of the first
 * offending offset (0 .. B*F), or B*F + 1 + e for the first offending rows[e]. */
des_status_t des_batch_validate(des_table_t *t, const des_batch_t *batch, const int32_t *rows, int64_t *first_bad,
                                void *stream);

/* Measurement aids (used by the benchmark, not by a training step): kernels that perform only the table accesses
 * of the forward gather and of the row update, on the caller's own index streams, with the lane mapping and the
 * load / store instructions of the real kernels and nothing else.  Their rates are the ceilings of this GPU for
 * these access patterns, against which the real kernels' times are read where the streaming figure of 8 TB/s is
 * not the limit that applies.
 * des_ceiling_gather: every entry e < n with 0 <= rows[e] < n_rows reads the dim floats of row rows[e] of emb
 *   (row r starts at emb + r * stride floats; stride = dim for a dense array) and, if w is not null, the one float
 *   w[r * w_stride], as the forward pass does for the first-order weight; one float per wave is left in `sink`
 *   (device, des_ceiling_gather_bytes bytes) so that the loads are live.  Logical bytes: 4 * dim (+ 4) per entry.
 * des_ceiling_update: for every u < n_uniq, row uniq_rows[u] (0 <= row < n_rows, else skipped) of emb and of acc
 *   (both with `stride` floats between rows) is read and written back unchanged.  Logical bytes: 16 * dim per row.
 * dim as for a table; stride a multiple of 4, >= dim; pointers device, emb / acc 16-byte aligned. */
des_status_t des_ceiling_gather_bytes(size_t *sink_bytes);
des_status_t des_ceiling_gather(const float *emb, int32_t dim, int64_t stride, const float *w, int64_t w_stride, int64_t n_rows,
                                const int32_t *rows, int64_t n, float *sink, size_t sink_bytes, void *stream);
des_status_t des_ceiling_update(float *emb, float *acc, int32_t dim, int64_t stride, int64_t n_rows, const int32_t *uniq_rows,
                                int64_t n_uniq, void *stream);

/* Per-kernel timing with HIP events recorded on the caller's stream around every launch.
 * enable != 0 starts collecting and clears earlier records.  des_profile_read synchronises,
 * then fills up to `max` records (kernel name, launches, total milliseconds) and returns the
 * number of distinct kernels through n_out.  Names are static strings.  There is one collector
 * per process, shared by all tables; library calls from several threads may record into it at
 * the same time, and enable / read may be called from any thread.  It is meant for benchmarks:
 * while it is on every launch costs two event records. */
typedef struct { const char *name; int64_t launches; double total_ms; } des_kernel_time_t;
des_status_t des_profile_enable(int32_t enable);
des_status_t des_profile_read(des_kernel_time_t *host_out, int32_t max, int32_t *n_out);

const char *des_status_string(des_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* DES_H_ */
