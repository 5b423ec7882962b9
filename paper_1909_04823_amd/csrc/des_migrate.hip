// Growth and eviction of a table (Section 1, "Dynamic Features": the parameter set of a streaming
// recommender changes and grows over time; Section 5: dynamic hash table).  The paper states the
// requirement, not a mechanism.  Here the rows to keep move, in ascending row order, into a second,
// empty table of any capacity that holds them, and that table's hash slots are built from the moved
// keys: flags -> exclusive prefix sum (new row numbers) -> coalesced row copy -> parallel re-insert.
// A maintenance operation, not part of the training step: it synchronises with the host twice to
// size its launches and to refuse a target that is too small before anything is written.
//
// des_table_compact is the same eviction inside one table, for tables too large for a second copy: the kept
// rows close up towards row 0.  A kept row never moves up, so the arrays are walked in ascending chunks of
// rows: the kept rows of a chunk are gathered into a staging buffer and then stored at their new place, which
// lies at or below the chunk and holds only rows that have already been moved or dropped.
#include "des_internal.h"

namespace des {
namespace {

inline unsigned blocks_for(int64_t n, int64_t cap = 1 << 20) {
  int64_t g = (n + kBlock - 1) / kBlock;
  return (unsigned)(g < 1 ? 1 : (g > cap ? cap : g));
}

__global__ __launch_bounds__(kBlock) void k_keep_flags(const uint8_t *__restrict__ keep, int64_t n,
                                                        unsigned long long *__restrict__ flags) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += stride)
    flags[r] = (!keep || keep[r]) ? 1ull : 0ull;
}

struct MoveArgs {
  const uint64_t *src_keys; uint64_t *dst_keys;
  const float *src_vec[3]; float *dst_vec[3];     // emb, acc_emb, acc2_emb  ([rows, D])
  const float *src_sc[3]; float *dst_sc[3];       // w, acc_w, acc2_w        ([rows])
  const uint32_t *src_aux; uint32_t *dst_aux;     // optional caller array, one word per row
  const uint8_t *keep;
  const unsigned long long *new_row;              // exclusive prefix sum of the keep flags
  int64_t n;
  int D;
};

// One lane group of D/4 lanes per source row: 16-byte loads and stores of the three vector arrays,
// lane 0 of the group moves the key, the scalars and the caller's word.  A state array that only the
// target has is zeroed for the moved rows; one that only the source has is dropped.
__global__ __launch_bounds__(kBlock) void k_move_rows(const MoveArgs a) {
  const int G = a.D / 4;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t r = gid / G;
  const int sub = (int)(gid % G);
  if (r >= a.n) return;
  if (a.keep && !a.keep[r]) return;
  const int64_t d = (int64_t)a.new_row[r];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    if (!a.dst_vec[i]) continue;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (a.src_vec[i]) v = *reinterpret_cast<const float4 *>(a.src_vec[i] + r * a.D + sub * 4);
    *reinterpret_cast<float4 *>(a.dst_vec[i] + d * a.D + sub * 4) = v;
  }
  if (sub == 0) {
    a.dst_keys[d] = a.src_keys[r];
#pragma unroll
    for (int i = 0; i < 3; ++i)
      if (a.dst_sc[i]) a.dst_sc[i][d] = a.src_sc[i] ? a.src_sc[i][r] : 0.f;
    if (a.dst_aux) a.dst_aux[d] = a.src_aux ? a.src_aux[r] : 0u;
  }
}

// Re-insert: row d's key claims the first empty slot of its probe sequence.  All keys are distinct,
// so a claimed slot is never claimed twice; the row is stored after the claim (nothing reads the
// slots until the stream has drained this kernel).
__global__ __launch_bounds__(kBlock) void k_rehash(Slot *__restrict__ slots, uint64_t slot_mask,
                                                    const uint64_t *__restrict__ row_keys, int64_t n,
                                                    Ctrl *__restrict__ ctrl) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; d < n; d += stride) {
    const uint64_t key = row_keys[d];
    uint64_t idx = mix64(key) & slot_mask;
    bool placed = false;
    for (uint64_t probe = 0; probe <= slot_mask; ++probe) {
      const unsigned long long old =
          atomicCAS(reinterpret_cast<unsigned long long *>(&slots[idx].key), kEmptyKey, key);
      if (old == kEmptyKey) {
        slots[idx].row = (int32_t)d;
        placed = true;
        break;
      }
      idx = (idx + 1) & slot_mask;
    }
    if (!placed) atomicCAS(&ctrl->status, 0, (int)DES_ERR_FULL);
  }
}

__global__ void k_set_rows(Ctrl *ctrl, long long n) { ctrl->n_rows = n; }

// In-place compaction of one per-row array of `upr` units of type T per row, rows [c0, c1).
// new_row: exclusive prefix sum of the keep flags over all n rows, new_row[n] = number of kept rows.
template <typename T>
__global__ __launch_bounds__(kBlock) void k_compact_gather(const T *__restrict__ arr, int upr,
                                                            const uint8_t *__restrict__ keep,
                                                            const unsigned long long *__restrict__ new_row, int64_t c0,
                                                            int64_t c1, T *__restrict__ staging) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t r = c0 + gid / upr;
  const int u = (int)(gid % upr);
  if (r >= c1 || !keep[r]) return;
  staging[(int64_t)(new_row[r] - new_row[c0]) * upr + u] = arr[r * upr + u];
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_compact_store(T *__restrict__ arr, int upr,
                                                           const unsigned long long *__restrict__ new_row, int64_t c0,
                                                           int64_t c1, const T *__restrict__ staging) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t i = gid / upr;
  const int u = (int)(gid % upr);
  const int64_t first = (int64_t)new_row[c0], kept = (int64_t)new_row[c1] - first;
  if (i >= kept) return;
  arr[(first + i) * upr + u] = staging[i * upr + u];
}

__global__ void k_take_rows(Ctrl *ctrl, const unsigned long long *total) { ctrl->n_rows = (long long)*total; }

__global__ void k_fill_words(uint32_t *p, int64_t n, uint32_t v) {
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) p[i] = v;
}

// empty slot = all-ones key, row -1: one 16-byte pattern of 0xFF
__global__ __launch_bounds__(kBlock) void k_fill_slots(uint4 *__restrict__ p, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const uint4 ones = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = ones;
}

template <typename T>
void compact_array(T *arr, int upr, const uint8_t *keep, const unsigned long long *new_row, int64_t n, void *staging,
                   size_t staging_bytes, hipStream_t s) {
  if (!arr) return;
  const int64_t chunk = (int64_t)(staging_bytes / ((size_t)upr * sizeof(T)));
  for (int64_t c0 = 0; c0 < n; c0 += chunk) {
    const int64_t c1 = c0 + chunk < n ? c0 + chunk : n;
    const unsigned grid = (unsigned)(((c1 - c0) * upr + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(k_compact_gather<T>, dim3(grid), dim3(kBlock), 0, s, (const T *)arr, upr, keep, new_row, c0, c1,
                       (T *)staging);
    hipLaunchKernelGGL(k_compact_store<T>, dim3(grid), dim3(kBlock), 0, s, arr, upr, new_row, c0, c1, (const T *)staging);
  }
}

__global__ __launch_bounds__(kBlock) void k_mark_seen(const int32_t *__restrict__ rows, int64_t n, uint32_t stamp,
                                                       uint32_t *__restrict__ last_seen) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) {
    const int32_t r = rows[e];
    if (r >= 0) last_seen[r] = stamp;               // entries of one row all store the same value
  }
}

__global__ __launch_bounds__(kBlock) void k_select_recent(const uint32_t *__restrict__ last_seen, int64_t n,
                                                           uint32_t min_stamp, uint8_t *__restrict__ keep) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += stride)
    keep[r] = last_seen[r] >= min_stamp ? 1 : 0;
}

// Smallest index whose value breaks the batch contract (see des_batch_validate); kept with an atomic minimum.
__global__ __launch_bounds__(kBlock) void k_validate(const int32_t *__restrict__ offsets, int64_t nbags, int64_t nnz,
                                                      const int32_t *__restrict__ rows, const Ctrl *__restrict__ ctrl,
                                                      unsigned long long *__restrict__ first_bad) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t total = nbags + 1 + (rows ? nnz : 0);
  const long long n_rows = ctrl->n_rows;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    bool bad;
    if (i <= nbags) {
      const int32_t o = offsets[i];
      bad = (i == 0 && o != 0) || (i == nbags && (int64_t)o != nnz) || (i > 0 && o < offsets[i - 1]) || o < 0 ||
            (int64_t)o > nnz;
    } else {
      const int32_t r = rows[i - nbags - 1];
      bad = r < -1 || (long long)r >= n_rows;
    }
    if (bad) atomicMin(first_bad, (unsigned long long)i);
  }
}

bool overlap(const void *a, size_t na, const void *b, size_t nb) {
  if (!a || !b) return false;
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

}  // namespace
}  // namespace des

using namespace des;

extern "C" {

des_status_t des_table_migrate_bytes(int64_t n_rows, size_t *workspace_bytes) {
  if (!workspace_bytes || n_rows < 0) return DES_ERR_INVALID_ARG;
  *workspace_bytes = 256 + align_up((size_t)(n_rows > 0 ? n_rows : 1) * 8, 256) + scan_scratch_bytes(n_rows > 0 ? n_rows : 1);
  return DES_OK;
}

des_status_t des_table_migrate(des_table_t *src, const uint8_t *keep, des_table_t *dst, const uint32_t *src_aux,
                               uint32_t *dst_aux, int64_t *n_rows_out, void *stream) {
  if (!src || !dst || src == dst) return DES_ERR_INVALID_ARG;
  const des_table_config_t &sc = src->cfg, &dc = dst->cfg;
  if (sc.dim != dc.dim || ((uintptr_t)src_aux & 3u) || ((uintptr_t)dst_aux & 3u)) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  int64_t n = 0, n_dst = 0;
  des_status_t st = des_table_size(src, &n);
  if (st != DES_OK) return st;
  st = des_table_size(dst, &n_dst);
  if (st != DES_OK) return st;
  if (n_dst != 0 || blocking_status(dst) != DES_OK || blocking_status(src) != DES_OK) return DES_ERR_INVALID_ARG;
  const size_t row_bytes = (size_t)sc.dim * 4;
  if (overlap(sc.emb, (size_t)sc.capacity_rows * row_bytes, dc.emb, (size_t)dc.capacity_rows * row_bytes) ||
      overlap(sc.row_keys, (size_t)sc.capacity_rows * 8, dc.row_keys, (size_t)dc.capacity_rows * 8) ||
      overlap(sc.w, (size_t)sc.capacity_rows * 4, dc.w, (size_t)dc.capacity_rows * 4) ||
      overlap(sc.slots, sc.slots_bytes, dc.slots, dc.slots_bytes))
    return DES_ERR_INVALID_ARG;
  if (n_rows_out) *n_rows_out = 0;
  src->last_stream = s;
  dst->last_stream = s;
  dst->prep.valid = false;
  if (n == 0) return DES_OK;
  size_t need = 0;
  (void)des_table_migrate_bytes(n, &need);
  if (dst->ws_bytes + 256 < need) return DES_ERR_WORKSPACE;
  unsigned long long *flags = (unsigned long long *)dst->ws;
  void *scan_scratch = dst->ws + align_up((size_t)n * 8, 256);
  ProfScope ps(KID_MIGRATE, s);
  hipLaunchKernelGGL(k_keep_flags, dim3(blocks_for(n)), dim3(kBlock), 0, s, keep, n, flags);
  // the total lands in the target's row counter, which is exactly what it is
  exclusive_scan_u64(flags, n, (unsigned long long *)&dst->ctrl->n_rows, scan_scratch, s);
  long long kept = 0;
  if (hipMemcpyAsync(&kept, &dst->ctrl->n_rows, sizeof(kept), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return DES_ERR_DEVICE;
  if (kept > dc.capacity_rows) {                       // refuse before anything is moved
    hipLaunchKernelGGL(k_set_rows, dim3(1), dim3(1), 0, s, dst->ctrl, 0ll);
    (void)hipStreamSynchronize(s);
    return DES_ERR_FULL;
  }
  MoveArgs a;
  a.src_keys = sc.row_keys; a.dst_keys = dc.row_keys;
  a.src_vec[0] = sc.emb; a.src_vec[1] = sc.acc_emb; a.src_vec[2] = sc.acc2_emb;
  a.dst_vec[0] = dc.emb; a.dst_vec[1] = dc.acc_emb; a.dst_vec[2] = dc.acc2_emb;
  a.src_sc[0] = sc.w; a.src_sc[1] = sc.acc_w; a.src_sc[2] = sc.acc2_w;
  a.dst_sc[0] = dc.w; a.dst_sc[1] = dc.acc_w; a.dst_sc[2] = dc.acc2_w;
  a.src_aux = src_aux; a.dst_aux = dst_aux;
  a.keep = keep; a.new_row = flags; a.n = n; a.D = sc.dim;
  const int64_t threads = n * (sc.dim / 4);
  hipLaunchKernelGGL(k_move_rows, dim3((unsigned)((threads + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, a);
  if (kept > 0)
    hipLaunchKernelGGL(k_rehash, dim3(blocks_for(kept, 1 << 16)), dim3(kBlock), 0, s, dst->slots, dst->n_slots - 1,
                       (const uint64_t *)dc.row_keys, (int64_t)kept, dst->ctrl);
  if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return DES_ERR_DEVICE;
  if (n_rows_out) *n_rows_out = kept;
  return blocking_status(dst);
}

des_status_t des_table_compact(des_table_t *t, const uint8_t *keep, uint32_t *aux, void *staging, size_t staging_bytes,
                               int64_t *n_rows_out, void *stream) {
  if (!t || ((uintptr_t)aux & 3u)) return DES_ERR_INVALID_ARG;
  const des_table_config_t &c = t->cfg;
  hipStream_t s = (hipStream_t)stream;
  int64_t n = 0;
  des_status_t st = des_table_size(t, &n);
  if (st != DES_OK) return st;
  if (blocking_status(t) != DES_OK) return DES_ERR_INVALID_ARG;
  if (n_rows_out) *n_rows_out = n;
  t->last_stream = s;
  t->prep.valid = false;
  if (n == 0 || !keep) return DES_OK;                       // nothing to drop
  // the staging buffer holds at least 4096 rows of the widest array at a time
  if (!staging || ((uintptr_t)staging & 15u) || staging_bytes < (size_t)4096 * (size_t)c.dim * 4) return DES_ERR_WORKSPACE;
  const size_t flags_bytes = align_up((size_t)(n + 1) * 8, 256);
  if (t->ws_bytes < flags_bytes + scan_scratch_bytes(n + 1)) return DES_ERR_WORKSPACE;
  unsigned long long *flags = (unsigned long long *)t->ws;
  void *scan_scratch = t->ws + flags_bytes;
  ProfScope ps(KID_MIGRATE, s);
  // n + 1 values with a zero at the end: after the scan flags[n] is the number of kept rows
  hipLaunchKernelGGL(k_keep_flags, dim3(blocks_for(n)), dim3(kBlock), 0, s, keep, n, flags);
  hipLaunchKernelGGL(k_fill_words, dim3(1), dim3(kWave), 0, s, (uint32_t *)(flags + n), (int64_t)2, 0u);
  exclusive_scan_u64(flags, n + 1, nullptr, scan_scratch, s);
  compact_array<float4>((float4 *)c.emb, c.dim / 4, keep, flags, n, staging, staging_bytes, s);
  compact_array<float4>((float4 *)c.acc_emb, c.dim / 4, keep, flags, n, staging, staging_bytes, s);
  compact_array<float4>((float4 *)c.acc2_emb, c.dim / 4, keep, flags, n, staging, staging_bytes, s);
  compact_array<uint32_t>((uint32_t *)c.w, 1, keep, flags, n, staging, staging_bytes, s);
  compact_array<uint32_t>((uint32_t *)c.acc_w, 1, keep, flags, n, staging, staging_bytes, s);
  compact_array<uint32_t>((uint32_t *)c.acc2_w, 1, keep, flags, n, staging, staging_bytes, s);
  compact_array<uint32_t>(aux, 1, keep, flags, n, staging, staging_bytes, s);
  compact_array<unsigned long long>((unsigned long long *)c.row_keys, 1, keep, flags, n, staging, staging_bytes, s);
  hipLaunchKernelGGL(k_take_rows, dim3(1), dim3(1), 0, s, t->ctrl, (const unsigned long long *)(flags + n));
  long long kept = 0;
  if (hipMemcpyAsync(&kept, flags + n, sizeof(kept), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return DES_ERR_DEVICE;
  // the slots are rebuilt from the kept keys
  hipLaunchKernelGGL(k_fill_slots, dim3(blocks_for((int64_t)t->n_slots, 1 << 16)), dim3(kBlock), 0, s, (uint4 *)t->slots,
                     (int64_t)t->n_slots);
  if (kept > 0)
    hipLaunchKernelGGL(k_rehash, dim3(blocks_for(kept, 1 << 16)), dim3(kBlock), 0, s, t->slots, t->n_slots - 1,
                       (const uint64_t *)c.row_keys, (int64_t)kept, t->ctrl);
  if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return DES_ERR_DEVICE;
  if (n_rows_out) *n_rows_out = kept;
  return blocking_status(t);
}

des_status_t des_batch_validate(des_table_t *t, const des_batch_t *batch, const int32_t *rows, int64_t *first_bad,
                                void *stream) {
  if (!t || !batch || batch->B < 0 || batch->F < 1 || batch->nnz < 0 || batch->nnz >= 2147483647ll ||
      batch->B * (int64_t)batch->F >= 2147483647ll || !batch->offsets || ((uintptr_t)batch->offsets & 3u) ||
      ((uintptr_t)rows & 3u))
    return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  unsigned long long *word = &t->ctrl->first_bad;
  const unsigned long long none = ~0ull;
  unsigned long long got = none;
  const int64_t nbags = batch->B * (int64_t)batch->F, total = nbags + 1 + (rows ? batch->nnz : 0);
  if (hipMemcpyAsync(word, &none, sizeof(none), hipMemcpyHostToDevice, s) != hipSuccess) return DES_ERR_DEVICE;
  hipLaunchKernelGGL(k_validate, dim3(blocks_for(total, 1 << 16)), dim3(kBlock), 0, s, batch->offsets, nbags, batch->nnz,
                     rows, t->ctrl, word);
  if (hipMemcpyAsync(&got, word, sizeof(got), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess || hipGetLastError() != hipSuccess)
    return DES_ERR_DEVICE;
  if (first_bad) *first_bad = got == none ? -1 : (int64_t)got;
  return got == none ? DES_OK : DES_ERR_INVALID_ARG;
}

des_status_t des_table_mark_seen(const int32_t *rows, int64_t n, uint32_t stamp, uint32_t *last_seen, void *stream) {
  if (n < 0 || (n > 0 && (!rows || !last_seen)) || ((uintptr_t)rows & 3u) || ((uintptr_t)last_seen & 3u))
    return DES_ERR_INVALID_ARG;
  if (n == 0) return DES_OK;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_MIGRATE, s);
  hipLaunchKernelGGL(k_mark_seen, dim3(blocks_for(n)), dim3(kBlock), 0, s, rows, n, stamp, last_seen);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_table_select_recent(const uint32_t *last_seen, int64_t n_rows, uint32_t min_stamp, uint8_t *keep,
                                     void *stream) {
  if (n_rows < 0 || (n_rows > 0 && (!last_seen || !keep)) || ((uintptr_t)last_seen & 3u)) return DES_ERR_INVALID_ARG;
  if (n_rows == 0) return DES_OK;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_MIGRATE, s);
  hipLaunchKernelGGL(k_select_recent, dim3(blocks_for(n_rows)), dim3(kBlock), 0, s, last_seen, n_rows, min_stamp, keep);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // extern "C"
