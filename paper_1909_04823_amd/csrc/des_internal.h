// Internal declarations shared by the translation units of libdes (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "des.h"

namespace des {

constexpr uint64_t kEmptyKey = 0xFFFFFFFFFFFFFFFFull;
constexpr int32_t kRowAbsent = -1;    // key not in the table
constexpr int32_t kRowPending = -2;   // claimed during the running call, row not assigned yet
constexpr int kWave = 64;
constexpr int kBlock = 256;

// One hash slot: key and row side by side so a probe is one 16-byte access.
struct __attribute__((aligned(16))) Slot {
  uint64_t key;
  int32_t row;        // -1 until the key's row is known
  uint32_t first;     // smallest entry index of the call that claimed the key (meaningful while row < 0)
};

// Device-resident control block at the head of the workspace.
struct Ctrl {
  long long n_rows;        // rows in use
  long long n_new;         // distinct unseen keys claimed by the running insert/find call
  long long n_uniq;        // distinct rows of the running backward call
  long long n_long;        // segments longer than the short-segment limit
  long long n_chunks;      // chunks those long segments were cut into
  int status;              // sticky des_status_t (table full): inserts stop until it is cleared
  int bad_keys;            // reserved keys seen since the status was last cleared (reported, not blocking)
  int pad[4];
  unsigned long long first_bad;   // verdict word of des_batch_validate
  long long n_multi;       // long segments of more than one chunk
  long long n_groups;      // groups of chunk partials that are pre-summed for the segments of very many chunks
};
static_assert(sizeof(Ctrl) <= 256, "control block must fit its reserved 256 bytes");

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- per-kernel timing (process-wide collector) ----------------------------------------
enum KernelId {
  KID_PROBE = 0, KID_ASSIGN, KID_PATCH, KID_INIT_ROWS,
  KID_FORWARD, KID_POOL_DENSE, KID_AGGREGATE, KID_FM_FINALIZE,
  KID_EXPAND, KID_SORT_HIST, KID_SORT_SCAN, KID_SORT_SCATTER,
  KID_HEADS, KID_CLASSIFY, KID_SHORT_UPDATE, KID_LONG_PARTIAL, KID_LONG_FINAL, KID_EXPORT,
  KID_FILL, KID_DNN_FORWARD, KID_DNN_GPOOL, KID_DNN_DW,
  KID_AGG_BIAS_ACT, KID_COLUMN_PARTIALS, KID_COLUMN_FINAL, KID_HEAD, KID_DENSE_UPDATE, KID_MIGRATE,
  KID_CROSS_PARTIAL, KID_CROSS_APPLY, KID_CROSS_GRAD, KID_CEILING_GATHER, KID_CEILING_UPDATE, KID_COUNT
};
void prof_begin(int kid, hipStream_t s);
void prof_end(int kid, hipStream_t s);
struct ProfScope {
  int kid; hipStream_t s;
  ProfScope(int k, hipStream_t st) : kid(k), s(st) { prof_begin(kid, s); }
  ~ProfScope() { prof_end(kid, s); }
};

// ---- device-wide primitives (des_sort.hip) ---------------------------------------------
// Scratch sizes in bytes for the primitives below.
size_t scan_scratch_bytes(int64_t n);
size_t sort_scratch_bytes(int64_t n);

// Exclusive prefix sum of 32-bit values in place; total written to *total_out (device, may be null).
void exclusive_scan_u32(uint32_t *data, int64_t n, uint32_t *total_out, void *scratch, hipStream_t s);
// Exclusive prefix sum of 64-bit values in place; total written to *total_out (device, may be null).
void exclusive_scan_u64(unsigned long long *data, int64_t n, unsigned long long *total_out,
                        void *scratch, hipStream_t s);

// Stable LSD radix sort of (32-bit key, 32-bit payload) pairs on the low `bits` bits of the key.
// Returns 0 if the sorted data is in the *_a buffers, 1 if in *_b.
struct SortBuffers { void *keys_a, *keys_b; uint32_t *pay_a, *pay_b; };
int radix_sort_u32_pairs(SortBuffers buf, int64_t n, int bits, void *scratch, hipStream_t s);

}  // namespace des

// Host handle.
struct des_table {
  des_table_config_t cfg;
  uint64_t n_slots;          // power of two
  des::Slot *slots;
  des::Ctrl *ctrl;           // in workspace
  char *ws;                  // workspace after the control block
  size_t ws_bytes;
  int64_t max_n;             // largest n the workspace was sized for (derived)
  float init_width;          // (float)(2*sqrt(3)*init_scale)
  hipStream_t last_stream;
  // Row-sorted form of a batch left in the workspace by des_backward_prepare: which batch it was
  // built for and which sort buffer holds the result.  Any call that reuses the workspace clears it.
  struct {
    bool valid;
    const int32_t *offsets, *rows;
    const float *vals;
    int64_t nnz, B;
    int F, side;
  } prep;
};

namespace des {
des_status_t forward_launch(des_table *t, const des_batch_t *b, const int32_t *rows, float *P_lr, float *P_sum,
                            float *P_sq, float *pool, hipStream_t s);
des_status_t pool_dense_launch(des_table *t, const des_batch_t *b, const int32_t *rows, float *P_pool, hipStream_t s);
des_status_t backward_launch(des_table *t, const des_batch_t *b, const int32_t *rows, const des_backward_io_t *io,
                             const des_optimizer_t *opt, hipStream_t s);
des_status_t backward_prepare_launch(des_table *t, const des_batch_t *b, const int32_t *rows, hipStream_t s);
size_t backward_ws_bytes(int D, int64_t max_n);
// The sticky status alone (table full, HIP error): what stops a table from growing or being reorganised.  Reserved keys
// that were passed are reported by des_table_status but block nothing.  Synchronises like des_table_status.
des_status_t blocking_status(des_table *t);
size_t insert_ws_bytes(int64_t max_n);
}  // namespace des
