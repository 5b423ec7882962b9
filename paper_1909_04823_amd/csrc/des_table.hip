// Dynamic hash table (Section 5, "Dynamic Hash Table"): open addressing with linear probing
// over 16-byte slots, 64-bit keys claimed with a compare-and-swap, plus the C entry points
// that do not belong to the forward or backward files.
//
// Row numbers must not depend on which thread wins a slot: they are those of a sequential
// insert loop (unseen distinct keys numbered in order of first occurrence).  An insert is
// therefore split in two: claiming a slot (racy, unobservable), during which every entry of a
// new key lowers the slot's "first occurrence" index with an atomic minimum, and numbering:
// the entries that ARE the first occurrence of a new key are counted with a prefix sum in
// entry order, row = n_rows + prefix.
#include <math.h>
#include <stddef.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <new>
#include <vector>
#include "des_internal.h"

using namespace des;

namespace {

constexpr int kFlagItems = 8;                       // entries per thread in the numbering kernels
constexpr int kFlagTile = kBlock * kFlagItems;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int64_t kSelfPrefixTiles = 4096;          // up to this many tiles the numbering kernel sums the tile counts itself

__device__ inline void set_status(Ctrl *c, int st) { atomicCAS(&c->status, 0, st); }

__device__ inline Slot load_slot(const Slot *p) {
  const uint4 raw = *reinterpret_cast<const uint4 *>(p);
  Slot s;
  s.key = ((uint64_t)raw.y << 32) | raw.x;
  s.row = (int32_t)raw.z;
  s.first = raw.w;
  return s;
}

// Pass A.  rows[e] = row (>= 0), kRowAbsent, or kRowPending for keys claimed in this call; for
// pending entries slot_of[e] remembers the slot so later passes need not probe again.
// A probe is one dependent chain (key -> hash -> slot), so every thread works on kProbeKeys keys at a time: all their
// keys are requested, then all their first slots, and only then is each chain resolved (later slots of a collision
// chain one by one; they mostly sit in the line already fetched).  That multiplies the random lines in flight.
constexpr int kProbeKeys = 4;
template <bool kInsert>
__global__ __launch_bounds__(kBlock) void k_probe(Slot *__restrict__ slots, uint64_t slot_mask,
                                                   const uint64_t *__restrict__ keys, int64_t n,
                                                   int32_t *__restrict__ rows, Ctrl *__restrict__ ctrl,
                                                   uint32_t *__restrict__ slot_of) {
  // after a sticky error the table no longer grows: the call degrades to a pure lookup, so
  // rows[] is still fully written with valid rows or kRowAbsent
  const bool can_insert = kInsert && ctrl->status == 0;
  const int64_t tile_stride = (int64_t)gridDim.x * kBlock * kProbeKeys;
  for (int64_t tile = (int64_t)blockIdx.x * kBlock * kProbeKeys; tile < n; tile += tile_stride) {
    uint64_t key[kProbeKeys], idx[kProbeKeys];
    Slot first[kProbeKeys];
#pragma unroll
    for (int i = 0; i < kProbeKeys; ++i) {
      const int64_t e = tile + (int64_t)i * kBlock + threadIdx.x;
      key[i] = e < n ? keys[e] : kEmptyKey;
    }
#pragma unroll
    for (int i = 0; i < kProbeKeys; ++i) {
      idx[i] = mix64(key[i]) & slot_mask;
      first[i].key = kEmptyKey; first[i].row = kRowAbsent; first[i].first = 0u;
      if (key[i] != kEmptyKey) first[i] = load_slot(&slots[idx[i]]);
    }
#pragma unroll
    for (int i = 0; i < kProbeKeys; ++i) {
      const int64_t e = tile + (int64_t)i * kBlock + threadIdx.x;
      if (e >= n) continue;
      int32_t out = kRowAbsent;
      if (key[i] == kEmptyKey) {                     // the reserved key is nobody's ID: absent, counted, nothing else is held up
        atomicAdd(&ctrl->bad_keys, 1);
        rows[e] = out;
        continue;
      }
      const uint64_t k = key[i];
      uint64_t at = idx[i];
      Slot s = first[i];
      bool done = false, pending = false;
      for (uint64_t probe = 0; probe <= slot_mask && !done; ++probe) {
        if (probe > 0) s = load_slot(&slots[at]);
        if (s.key == k) {
          // a negative row under a key is a claim of the running call, or the leftover of a
          // call that failed: only a call that can insert resolves it
          if (s.row >= 0) out = s.row; else pending = can_insert;
          done = true;
        } else if (s.key == kEmptyKey) {
          if (!can_insert) {
            done = true;
          } else {
            const unsigned long long old =
                atomicCAS(reinterpret_cast<unsigned long long *>(&slots[at].key), kEmptyKey, k);
            if (old == kEmptyKey || old == k) {   // claimed here, or by another entry of the same key
              pending = true;
              done = true;
            } else {
              at = (at + 1) & slot_mask;          // lost the slot to a different key
            }
          }
        } else {
          at = (at + 1) & slot_mask;
        }
      }
      if (!done) set_status(ctrl, DES_ERR_FULL);     // every slot visited
      if (pending) {
        atomicMin(&slots[at].first, (uint32_t)e);
        slot_of[e] = (uint32_t)at;
        out = kRowPending;
      }
      rows[e] = out;
    }
  }
}

__device__ inline uint32_t wave_incl_scan_u32(uint32_t v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  return v;
}

__device__ inline uint32_t block_excl_scan_u32(uint32_t v, uint32_t *lds, uint32_t &total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t inc = wave_incl_scan_u32(v);
  if (lane == kWave - 1) lds[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) {
    const uint32_t x = lds[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + inc - v;
}

// entry e opens a new row iff it is pending and is the first occurrence recorded in its slot
__device__ inline bool opens_row(const Slot *slots, int32_t row_e, const uint32_t *slot_of, int64_t e) {
  return row_e == kRowPending && slots[slot_of[e]].first == (uint32_t)e;
}

// rows[] of the thread's kFlagItems consecutive entries (16-byte loads when they all exist and the caller's array
// is 16-byte aligned; it only has to be 4-byte aligned); entries past n read as absent
__device__ inline void load_flag_rows(const int32_t *__restrict__ rows, int64_t base, int64_t n, int32_t (&r)[kFlagItems]) {
  static_assert(kFlagItems % 4 == 0, "whole int4 loads");
  if (base + kFlagItems <= n && ((uintptr_t)rows & 15u) == 0) {
#pragma unroll
    for (int q = 0; q < kFlagItems / 4; ++q) {
      const int4 v = *reinterpret_cast<const int4 *>(rows + base + q * 4);
      r[q * 4 + 0] = v.x; r[q * 4 + 1] = v.y; r[q * 4 + 2] = v.z; r[q * 4 + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kFlagItems; ++i) r[i] = base + i < n ? rows[base + i] : kRowAbsent;
  }
}

// Pass B1: per tile, how many entries open a new row.
__global__ __launch_bounds__(kBlock) void k_new_count(const Slot *__restrict__ slots, const int32_t *__restrict__ rows,
                                                       const uint32_t *__restrict__ slot_of, int64_t n,
                                                       uint32_t *__restrict__ tile_sums) {
  __shared__ uint32_t lds[kWavesPerBlock];
  const int64_t base = (int64_t)blockIdx.x * kFlagTile + (int64_t)threadIdx.x * kFlagItems;
  uint32_t cnt = 0;
  int32_t r[kFlagItems];
  load_flag_rows(rows, base, n, r);
#pragma unroll
  for (int i = 0; i < kFlagItems; ++i)
    if (base + i < n && opens_row(slots, r[i], slot_of, base + i)) ++cnt;
  uint32_t total;
  block_excl_scan_u32(cnt, lds, total);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// Pass B2: one workgroup turns the tile counts into tile offsets, publishes the number of new
// rows and checks the capacity.
__global__ __launch_bounds__(kBlock) void k_new_sums(uint32_t *__restrict__ tile_sums, int64_t nb,
                                                      Ctrl *__restrict__ ctrl, int64_t capacity) {
  __shared__ uint32_t lds[kWavesPerBlock];
  uint32_t carry = 0;
  for (int64_t base = 0; base < nb; base += kBlock) {
    const int64_t i = base + threadIdx.x;
    const uint32_t v = i < nb ? tile_sums[i] : 0u;
    uint32_t total;
    const uint32_t ex = block_excl_scan_u32(v, lds, total);
    if (i < nb) tile_sums[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    ctrl->n_new = carry;
    if (ctrl->n_rows + (long long)carry > capacity) set_status(ctrl, DES_ERR_FULL);
  }
}

// Pass B3: number the new rows in entry order; the slot learns its row.
// kSelfPrefix: tile_sums still holds the tiles' counts; every workgroup adds up all of them itself (few tiles:
// cheaper than a launch that does it once), which gives it the rows before its tile, the number of new rows and the
// capacity verdict, the same in every workgroup.  The first workgroup publishes the latter two.
template <bool kSelfPrefix>
__global__ __launch_bounds__(kBlock) void k_new_assign(Slot *__restrict__ slots, const int32_t *__restrict__ rows,
                                                        const uint32_t *__restrict__ slot_of,
                                                        const uint64_t *__restrict__ keys, int64_t n,
                                                        const uint32_t *__restrict__ tile_sums,
                                                        Ctrl *__restrict__ ctrl, uint64_t *__restrict__ row_keys,
                                                        int32_t *__restrict__ first_idx, int64_t capacity) {
  __shared__ uint32_t lds[kWavesPerBlock];
  uint32_t tile_base;
  if (kSelfPrefix) {
    uint32_t before = 0, rest = 0;
    for (uint32_t i = threadIdx.x; i < gridDim.x; i += kBlock) {
      const uint32_t v = tile_sums[i];
      if (i < blockIdx.x) before += v; else rest += v;
    }
    uint32_t rest_total;
    block_excl_scan_u32(before, lds, tile_base);
    block_excl_scan_u32(rest, lds, rest_total);
    const long long n_new = (long long)tile_base + rest_total;
    const bool full = ctrl->n_rows + n_new > capacity;            // n_rows does not change before the commit
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      ctrl->n_new = n_new;
      if (full) set_status(ctrl, DES_ERR_FULL);
    }
    if (full || ctrl->status != 0) return;            // uniform over the grid: a status set earlier, or by a peer just now
  } else {
    if (ctrl->status != 0) return;                    // uniform: includes "would exceed the capacity"
    tile_base = tile_sums[blockIdx.x];
  }
  const long long n_rows = ctrl->n_rows;
  const int64_t base = (int64_t)blockIdx.x * kFlagTile + (int64_t)threadIdx.x * kFlagItems;
  bool flag[kFlagItems];
  uint32_t cnt = 0;
  int32_t r[kFlagItems];
  load_flag_rows(rows, base, n, r);
#pragma unroll
  for (int i = 0; i < kFlagItems; ++i) {
    flag[i] = base + i < n && opens_row(slots, r[i], slot_of, base + i);
    cnt += flag[i] ? 1u : 0u;
  }
  uint32_t total;
  uint32_t rank = tile_base + block_excl_scan_u32(cnt, lds, total);
#pragma unroll
  for (int i = 0; i < kFlagItems; ++i) {
    if (flag[i]) {
      const int64_t e = base + i;
      const long long row = n_rows + rank;
      slots[slot_of[e]].row = (int32_t)row;
      row_keys[row] = keys[e];
      first_idx[rank] = (int32_t)e;
      ++rank;
    }
  }
}

// Rows created by this call get initialiser weights and zero optimizer state.
// One thread per group of four columns; the group with index D/4 holds the LR weight.
__global__ __launch_bounds__(kBlock) void k_init_rows(const Ctrl *__restrict__ ctrl, int D, uint64_t seed,
                                                       float width, const uint64_t *__restrict__ row_keys,
                                                       float *__restrict__ emb, float *__restrict__ w,
                                                       float *__restrict__ acc_emb, float *__restrict__ acc_w,
                                                       float *__restrict__ acc2_emb, float *__restrict__ acc2_w,
                                                       int64_t capacity) {
  if (ctrl->status != 0) return;
  const long long n_new = ctrl->n_new, n_rows = ctrl->n_rows;
  if (n_rows + n_new > capacity) return;
  const int groups = D / 4 + 1;
  const int64_t total = n_new * groups;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t row = n_rows + i / groups;
    const int g = (int)(i % groups);
    const uint64_t key = row_keys[row];
    if (g < D / 4) {
      float v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint64_t h = mix64(key ^ mix64(seed + (uint64_t)(g * 4 + k)));
        const float u = (float)(h >> 40) * (1.0f / 16777216.0f);
        v[k] = __fmul_rn(__fsub_rn(u, 0.5f), width);
      }
      *reinterpret_cast<float4 *>(&emb[row * D + g * 4]) = make_float4(v[0], v[1], v[2], v[3]);
      if (acc_emb) *reinterpret_cast<float4 *>(&acc_emb[row * D + g * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);
      if (acc2_emb) *reinterpret_cast<float4 *>(&acc2_emb[row * D + g * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
      const uint64_t h = mix64(key ^ mix64(seed + (uint64_t)D));
      const float u = (float)(h >> 40) * (1.0f / 16777216.0f);
      w[row] = __fmul_rn(__fsub_rn(u, 0.5f), width);
      if (acc_w) acc_w[row] = 0.f;
      if (acc2_w) acc2_w[row] = 0.f;
    }
  }
}

// Pass D.  Entries that saw a pending key read the row from the slot they remembered.
// It is also the last kernel of an insert, so its first thread makes the new rows part of the table (no kernel of
// the call reads the row count after this one was launched).
__global__ __launch_bounds__(kBlock) void k_patch(const Slot *__restrict__ slots, int64_t n,
                                                   int32_t *__restrict__ rows, const uint32_t *__restrict__ slot_of,
                                                   Ctrl *__restrict__ ctrl, int64_t capacity) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) {
    if (rows[e] != kRowPending) continue;
    const int32_t row = slots[slot_of[e]].row;
    rows[e] = row >= 0 ? row : kRowAbsent;         // negative only after a failed call
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (ctrl->status == 0 && ctrl->n_rows + ctrl->n_new <= capacity) ctrl->n_rows += ctrl->n_new;
    ctrl->n_new = 0;
  }
}

// Pass E (host values given): new row j copies the values of its first occurrence.
__global__ __launch_bounds__(kBlock) void k_copy_values(const Ctrl *__restrict__ ctrl, int D,
                                                         const float *__restrict__ values,
                                                         const int32_t *__restrict__ first_idx,
                                                         float *__restrict__ emb, float *__restrict__ w,
                                                         float *__restrict__ acc_emb, float *__restrict__ acc_w,
                                                         float *__restrict__ acc2_emb, float *__restrict__ acc2_w,
                                                         int64_t capacity) {
  if (ctrl->status != 0) return;
  const long long n_new = ctrl->n_new, n_rows = ctrl->n_rows;
  if (n_rows + n_new > capacity) return;
  const int cols = D + 1;
  const int64_t total = n_new * cols;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t j = i / cols;
    const int c = (int)(i % cols);
    const int64_t row = n_rows + j;
    const int32_t src = first_idx[j];
    const float val = values[(int64_t)src * cols + c];
    if (c < D) {
      emb[row * D + c] = val;
      if (acc_emb) acc_emb[row * D + c] = 0.f;
      if (acc2_emb) acc2_emb[row * D + c] = 0.f;
    } else {
      w[row] = val;
      if (acc_w) acc_w[row] = 0.f;
      if (acc2_w) acc2_w[row] = 0.f;
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_fill_u64x2(uint4 *__restrict__ p, int64_t n16, uint4 v) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = v;
}

__global__ void k_zero_ctrl(Ctrl *ctrl) {
  ctrl->n_rows = 0; ctrl->n_new = 0; ctrl->n_uniq = 0; ctrl->n_long = 0; ctrl->n_chunks = 0; ctrl->status = 0;
  ctrl->n_multi = 0; ctrl->n_groups = 0; ctrl->bad_keys = 0;
}

// des_table_clear_status: the status words start over, and the slots that a failed insert claimed without
// giving them a row forget that call's entry numbers, so that the next insert of their key numbers them afresh.
__global__ __launch_bounds__(kBlock) void k_clear_status(Slot *__restrict__ slots, uint64_t n_slots, Ctrl *ctrl) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < (int64_t)n_slots; i += stride) {
    const Slot s = load_slot(&slots[i]);
    if (s.key != kEmptyKey && s.row < 0 && s.first != 0xFFFFFFFFu) slots[i].first = 0xFFFFFFFFu;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { ctrl->status = 0; ctrl->bad_keys = 0; ctrl->n_new = 0; }
}

// Copy of the row -> key map for the rows in use (the count lives on the device).
__global__ __launch_bounds__(kBlock) void k_export_keys(const Ctrl *__restrict__ ctrl, const uint64_t *__restrict__ row_keys,
                                                         uint64_t *__restrict__ out, int64_t max_rows) {
  const int64_t n = min((int64_t)ctrl->n_rows, max_rows);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = row_keys[i];
}

// out[i] = sum over the K shards of P[s*n + i], summed in double and rounded once
template <bool kVec4>
__global__ __launch_bounds__(kBlock) void k_aggregate(const float *__restrict__ P, int K, int64_t n,
                                                       float *__restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  if (kVec4) {
    const int64_t n4 = n / 4;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
      double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll 8
      for (int s = 0; s < K; ++s) {
        const float4 p = *reinterpret_cast<const float4 *>(&P[(int64_t)s * n + i * 4]);
        a0 += (double)p.x; a1 += (double)p.y; a2 += (double)p.z; a3 += (double)p.w;
      }
      *reinterpret_cast<float4 *>(&out[i * 4]) = make_float4((float)a0, (float)a1, (float)a2, (float)a3);
    }
  } else {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
      double a = 0.0;
#pragma unroll 8
      for (int s = 0; s < K; ++s) a += (double)P[(int64_t)s * n + i];
      out[i] = (float)a;
    }
  }
}

// fm2[b] = (<A_sum[b], A_sum[b]> - A_sq[b]) / 2, the two reductions in double: the inner
// product is an order of magnitude larger than the result.  Eight lanes per sample.
__global__ __launch_bounds__(kBlock) void k_fm_finalize(const float *__restrict__ A_sum,
                                                         const float *__restrict__ A_sq, int64_t B, int D,
                                                         float *__restrict__ fm2) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t b = gid / 8;
  const int sub = (int)(gid % 8);
  double q = 0.0;
  if (b < B)
    for (int d = sub; d < D; d += 8) {
      const double a = (double)A_sum[b * D + d];
      q += a * a;
    }
  q += __shfl_xor(q, 1, 8);
  q += __shfl_xor(q, 2, 8);
  q += __shfl_xor(q, 4, 8);
  if (b < B && sub == 0) fm2[b] = (float)(0.5 * (q - (double)A_sq[b]));
}

// The three aggregations of one forward pass and the FM substitution operator in one launch: eight lanes
// per sample sum the K shards' partials of their columns in double, square the sums for fm2 before they
// are rounded, and lane 0 adds the two scalars.  Any of the LR and FM groups may be absent.
__global__ __launch_bounds__(kBlock) void k_aggregate_forward(const float *__restrict__ P_lr,
                                                               const float *__restrict__ P_sum,
                                                               const float *__restrict__ P_sq, int K, int64_t B, int D,
                                                               float *__restrict__ A_lr, float *__restrict__ A_sum,
                                                               float *__restrict__ A_sq, float *__restrict__ fm2) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t b = gid / 8;
  const int sub = (int)(gid % 8);
  double q = 0.0;
  if (b < B && P_sum)
    for (int d4 = sub; d4 < D / 4; d4 += 8) {
      double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll 8
      for (int s = 0; s < K; ++s) {                       // the shards' loads are independent: several in flight
        const float4 p = *reinterpret_cast<const float4 *>(P_sum + ((int64_t)s * B + b) * D + d4 * 4);
        a0 += (double)p.x; a1 += (double)p.y; a2 += (double)p.z; a3 += (double)p.w;
      }
      *reinterpret_cast<float4 *>(A_sum + b * D + d4 * 4) = make_float4((float)a0, (float)a1, (float)a2, (float)a3);
      q += a0 * a0 + a1 * a1 + a2 * a2 + a3 * a3;
    }
  q += __shfl_xor(q, 1, 8);
  q += __shfl_xor(q, 2, 8);
  q += __shfl_xor(q, 4, 8);
  if (b < B && sub == 0) {
    if (P_sum) {
      double sq = 0.0;
#pragma unroll 8
      for (int s = 0; s < K; ++s) sq += (double)P_sq[(int64_t)s * B + b];
      A_sq[b] = (float)sq;
      if (fm2) fm2[b] = (float)(0.5 * (q - sq));
    }
    if (P_lr) {
      double l = 0.0;
#pragma unroll 8
      for (int s = 0; s < K; ++s) l += (double)P_lr[(int64_t)s * B + b];
      A_lr[b] = (float)l;
    }
  }
}

inline unsigned grid_for(int64_t n, int per_block = kBlock, int64_t cap = 1 << 20) {
  int64_t g = (n + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (unsigned)g;
}

bool pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

des_status_t validate_cfg(const des_table_config_t *c) {
  if (!c) return DES_ERR_INVALID_ARG;
  if (c->dim < 4 || c->dim > 256 || !pow2(c->dim)) return DES_ERR_INVALID_ARG;
  if (c->capacity_rows < 1 || c->capacity_rows > 2147483646ll) return DES_ERR_INVALID_ARG;
  if (c->num_shards < 1 || c->num_shards > 256) return DES_ERR_INVALID_ARG;
  if (c->shard_policy != DES_SHARD_KEY_HASH && c->shard_policy != DES_SHARD_FIELD_MOD) return DES_ERR_INVALID_ARG;
  if (c->opt < DES_OPT_NONE || c->opt > DES_OPT_FTRL) return DES_ERR_INVALID_ARG;
  if (!(c->init_scale >= 0.f)) return DES_ERR_INVALID_ARG;
  return DES_OK;
}

uint64_t slots_for(int64_t capacity) {
  uint64_t want = (uint64_t)capacity + (uint64_t)capacity / 3 + 1;   // load factor <= 0.75
  uint64_t n = 1024;
  while (n < want) n <<= 1;
  return n;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

namespace des {

size_t insert_ws_bytes(int64_t n) {
  const size_t m = (size_t)(n > 0 ? n : 1);
  return align_up(m * 4, 256)                                   // rows when the caller passes none
         + align_up(m * 4, 256)                                 // slot of each pending entry
         + align_up(m * 4, 256)                                 // first-occurrence entry of each new row
         + align_up(((m + kFlagTile - 1) / kFlagTile + 1) * 4, 256);   // per-tile counts
}

// ---- profiler ------------------------------------------------------------------------------
namespace {
struct ProfRec { int kid; hipEvent_t a, b; };
// Collector shared by all tables and threads of the process: the switch is atomic, the record list is guarded by a
// mutex, and the event that opens a launch is kept per thread (a launch is opened and closed by the same call).
std::atomic<bool> g_prof_on{false};
std::mutex g_prof_mutex;
std::vector<ProfRec> g_prof;
thread_local hipEvent_t g_open[KID_COUNT];
const char *kKernelNames[KID_COUNT] = {
    "table_probe", "table_number_new_rows", "table_patch_rows", "table_init_rows",
    "forward_gather_pool", "forward_pool_dense", "aggregate_partials", "fm_finalize",
    "backward_expand", "sort_histogram", "sort_scan", "sort_scatter",
    "backward_segment_heads", "backward_classify", "backward_short_update", "backward_long_partial",
    "backward_long_final", "backward_export", "fill",
    "dnn_forward", "dnn_grad_pool", "dnn_grad_weights",
    "aggregate_bias_act", "column_partials", "column_final", "output_unit", "dense_update", "table_migrate",
    "cross_partial", "cross_apply", "cross_backward", "ceiling_gather", "ceiling_update"};
}  // namespace

des_status_t blocking_status(des_table *t) {
  int v = 0;
  if (hipStreamSynchronize(t->last_stream) != hipSuccess) return DES_ERR_DEVICE;
  if (hipMemcpy(&v, &t->ctrl->status, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return DES_ERR_DEVICE;
  return (des_status_t)v;
}

void prof_begin(int kid, hipStream_t s) {
  if (!g_prof_on.load(std::memory_order_relaxed)) return;
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return;
  (void)hipEventRecord(e, s);
  g_open[kid] = e;
}

void prof_end(int kid, hipStream_t s) {
  if (!g_open[kid]) return;
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return;
  (void)hipEventRecord(e, s);
  {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof.push_back({kid, g_open[kid], e});
  }
  g_open[kid] = nullptr;
}

}  // namespace des

extern "C" {

const char *des_status_string(des_status_t s) {
  switch (s) {
    case DES_OK: return "ok";
    case DES_ERR_INVALID_ARG: return "invalid argument";
    case DES_ERR_INVALID_KEY: return "reserved key passed (treated as absent)";
    case DES_ERR_FULL: return "table full";
    case DES_ERR_WORKSPACE: return "slots or workspace too small";
    case DES_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown";
}

des_status_t des_profile_enable(int32_t enable) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (auto &r : g_prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_prof.clear();
  g_prof_on.store(enable != 0);
  return DES_OK;
}

des_status_t des_profile_read(des_kernel_time_t *out, int32_t max, int32_t *n_out) {
  if (!out || !n_out || max < 0) return DES_ERR_INVALID_ARG;
  if (hipDeviceSynchronize() != hipSuccess) return DES_ERR_DEVICE;
  double ms[KID_COUNT] = {0};
  int64_t cnt[KID_COUNT] = {0};
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (auto &r : g_prof) {
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) { ms[r.kid] += t; cnt[r.kid]++; }
  }
  int k = 0;
  for (int i = 0; i < KID_COUNT && k < max; ++i)
    if (cnt[i]) { out[k].name = kKernelNames[i]; out[k].launches = cnt[i]; out[k].total_ms = ms[i]; ++k; }
  *n_out = k;
  return DES_OK;
}

des_status_t des_table_query_bytes(const des_table_config_t *cfg, int64_t max_n, size_t *slots_bytes,
                                   size_t *workspace_bytes) {
  des_status_t st = validate_cfg(cfg);
  if (st != DES_OK) return st;
  if (max_n < 0 || max_n >= 2147483647ll) return DES_ERR_INVALID_ARG;
  if (slots_bytes) *slots_bytes = (size_t)slots_for(cfg->capacity_rows) * sizeof(Slot);
  if (workspace_bytes) {
    const size_t a = insert_ws_bytes(max_n), b = backward_ws_bytes(cfg->dim, max_n);
    *workspace_bytes = 256 + (a > b ? a : b);
  }
  return DES_OK;
}

des_status_t des_table_create(const des_table_config_t *cfg, des_table_t **out) {
  if (!out) return DES_ERR_INVALID_ARG;
  *out = nullptr;
  des_status_t st = validate_cfg(cfg);
  if (st != DES_OK) return st;
  if (!cfg->emb || !cfg->w || !cfg->row_keys || !cfg->slots || !cfg->workspace) return DES_ERR_INVALID_ARG;
  if (cfg->opt == DES_OPT_ADAGRAD && (!cfg->acc_emb || !cfg->acc_w)) return DES_ERR_INVALID_ARG;
  if (cfg->opt == DES_OPT_ADAM && (!cfg->acc_emb || !cfg->acc_w || !cfg->acc2_emb || !cfg->acc2_w)) return DES_ERR_INVALID_ARG;
  if (cfg->opt == DES_OPT_FTRL && (!cfg->acc_w || !cfg->acc2_w)) return DES_ERR_INVALID_ARG;
  if ((cfg->acc2_emb && !aligned16(cfg->acc2_emb)) || ((uintptr_t)cfg->acc2_w & 3u)) return DES_ERR_INVALID_ARG;
  if (!aligned16(cfg->emb) || !aligned16(cfg->slots) || !aligned16(cfg->workspace) ||
      (cfg->acc_emb && !aligned16(cfg->acc_emb)) || ((uintptr_t)cfg->row_keys & 7u) || ((uintptr_t)cfg->w & 3u))
    return DES_ERR_INVALID_ARG;
  const uint64_t n_slots = slots_for(cfg->capacity_rows);
  if (cfg->slots_bytes < n_slots * sizeof(Slot)) return DES_ERR_WORKSPACE;
  if (cfg->workspace_bytes < 256 + insert_ws_bytes(1)) return DES_ERR_WORKSPACE;
  des_table *t = new (std::nothrow) des_table;
  if (!t) return DES_ERR_DEVICE;
  t->cfg = *cfg;
  t->n_slots = n_slots;
  t->slots = (Slot *)cfg->slots;
  t->ctrl = (Ctrl *)cfg->workspace;
  t->ws = (char *)cfg->workspace + 256;
  t->ws_bytes = cfg->workspace_bytes - 256;
  t->max_n = 0;
  t->init_width = (float)(2.0 * sqrt(3.0) * (double)cfg->init_scale);
  t->last_stream = nullptr;
  t->prep.valid = false;
  // empty slot = all-ones key, row -1: one 16-byte pattern of 0xFF
  const uint4 ones = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
  hipLaunchKernelGGL(k_fill_u64x2, dim3(grid_for((int64_t)n_slots, kBlock, 65536)), dim3(kBlock), 0, nullptr,
                     (uint4 *)t->slots, (int64_t)n_slots, ones);
  hipLaunchKernelGGL(k_zero_ctrl, dim3(1), dim3(1), 0, nullptr, t->ctrl);
  if (hipStreamSynchronize(nullptr) != hipSuccess || hipGetLastError() != hipSuccess) {
    delete t;
    return DES_ERR_DEVICE;
  }
  *out = t;
  return DES_OK;
}

des_status_t des_table_destroy(des_table_t *t) {
  if (!t) return DES_ERR_INVALID_ARG;
  (void)hipStreamSynchronize(t->last_stream);
  delete t;
  return DES_OK;
}

static des_status_t insert_impl(des_table_t *t, const uint64_t *keys, int64_t n, const float *values,
                                int32_t *rows_out, bool insert, hipStream_t s) {
  if (!t || n < 0 || n >= 2147483647ll || (n > 0 && !keys)) return DES_ERR_INVALID_ARG;
  if (((uintptr_t)keys & 7u) || ((uintptr_t)rows_out & 3u) || ((uintptr_t)values & 3u)) return DES_ERR_INVALID_ARG;
  t->last_stream = s;
  // a prepared (row-sorted) batch does not survive any lookup: an insert reuses its workspace, and a lookup may
  // be refilling the very rows array the sorted form was built from
  t->prep.valid = false;
  if (n == 0) return DES_OK;
  if (insert && insert_ws_bytes(n) > t->ws_bytes) return DES_ERR_WORKSPACE;
  const uint64_t mask = t->n_slots - 1;
  if (!insert) {
    if (!rows_out) return DES_ERR_INVALID_ARG;
    ProfScope ps(KID_PROBE, s);
    hipLaunchKernelGGL(k_probe<false>, dim3(grid_for(n, kBlock * kProbeKeys)), dim3(kBlock), 0, s, t->slots, mask, keys, n, rows_out,
                       t->ctrl, (uint32_t *)nullptr);
    return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
  }
  const size_t m = (size_t)n;
  char *p = t->ws;
  int32_t *tmp_rows = (int32_t *)p; p += align_up(m * 4, 256);
  uint32_t *slot_of = (uint32_t *)p; p += align_up(m * 4, 256);
  int32_t *first_idx = (int32_t *)p; p += align_up(m * 4, 256);
  uint32_t *tile_sums = (uint32_t *)p;
  int32_t *rows = rows_out ? rows_out : tmp_rows;
  const des_table_config_t &c = t->cfg;
  const int64_t nb = (n + kFlagTile - 1) / kFlagTile;
  {
    ProfScope ps(KID_PROBE, s);
    hipLaunchKernelGGL(k_probe<true>, dim3(grid_for(n, kBlock * kProbeKeys)), dim3(kBlock), 0, s, t->slots, mask, keys, n, rows, t->ctrl,
                       slot_of);
  }
  {
    ProfScope ps(KID_ASSIGN, s);
    hipLaunchKernelGGL(k_new_count, dim3((unsigned)nb), dim3(kBlock), 0, s, t->slots, rows, slot_of, n, tile_sums);
    if (nb > kSelfPrefixTiles) {
      hipLaunchKernelGGL(k_new_sums, dim3(1), dim3(kBlock), 0, s, tile_sums, nb, t->ctrl, c.capacity_rows);
      hipLaunchKernelGGL(k_new_assign<false>, dim3((unsigned)nb), dim3(kBlock), 0, s, t->slots, rows, slot_of, keys, n,
                         tile_sums, t->ctrl, c.row_keys, first_idx, c.capacity_rows);
    } else {
      hipLaunchKernelGGL(k_new_assign<true>, dim3((unsigned)nb), dim3(kBlock), 0, s, t->slots, rows, slot_of, keys, n,
                         tile_sums, t->ctrl, c.row_keys, first_idx, c.capacity_rows);
    }
  }
  {
    ProfScope ps(KID_INIT_ROWS, s);
    if (values)
      hipLaunchKernelGGL(k_copy_values, dim3(grid_for(n * (c.dim + 1), kBlock, 2048)), dim3(kBlock), 0, s, t->ctrl,
                         c.dim, values, first_idx, c.emb, c.w, c.acc_emb, c.acc_w, c.acc2_emb, c.acc2_w, c.capacity_rows);
    else
      hipLaunchKernelGGL(k_init_rows, dim3(grid_for(n * (c.dim / 4 + 1), kBlock, 2048)), dim3(kBlock), 0, s, t->ctrl,
                         c.dim, c.init_seed, t->init_width, c.row_keys, c.emb, c.w, c.acc_emb, c.acc_w,
                         c.acc2_emb, c.acc2_w, c.capacity_rows);
  }
  {
    ProfScope ps(KID_PATCH, s);
    hipLaunchKernelGGL(k_patch, dim3(grid_for(n)), dim3(kBlock), 0, s, t->slots, n, rows, slot_of, t->ctrl, c.capacity_rows);
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_table_insert(des_table_t *t, const uint64_t *keys, int64_t n, const float *values,
                              int32_t *rows_out, void *stream) {
  return insert_impl(t, keys, n, values, rows_out, true, (hipStream_t)stream);
}

des_status_t des_table_find(des_table_t *t, const uint64_t *keys, int64_t n, int32_t miss, int32_t *rows_out,
                            void *stream) {
  if (miss != DES_MISS_ZERO && miss != DES_MISS_INSERT) return DES_ERR_INVALID_ARG;
  if (n > 0 && !rows_out) return DES_ERR_INVALID_ARG;
  return insert_impl(t, keys, n, nullptr, rows_out, miss == DES_MISS_INSERT, (hipStream_t)stream);
}

des_status_t des_table_size(des_table_t *t, int64_t *n_rows_host) {
  if (!t || !n_rows_host) return DES_ERR_INVALID_ARG;
  long long v = 0;
  if (hipStreamSynchronize(t->last_stream) != hipSuccess) return DES_ERR_DEVICE;
  if (hipMemcpy(&v, &t->ctrl->n_rows, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return DES_ERR_DEVICE;
  *n_rows_host = v;
  return DES_OK;
}

des_status_t des_table_status(des_table_t *t) {
  if (!t) return DES_ERR_INVALID_ARG;
  int v[2] = {0, 0};                               // status, bad_keys: adjacent in the control block
  static_assert(offsetof(Ctrl, bad_keys) == offsetof(Ctrl, status) + sizeof(int), "read as one pair");
  if (hipStreamSynchronize(t->last_stream) != hipSuccess) return DES_ERR_DEVICE;
  if (hipMemcpy(v, &t->ctrl->status, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return DES_ERR_DEVICE;
  if (v[0] != 0) return (des_status_t)v[0];
  return v[1] != 0 ? DES_ERR_INVALID_KEY : DES_OK;
}

des_status_t des_table_clear_status(des_table_t *t) {
  if (!t) return DES_ERR_INVALID_ARG;
  hipStream_t s = t->last_stream;
  t->prep.valid = false;
  hipLaunchKernelGGL(k_clear_status, dim3(grid_for((int64_t)t->n_slots, kBlock, 65536)), dim3(kBlock), 0, s, t->slots,
                     t->n_slots, t->ctrl);
  if (hipStreamSynchronize(s) != hipSuccess || hipGetLastError() != hipSuccess) return DES_ERR_DEVICE;
  return DES_OK;
}

des_status_t des_table_export_keys(des_table_t *t, uint64_t *row_keys_out, int64_t max_rows, void *stream) {
  if (!t || max_rows < 0 || (max_rows > 0 && !row_keys_out) || ((uintptr_t)row_keys_out & 7u)) return DES_ERR_INVALID_ARG;
  if (max_rows == 0) return DES_OK;
  hipStream_t s = (hipStream_t)stream;
  t->last_stream = s;
  ProfScope ps(KID_EXPORT, s);
  const int64_t most = max_rows < t->cfg.capacity_rows ? max_rows : t->cfg.capacity_rows;
  hipLaunchKernelGGL(k_export_keys, dim3(grid_for(most, kBlock, 65536)), dim3(kBlock), 0, s, t->ctrl, t->cfg.row_keys,
                     row_keys_out, max_rows);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_aggregate_partials(const float *P, int32_t K, int64_t n, float *out, void *stream) {
  if (K < 1 || n < 0 || (n > 0 && (!P || !out))) return DES_ERR_INVALID_ARG;
  if (((uintptr_t)P & 3u) || ((uintptr_t)out & 3u)) return DES_ERR_INVALID_ARG;
  if (n == 0) return DES_OK;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_AGGREGATE, s);
  const bool vec = (n % 4 == 0) && aligned16(P) && aligned16(out);
  if (vec)
    hipLaunchKernelGGL(k_aggregate<true>, dim3(grid_for(n / 4)), dim3(kBlock), 0, s, P, K, n, out);
  else
    hipLaunchKernelGGL(k_aggregate<false>, dim3(grid_for(n)), dim3(kBlock), 0, s, P, K, n, out);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_aggregate_forward(const float *P_lr, const float *P_sum, const float *P_sq, int32_t K, int64_t B,
                                   int32_t D, float *A_lr, float *A_sum, float *A_sq, float *fm2, void *stream) {
  if (K < 1 || B < 0 || D < 4 || (D & 3)) return DES_ERR_INVALID_ARG;
  if ((P_sum == nullptr) != (P_sq == nullptr) || (!P_lr && !P_sum)) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  if ((P_lr && !A_lr) || (P_sum && (!A_sum || !A_sq))) return DES_ERR_INVALID_ARG;
  if (P_sum && (!aligned16(P_sum) || !aligned16(A_sum))) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_AGGREGATE, s);
  hipLaunchKernelGGL(k_aggregate_forward, dim3(grid_for(B * 8, kBlock, 1ll << 30)), dim3(kBlock), 0, s, P_lr, P_sum, P_sq,
                     K, B, D, A_lr, A_sum, A_sq, fm2);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_fm_finalize(const float *A_sum, const float *A_sq, int64_t B, int32_t D, float *fm2, void *stream) {
  if (B < 0 || D < 1 || (B > 0 && (!A_sum || !A_sq || !fm2))) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_FM_FINALIZE, s);
  hipLaunchKernelGGL(k_fm_finalize, dim3(grid_for(B * 8, kBlock, 1ll << 30)), dim3(kBlock), 0, s, A_sum, A_sq, B, D, fm2);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

static des_status_t check_batch(des_table_t *t, const des_batch_t *b, const int32_t *rows) {
  if (!t || !b) return DES_ERR_INVALID_ARG;
  if (b->B < 0 || b->F < 1 || b->nnz < 0 || b->nnz >= 2147483647ll || b->B * (int64_t)b->F >= 2147483647ll)
    return DES_ERR_INVALID_ARG;
  if (!b->offsets) return DES_ERR_INVALID_ARG;
  if (b->nnz > 0 && (!b->keys || !rows)) return DES_ERR_INVALID_ARG;
  if (((uintptr_t)b->keys & 7u) || ((uintptr_t)b->offsets & 3u) || ((uintptr_t)rows & 3u) || ((uintptr_t)b->vals & 3u))
    return DES_ERR_INVALID_ARG;
  return DES_OK;
}

des_status_t des_partial_forward(des_table_t *t, const des_batch_t *batch, const int32_t *rows, float *P_lr,
                                 float *P_sum, float *P_sq, float *pool, void *stream) {
  des_status_t st = check_batch(t, batch, rows);
  if (st != DES_OK) return st;
  if ((P_sum == nullptr) != (P_sq == nullptr)) return DES_ERR_INVALID_ARG;
  if (!P_lr && !P_sum && !pool) return DES_ERR_INVALID_ARG;
  if ((P_sum && !aligned16(P_sum)) || (pool && !aligned16(pool))) return DES_ERR_INVALID_ARG;
  t->last_stream = (hipStream_t)stream;
  return forward_launch(t, batch, rows, P_lr, P_sum, P_sq, pool, (hipStream_t)stream);
}

des_status_t des_partial_forward_lr(des_table_t *t, const des_batch_t *batch, const int32_t *rows, float *P_lr,
                                    void *stream) {
  if (!P_lr) return DES_ERR_INVALID_ARG;
  return des_partial_forward(t, batch, rows, P_lr, nullptr, nullptr, nullptr, stream);
}

des_status_t des_partial_forward_fm(des_table_t *t, const des_batch_t *batch, const int32_t *rows, float *P_sum,
                                    float *P_sq, void *stream) {
  if (!P_sum || !P_sq) return DES_ERR_INVALID_ARG;
  return des_partial_forward(t, batch, rows, nullptr, P_sum, P_sq, nullptr, stream);
}

des_status_t des_partial_forward_pool(des_table_t *t, const des_batch_t *batch, const int32_t *rows, float *P_pool,
                                      int32_t dense_k, void *stream) {
  if (!P_pool) return DES_ERR_INVALID_ARG;
  if (!dense_k) return des_partial_forward(t, batch, rows, nullptr, nullptr, nullptr, P_pool, stream);
  des_status_t st = check_batch(t, batch, rows);
  if (st != DES_OK) return st;
  if (!aligned16(P_pool)) return DES_ERR_INVALID_ARG;
  t->last_stream = (hipStream_t)stream;
  return pool_dense_launch(t, batch, rows, P_pool, (hipStream_t)stream);
}

static bool state_ok(const des_table_config_t &c, int opt, bool emb) {
  const float *s1 = emb ? c.acc_emb : c.acc_w, *s2 = emb ? c.acc2_emb : c.acc2_w;
  switch (opt) {
    case DES_OPT_SGD: return true;
    case DES_OPT_ADAGRAD: return s1 != nullptr;
    case DES_OPT_ADAM: return s1 != nullptr && s2 != nullptr;
    case DES_OPT_FTRL: return !emb && s1 != nullptr && s2 != nullptr;
  }
  return false;
}

static des_status_t backward_api(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                 const des_backward_io_t *io, const des_optimizer_t *o, void *stream) {
  des_status_t st = check_batch(t, batch, rows);
  if (st != DES_OK) return st;
  if (!io || !o) return DES_ERR_INVALID_ARG;
  if ((io->g_fm == nullptr) != (io->A_sum == nullptr)) return DES_ERR_INVALID_ARG;
  if ((io->A_sum && !aligned16(io->A_sum)) || (io->g_pool && !aligned16(io->g_pool))) return DES_ERR_INVALID_ARG;
  const bool merge_only = o->opt_emb == DES_OPT_NONE && o->opt_w == DES_OPT_NONE;
  if (!merge_only) {
    if (!state_ok(t->cfg, o->opt_emb, true) || !state_ok(t->cfg, o->opt_w, false)) return DES_ERR_INVALID_ARG;
    const bool adagrad = o->opt_emb == DES_OPT_ADAGRAD || o->opt_w == DES_OPT_ADAGRAD;
    const bool adam = o->opt_emb == DES_OPT_ADAM || o->opt_w == DES_OPT_ADAM;
    if (!(o->lr == o->lr)) return DES_ERR_INVALID_ARG;
    if ((adagrad || adam) && !(o->eps > 0.f)) return DES_ERR_INVALID_ARG;
    if (adam && (!(o->beta1 >= 0.f && o->beta1 < 1.f) || !(o->beta2 >= 0.f && o->beta2 < 1.f) || o->step < 1))
      return DES_ERR_INVALID_ARG;
    if (o->opt_w == DES_OPT_FTRL && (!(o->ftrl_alpha > 0.f) || !(o->ftrl_beta >= 0.f) || !(o->ftrl_l1 >= 0.f) ||
                                    !(o->ftrl_l2 >= 0.f)))
      return DES_ERR_INVALID_ARG;
  }
  if (256 + backward_ws_bytes(t->cfg.dim, batch->nnz) > t->cfg.workspace_bytes) return DES_ERR_WORKSPACE;
  t->last_stream = (hipStream_t)stream;
  return backward_launch(t, batch, rows, io, o, (hipStream_t)stream);
}

static des_optimizer_t simple_optimizer(int opt, float lr, float eps) {
  des_optimizer_t o;
  memset(&o, 0, sizeof(o));
  o.opt_emb = o.opt_w = opt;
  o.lr = lr;
  o.eps = eps;
  o.step = 1;
  return o;
}

des_status_t des_backward_update_sgd(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                     const des_backward_io_t *io, float lr, void *stream) {
  const des_optimizer_t o = simple_optimizer(DES_OPT_SGD, lr, 0.f);
  return backward_api(t, batch, rows, io, &o, stream);
}

des_status_t des_backward_update_adagrad(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                         const des_backward_io_t *io, float lr, float eps, void *stream) {
  const des_optimizer_t o = simple_optimizer(DES_OPT_ADAGRAD, lr, eps);
  return backward_api(t, batch, rows, io, &o, stream);
}

des_status_t des_backward_update(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                 const des_backward_io_t *io, const des_optimizer_t *optimizer, void *stream) {
  if (optimizer && (optimizer->opt_emb == DES_OPT_NONE) != (optimizer->opt_w == DES_OPT_NONE)) return DES_ERR_INVALID_ARG;
  return backward_api(t, batch, rows, io, optimizer, stream);
}

des_status_t des_backward_prepare(des_table_t *t, const des_batch_t *batch, const int32_t *rows, void *stream) {
  des_status_t st = check_batch(t, batch, rows);
  if (st != DES_OK) return st;
  if (256 + backward_ws_bytes(t->cfg.dim, batch->nnz) > t->cfg.workspace_bytes) return DES_ERR_WORKSPACE;
  return backward_prepare_launch(t, batch, rows, (hipStream_t)stream);
}

des_status_t des_backward_merge(des_table_t *t, const des_batch_t *batch, const int32_t *rows,
                                const des_backward_io_t *io, void *stream) {
  const des_optimizer_t o = simple_optimizer(DES_OPT_NONE, 0.f, 0.f);
  return backward_api(t, batch, rows, io, &o, stream);
}

}  // extern "C"
