// Backward of the sparse operators, duplicate-key merge and fused optimizer update.
//
// Section 3.2.2 (back-propagation phase): the gradient of each aggregate is handed unchanged to
// every shard's sub-operator, so the backward pass needs no exchange.  Section 5: the merged
// gradient of a weight is applied locally and the table row is updated.
//
// Steps: (1) expand the CSR batch to (row, bag) pairs, (2) stable radix sort by row, (3) mark
// segment heads and compact them (ascending row order), (4) one lane group per segment of up to
// kShortMax entries reduces its entries in registers and updates the row in the same kernel; longer
// segments are cut into chunks of kChunk entries, one wave each: a segment that is a single chunk
// is updated by that wave, the others are combined and updated by one workgroup per segment.
// Steps (1)-(3) need the batch and its rows only and can be issued ahead of the gradients
// (des_backward_prepare).
//
// Per entry e of bag (b,f) with value x:  d/dw += x*g_lr[b],
//   d/dv += x*(g_fm[b]*A_sum[b,:] + g_pool[b,f,:]) - v * (x*x*g_fm[b])
// i.e. the row's own vector v enters only through one scalar per segment, so v is read once.
#include <math.h>
#include "des_internal.h"

namespace des {
namespace {

constexpr int kShortMax = 32;              // segments up to this many entries are reduced by one lane group
constexpr int kChunk = 512;                // entries per chunk of a longer segment (one wave per chunk)
constexpr int kMidFan = 64;                // chunk partials that one wave pre-sums for segments of more chunks than this
constexpr int kShortGrid = 65536;          // most workgroups of the short-segment kernel (it strides over the segments)
constexpr int kHeadItems = 8;
constexpr int kHeadTile = kBlock * kHeadItems;
constexpr int64_t kHeadsSelfPrefix = 4096;  // up to this many tiles every workgroup sums the earlier tiles' head counts itself
constexpr int kWavesPerBlock = kBlock / kWave;

struct BwdArgs {
  // batch and upstream gradients
  const int32_t *offsets;
  const float *vals;
  const int32_t *rows;
  const float *g_lr, *g_fm, *A_sum, *g_pool;
  int64_t n;            // nnz
  int64_t nbags;
  int F;
  uint32_t missing;     // sort key of entries without a row (= capacity, sorts last)
  // table
  float *emb, *w, *acc_emb, *acc_w, *acc2_emb, *acc2_w;
  const uint64_t *row_keys;
  Ctrl *ctrl;
  // workspace
  uint32_t *key_sorted, *pay_sorted;
  int32_t *bag_of;      // entry -> bag, only with vals
  int32_t *seg_off;     // [n+1]
  int32_t *uniq_rows;   // [n]
  uint32_t *first_pay;  // [n]  payload of the first entry of each segment
  uint32_t *head_sums;
  int32_t *long_seg;    // segment index of long segment j
  uint32_t *long_c0;    // first chunk of long segment j
  int32_t *multi_seg;   // long segment indices j of the segments with more than one chunk
  int32_t *group_seg;   // long segment index j of pre-summed group i (segments of more than kMidFan chunks)
  uint32_t *group_c;    // first chunk of that group
  int32_t *chunk_owner; // long segment index of chunk c
  double *partials;     // [chunks][D+4]
  // optimizer (opt_emb == DES_OPT_NONE: merge only)
  int opt_emb, opt_w;
  float lr, eps;
  float b1, b2, c1, c2;   // Adam: decay rates and bias corrections 1/(1-b1^t), 1/(1-b2^t)
  float f_alpha, f_beta, f_l1, f_l2;
  // optional outputs
  int32_t *uniq_rows_out;
  uint64_t *uniq_keys_out;
  int32_t *counts_out;
  float *merged_out;
  int64_t *n_uniq_out;
};

__device__ inline float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ inline void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
// Streaming variants for data that is touched once per call (table rows of one-entry segments,
// upstream gradient rows): they do not displace the reusable lines in the caches.
typedef float v4f __attribute__((ext_vector_type(4)));
__device__ inline float4 ld4_stream(const float *p) {
  const v4f r = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
  return make_float4(r.x, r.y, r.z, r.w);
}
__device__ inline void st4_stream(float *p, float4 v) {
  v4f r; r.x = v.x; r.y = v.y; r.z = v.z; r.w = v.w;
  __builtin_nontemporal_store(r, reinterpret_cast<v4f *>(p));
}
__device__ inline float4 f4zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ inline float4 f4add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// (1) sort key = row (or `missing`), payload = bag (or entry index with vals).  A workgroup takes
// kBlock consecutive bags, i.e. one contiguous range of entries, stages their offsets in LDS and
// walks the entries with consecutive threads (coalesced reads and writes); the bag of an entry
// is found by binary search in the staged offsets.
template <bool kHasVals>
__global__ __launch_bounds__(kBlock) void k_expand(const BwdArgs a, uint32_t *__restrict__ key_out,
                                                    uint32_t *__restrict__ pay_out) {
  __shared__ int offs[kBlock + 1];
  for (int64_t bag0 = (int64_t)blockIdx.x * kBlock; bag0 < a.nbags; bag0 += (int64_t)gridDim.x * kBlock) {
    const int nb = (int)min((int64_t)kBlock, a.nbags - bag0);
    __syncthreads();
    for (int i = threadIdx.x; i <= nb; i += kBlock) offs[i] = a.offsets[bag0 + i];
    __syncthreads();
    const int e0 = offs[0], e1 = offs[nb];
    for (int e = e0 + threadIdx.x; e < e1; e += kBlock) {
      int lo = 0, hi = nb;                              // largest i with offs[i] <= e
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offs[mid] <= e) lo = mid; else hi = mid;
      }
      const int r = a.rows[e];
      key_out[e] = r >= 0 ? (uint32_t)r : a.missing;
      pay_out[e] = kHasVals ? (uint32_t)e : (uint32_t)(bag0 + lo);
      if (kHasVals) a.bag_of[e] = (int32_t)(bag0 + lo);
    }
  }
}

// (3) segment heads.  flag(i) = key[i] is a row and differs from key[i-1].
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

// The thread's kHeadItems consecutive sorted keys (two 16-byte loads when they all exist); missing ones read as `fill`.
__device__ inline void load_head_keys(const uint32_t *__restrict__ keys, int64_t base, int64_t n, uint32_t fill,
                                      uint32_t (&k)[kHeadItems]) {
  static_assert(kHeadItems == 8, "two uint4 per thread");
  if (base + kHeadItems <= n) {
    const uint4 lo = *reinterpret_cast<const uint4 *>(keys + base);
    const uint4 hi = *reinterpret_cast<const uint4 *>(keys + base + 4);
    k[0] = lo.x; k[1] = lo.y; k[2] = lo.z; k[3] = lo.w; k[4] = hi.x; k[5] = hi.y; k[6] = hi.z; k[7] = hi.w;
  } else {
#pragma unroll
    for (int i = 0; i < kHeadItems; ++i) k[i] = base + i < n ? keys[base + i] : fill;
  }
}

__global__ __launch_bounds__(kBlock) void k_heads_count(const BwdArgs a) {
  __shared__ uint32_t lds[kWavesPerBlock];
  const int64_t n = a.n;
  const int64_t base = (int64_t)blockIdx.x * kHeadTile + (int64_t)threadIdx.x * kHeadItems;
  uint32_t cnt = 0;
  uint32_t prev = base > 0 && base <= n ? a.key_sorted[base - 1] : 0xFFFFFFFFu;
  uint32_t keys[kHeadItems];
  load_head_keys(a.key_sorted, base, n, a.missing, keys);
#pragma unroll
  for (int i = 0; i < kHeadItems; ++i) {
    if (base + i < n) {
      const uint32_t k = keys[i];
      cnt += (k != a.missing && (base + i == 0 || k != prev)) ? 1u : 0u;
      prev = k;
    }
  }
  uint32_t total;
  block_excl_scan_u32(cnt, lds, total);
  if (threadIdx.x == 0) a.head_sums[blockIdx.x] = total;
}

// Bookkeeping after a device-wide scan of the tile counts (many tiles): the scan left the total behind the counts.
__device__ inline void heads_bookkeeping(const BwdArgs &a, uint32_t n_uniq) {
  a.ctrl->n_uniq = n_uniq;
  a.ctrl->n_long = 0;
  a.ctrl->n_chunks = 0;
  a.ctrl->n_multi = 0;
  a.ctrl->n_groups = 0;
  if (a.n_uniq_out) *a.n_uniq_out = n_uniq;
}

__global__ void k_heads_finish(const BwdArgs a, const uint32_t *total) { heads_bookkeeping(a, *total); }

// kSelfPrefix: head_sums still holds the tiles' counts and every workgroup adds up the counts of the tiles before
// its own (few tiles: cheaper than a launch that does it once); the last workgroup then also publishes the
// number of segments and resets the counters of the classify pass.
template <bool kSelfPrefix>
__global__ __launch_bounds__(kBlock) void k_heads_write(const BwdArgs a) {
  __shared__ uint32_t lds[kWavesPerBlock];
  __shared__ uint32_t l_key[kHeadTile];
  __shared__ int32_t l_idx[kHeadTile];
  const int64_t n = a.n;
  const int64_t base = (int64_t)blockIdx.x * kHeadTile + (int64_t)threadIdx.x * kHeadItems;
  uint32_t key[kHeadItems];
  bool flag[kHeadItems];
  uint32_t cnt = 0;
  uint32_t prev = base > 0 && base <= n ? a.key_sorted[base - 1] : 0xFFFFFFFFu;
  const uint32_t first_prev = prev;
  load_head_keys(a.key_sorted, base, n, a.missing, key);
#pragma unroll
  for (int i = 0; i < kHeadItems; ++i) {
    flag[i] = false;
    if (base + i < n) {
      flag[i] = key[i] != a.missing && (base + i == 0 || key[i] != prev);
      cnt += flag[i] ? 1u : 0u;
      prev = key[i];
    }
  }
  uint32_t total;
  uint32_t u0;                                          // heads before this tile
  if (kSelfPrefix) {
    uint32_t part = 0;
    for (uint32_t i = threadIdx.x; i < blockIdx.x; i += kBlock) part += a.head_sums[i];
    block_excl_scan_u32(part, lds, u0);
  } else {
    u0 = a.head_sums[blockIdx.x];
  }
  uint32_t loc = block_excl_scan_u32(cnt, lds, total);  // heads before this thread inside the tile
  if (kSelfPrefix && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) heads_bookkeeping(a, u0 + total);
  prev = first_prev;
#pragma unroll
  for (int i = 0; i < kHeadItems; ++i) {
    const int64_t idx = base + i;
    if (idx < n) {
      if (flag[i]) {
        l_key[loc] = key[i];
        l_idx[loc] = (int32_t)idx;
        ++loc;
      }
      // end of the last segment: first entry without a row, or the end of the array
      if (key[i] == a.missing && (idx == 0 || prev != a.missing)) a.seg_off[u0 + loc] = (int32_t)idx;
      if (idx == n - 1 && key[i] != a.missing) a.seg_off[u0 + loc] = (int32_t)n;
      prev = key[i];
    }
  }
  __syncthreads();
  // the tile's heads occupy consecutive output positions: write them with consecutive threads
  for (uint32_t j = threadIdx.x; j < total; j += kBlock) {
    const int32_t idx = l_idx[j];
    a.uniq_rows[u0 + j] = (int32_t)l_key[j];
    a.seg_off[u0 + j] = idx;
    a.first_pay[u0 + j] = a.pay_sorted[idx];
  }
}

// Long segments get a chunk range.  The order of the list is irrelevant to the results, so
// ranges are handed out with one atomic pair per workgroup.
__global__ __launch_bounds__(kBlock) void k_classify(const BwdArgs a) {
  __shared__ uint32_t lds[kWavesPerBlock];
  __shared__ unsigned long long base_long, base_chunk, base_multi, base_group;
  const long long U = a.ctrl->n_uniq;
  const int64_t tile0 = (int64_t)blockIdx.x * kHeadTile + (int64_t)threadIdx.x * kHeadItems;
  if ((int64_t)blockIdx.x * kHeadTile >= U) return;          // uniform per workgroup
  uint32_t nl = 0, nc = 0, nm = 0, ng = 0;
  int len[kHeadItems];
  if (tile0 + kHeadItems <= U) {                  // the thread's nine segment bounds: two 16-byte loads and one more
    const int4 lo = *reinterpret_cast<const int4 *>(a.seg_off + tile0);
    const int4 hi = *reinterpret_cast<const int4 *>(a.seg_off + tile0 + 4);
    const int last = a.seg_off[tile0 + kHeadItems];
    len[0] = lo.y - lo.x; len[1] = lo.z - lo.y; len[2] = lo.w - lo.z; len[3] = hi.x - lo.w;
    len[4] = hi.y - hi.x; len[5] = hi.z - hi.y; len[6] = hi.w - hi.z; len[7] = last - hi.w;
  } else {
#pragma unroll
    for (int i = 0; i < kHeadItems; ++i) {
      const int64_t u = tile0 + i;
      len[i] = u < U ? a.seg_off[u + 1] - a.seg_off[u] : 0;
    }
  }
#pragma unroll
  for (int i = 0; i < kHeadItems; ++i) {
    if (len[i] > kShortMax) {
      const uint32_t nch = (uint32_t)((len[i] + kChunk - 1) / kChunk);
      ++nl; nc += nch;
      if (nch > 1) ++nm;
      if (nch > kMidFan) ng += (nch + kMidFan - 1) / kMidFan;
    }
  }
  uint32_t tot_l, tot_c, tot_m, tot_g;
  uint32_t ex_l = block_excl_scan_u32(nl, lds, tot_l);
  uint32_t ex_c = block_excl_scan_u32(nc, lds, tot_c);
  if (tot_l == 0) return;                                    // uniform: the scans synchronised the workgroup
  uint32_t ex_m = block_excl_scan_u32(nm, lds, tot_m);
  uint32_t ex_g = block_excl_scan_u32(ng, lds, tot_g);
  if (threadIdx.x == 0) {
    typedef unsigned long long ull;
    base_long = atomicAdd(reinterpret_cast<ull *>(&a.ctrl->n_long), (ull)tot_l);
    base_chunk = atomicAdd(reinterpret_cast<ull *>(&a.ctrl->n_chunks), (ull)tot_c);
    base_multi = tot_m ? atomicAdd(reinterpret_cast<ull *>(&a.ctrl->n_multi), (ull)tot_m) : 0ull;
    base_group = tot_g ? atomicAdd(reinterpret_cast<ull *>(&a.ctrl->n_groups), (ull)tot_g) : 0ull;
  }
  __syncthreads();
  uint32_t j = (uint32_t)base_long + ex_l, c0 = (uint32_t)base_chunk + ex_c;
  uint32_t jm = (uint32_t)base_multi + ex_m, gi = (uint32_t)base_group + ex_g;
#pragma unroll
  for (int i = 0; i < kHeadItems; ++i) {
    if (len[i] > kShortMax) {
      const uint32_t nch = (uint32_t)((len[i] + kChunk - 1) / kChunk);
      a.long_seg[j] = (int32_t)(tile0 + i);
      a.long_c0[j] = c0;
      if (nch > 1) a.multi_seg[jm++] = (int32_t)j;           // what the per-segment combine has to visit
      if (nch > kMidFan)                                      // and the groups of chunk sums that are added up first
        for (uint32_t k = 0; k < nch; k += kMidFan) { a.group_seg[gi] = (int32_t)j; a.group_c[gi] = c0 + k; ++gi; }
      ++j;
      c0 += nch;
    }
  }
}

// one workgroup per long segment writes the owner of each of its chunks
__global__ __launch_bounds__(kBlock) void k_chunk_owner(const BwdArgs a) {
  const long long NL = a.ctrl->n_long;
  for (int64_t j = blockIdx.x; j < NL; j += gridDim.x) {
    const int u = a.long_seg[j];
    const int nch = (a.seg_off[u + 1] - a.seg_off[u] + kChunk - 1) / kChunk;
    const uint32_t c0 = a.long_c0[j];
    for (int i = threadIdx.x; i < nch; i += blockDim.x) a.chunk_owner[c0 + i] = (int32_t)j;
  }
}

// Gradient sums of the sorted entries [i0, i1) seen by the lane holding columns 4*sub..4*sub+3:
//   s1 = sum x*(g_fm[b]*A_sum[b,:] + g_pool[bag,:]),  s2 = sum x*x*g_fm[b],  gw = sum x*g_lr[b]
// Accumulated in double: the first Adagrad step divides the merged gradient by |G| + eps, so a
// gradient that cancels to the order of eps must keep an absolute accuracy far below fp32's.
struct Acc {
  double v[4];
  double s2, gw;
};
__device__ inline Acc acc_zero() { Acc r; r.v[0] = r.v[1] = r.v[2] = r.v[3] = 0.0; r.s2 = 0.0; r.gw = 0.0; return r; }

// Adds the terms of up to U entries whose bags (and values) are already known: all their upstream
// gradient rows are requested before the first is used.
template <int D, int U>
__device__ inline void accumulate_batch(const BwdArgs &a, const uint32_t (&bag)[U], const bool (&live)[U],
                                        const float (&x)[U], int sub, Acc &acc) {
  float gf[U], gl[U];
  float4 gp[U], as[U];
#pragma unroll
  for (int k = 0; k < U; ++k) {
    const uint32_t b = bag[k] / (uint32_t)a.F;
    gp[k] = (live[k] && a.g_pool) ? ld4(a.g_pool + (int64_t)bag[k] * D + sub * 4) : f4zero();
    as[k] = (live[k] && a.g_fm) ? ld4(a.A_sum + (int64_t)b * D + sub * 4) : f4zero();
    gf[k] = (live[k] && a.g_fm) ? a.g_fm[b] : 0.f;
    gl[k] = (live[k] && a.g_lr) ? a.g_lr[b] : 0.f;
  }
#pragma unroll
  for (int k = 0; k < U; ++k) {
    if (!live[k]) continue;
    const double xd = (double)x[k];
    const double xg = xd * (double)gf[k];
    acc.v[0] += xd * (double)gp[k].x + xg * (double)as[k].x;
    acc.v[1] += xd * (double)gp[k].y + xg * (double)as[k].y;
    acc.v[2] += xd * (double)gp[k].z + xg * (double)as[k].z;
    acc.v[3] += xd * (double)gp[k].w + xg * (double)as[k].w;
    acc.s2 += xd * xg;
    acc.gw += xd * (double)gl[k];
  }
}

// Bags (and values) of the sorted entries i .. i+U-1, clipped at i1.
template <bool kHasVals, int U>
__device__ inline void load_batch_meta(const BwdArgs &a, int i, int i1, uint32_t (&bag)[U], bool (&live)[U], float (&x)[U]) {
#pragma unroll
  for (int k = 0; k < U; ++k) {
    live[k] = i + k < i1;
    uint32_t p = live[k] ? a.pay_sorted[i + k] : 0u;
    x[k] = 1.f;
    if (kHasVals) {
      if (live[k]) x[k] = a.vals[p];
      p = live[k] ? (uint32_t)a.bag_of[p] : 0u;
    }
    bag[k] = p;
  }
}

// Per-sample values of the entry processed last by a lane group: entries of one row arrive in batch order, so a
// row that occurs many times in one sample (the hot IDs of a skewed batch) brings runs of entries with the same
// sample, which then reuse these instead of fetching them again.
struct SampleRun {
  uint32_t b;
  float4 as;
  float gf, gl;
};

// accumulate_batch for such runs: the A_sum row, g_fm and g_lr of an entry are fetched only if its sample differs
// from the previous entry's.  Same values, same order of additions as accumulate_batch.
template <int D, int U>
__device__ inline void accumulate_batch_runs(const BwdArgs &a, const uint32_t (&bag)[U], const bool (&live)[U],
                                             const float (&x)[U], int sub, Acc &acc, SampleRun &run) {
  float gf[U], gl[U];
  float4 gp[U], as[U];
  uint32_t b[U];
  bool same[U];
  uint32_t prev = run.b;
#pragma unroll
  for (int k = 0; k < U; ++k) {
    b[k] = bag[k] / (uint32_t)a.F;
    same[k] = live[k] && b[k] == prev;
    if (live[k]) prev = b[k];
    gp[k] = (live[k] && a.g_pool) ? ld4(a.g_pool + (int64_t)bag[k] * D + sub * 4) : f4zero();
    as[k] = (live[k] && !same[k] && a.g_fm) ? ld4(a.A_sum + (int64_t)b[k] * D + sub * 4) : f4zero();
    gf[k] = (live[k] && !same[k] && a.g_fm) ? a.g_fm[b[k]] : 0.f;
    gl[k] = (live[k] && !same[k] && a.g_lr) ? a.g_lr[b[k]] : 0.f;
  }
#pragma unroll
  for (int k = 0; k < U; ++k) {
    if (!live[k]) continue;
    if (same[k]) { as[k] = run.as; gf[k] = run.gf; gl[k] = run.gl; }
    run.b = b[k]; run.as = as[k]; run.gf = gf[k]; run.gl = gl[k];
    const double xd = (double)x[k];
    const double xg = xd * (double)gf[k];
    acc.v[0] += xd * (double)gp[k].x + xg * (double)as[k].x;
    acc.v[1] += xd * (double)gp[k].y + xg * (double)as[k].y;
    acc.v[2] += xd * (double)gp[k].z + xg * (double)as[k].z;
    acc.v[3] += xd * (double)gp[k].w + xg * (double)as[k].w;
    acc.s2 += xd * xg;
    acc.gw += xd * (double)gl[k];
  }
}

// Sums over the sorted entries [i0, i1), U at a time; the payloads of the next U entries are requested
// before the gradient rows of the current ones, so a batch costs one memory round trip, not two.
// kRuns: reuse the per-sample values along runs of entries of one sample (long segments).
template <int D, bool kHasVals, int U, bool kRuns = false>
__device__ inline void reduce_entries(const BwdArgs &a, int i0, int i1, int sub, Acc &acc) {
  uint32_t nbag[U];
  bool nlive[U];
  float nx[U];
  SampleRun run;
  run.b = 0xFFFFFFFFu; run.as = f4zero(); run.gf = 0.f; run.gl = 0.f;
  if (i0 < i1) load_batch_meta<kHasVals, U>(a, i0, i1, nbag, nlive, nx);
  for (int i = i0; i < i1; i += U) {
    uint32_t bag[U];
    bool live[U];
    float x[U];
#pragma unroll
    for (int k = 0; k < U; ++k) { bag[k] = nbag[k]; live[k] = nlive[k]; x[k] = nx[k]; }
    if (i + U < i1) load_batch_meta<kHasVals, U>(a, i + U, i1, nbag, nlive, nx);
    if (kRuns) accumulate_batch_runs<D, U>(a, bag, live, x, sub, acc, run);
    else accumulate_batch<D, U>(a, bag, live, x, sub, acc);
  }
}

// Pre-update state of one row as seen by the lane that owns columns 4*sub..4*sub+3 (sub 0 also
// owns the LR weight).  Loaded before the gradient reduction so that the row's memory latency
// overlaps the gathers of the upstream gradients.
struct RowState {
  float4 v, s, s2;      // latent columns and their first / second state arrays
  float w, aw, aw2;     // LR weight and its state
};

// kSecond = false: the caller knows that no second state array is in use (SGD, Adagrad), which frees its registers.
template <int D, bool kSecond = true>
__device__ inline RowState load_row(const BwdArgs &a, int row, int sub) {
  RowState st;
  st.v = ld4_stream(a.emb + (int64_t)row * D + sub * 4);
  st.s = f4zero();
  st.s2 = f4zero();
  st.w = st.aw = st.aw2 = 0.f;
  if (a.opt_emb == DES_OPT_ADAGRAD || a.opt_emb == DES_OPT_ADAM)
    st.s = ld4_stream(a.acc_emb + (int64_t)row * D + sub * 4);
  if (kSecond && a.opt_emb == DES_OPT_ADAM) st.s2 = ld4_stream(a.acc2_emb + (int64_t)row * D + sub * 4);
  if (sub == 0 && a.opt_w != DES_OPT_NONE) {
    st.w = a.w[row];
    if (a.opt_w != DES_OPT_SGD) st.aw = a.acc_w[row];
    if (kSecond && (a.opt_w == DES_OPT_ADAM || a.opt_w == DES_OPT_FTRL)) st.aw2 = a.acc2_w[row];
  }
  return st;
}

__device__ inline float adam_step(const BwdArgs &a, float g, float &m, float &v) {
  m = a.b1 * m + (1.f - a.b1) * g;
  v = a.b2 * v + (1.f - a.b2) * g * g;
  return a.lr * (m * a.c1) / (sqrtf(v * a.c2) + a.eps);
}

// Apply the merged gradient of one row.  The merged gradient is formed in double and rounded
// once; the optimizer arithmetic itself is well conditioned and runs in fp32 (FTRL, one scalar
// per row with a difference of square roots, in double).
template <int D, bool kSecond = true>
__device__ inline void apply_row(const BwdArgs &a, int64_t u, int row, int sub, const RowState &st, const Acc &acc) {
  const float4 v = st.v;
  const float4 G = make_float4((float)(acc.v[0] - (double)v.x * acc.s2), (float)(acc.v[1] - (double)v.y * acc.s2),
                               (float)(acc.v[2] - (double)v.z * acc.s2), (float)(acc.v[3] - (double)v.w * acc.s2));
  const float gw = (float)acc.gw;
  float *vp = a.emb + (int64_t)row * D + sub * 4;
  if (a.merged_out) {
    float *m = a.merged_out + u * (D + 1) + sub * 4;
    m[0] = G.x; m[1] = G.y; m[2] = G.z; m[3] = G.w;
    if (sub == 0) a.merged_out[u * (D + 1) + D] = gw;
  }
  if (a.opt_emb == DES_OPT_SGD) {
    st4_stream(vp, make_float4(v.x - a.lr * G.x, v.y - a.lr * G.y, v.z - a.lr * G.z, v.w - a.lr * G.w));
  } else if (a.opt_emb == DES_OPT_ADAGRAD) {
    float4 s = st.s;
    s.x += G.x * G.x; s.y += G.y * G.y; s.z += G.z * G.z; s.w += G.w * G.w;
    st4_stream(a.acc_emb + (int64_t)row * D + sub * 4, s);
    st4_stream(vp, make_float4(v.x - a.lr * G.x / (sqrtf(s.x) + a.eps), v.y - a.lr * G.y / (sqrtf(s.y) + a.eps),
                               v.z - a.lr * G.z / (sqrtf(s.z) + a.eps), v.w - a.lr * G.w / (sqrtf(s.w) + a.eps)));
  } else if (kSecond && a.opt_emb == DES_OPT_ADAM) {
    float4 m = st.s, q = st.s2;
    const float dx = adam_step(a, G.x, m.x, q.x), dy = adam_step(a, G.y, m.y, q.y);
    const float dz = adam_step(a, G.z, m.z, q.z), dw = adam_step(a, G.w, m.w, q.w);
    st4_stream(a.acc_emb + (int64_t)row * D + sub * 4, m);
    st4_stream(a.acc2_emb + (int64_t)row * D + sub * 4, q);
    st4_stream(vp, make_float4(v.x - dx, v.y - dy, v.z - dz, v.w - dw));
  }
  if (sub == 0) {
    if (a.opt_w == DES_OPT_SGD) {
      a.w[row] = st.w - a.lr * gw;
    } else if (a.opt_w == DES_OPT_ADAGRAD) {
      const float aw = st.aw + gw * gw;
      a.acc_w[row] = aw;
      a.w[row] = st.w - a.lr * gw / (sqrtf(aw) + a.eps);
    } else if (kSecond && a.opt_w == DES_OPT_ADAM) {
      float m = st.aw, q = st.aw2;
      const float d = adam_step(a, gw, m, q);
      a.acc_w[row] = m;
      a.acc2_w[row] = q;
      a.w[row] = st.w - d;
    } else if (kSecond && a.opt_w == DES_OPT_FTRL) {
      const double g = acc.gw, n0 = (double)st.aw, alpha = (double)a.f_alpha;
      const double n1 = n0 + g * g;
      const double sigma = (sqrt(n1) - sqrt(n0)) / alpha;
      const double z = (double)st.aw2 + g - sigma * (double)st.w;
      const double l1 = (double)a.f_l1;
      const double wn = fabs(z) <= l1 ? 0.0
                                      : -(z - (z > 0.0 ? l1 : -l1)) / (((double)a.f_beta + sqrt(n1)) / alpha + (double)a.f_l2);
      a.acc_w[row] = (float)n1;
      a.acc2_w[row] = (float)z;
      a.w[row] = (float)wn;
    }
  }
}

// Terms of one entry with payload p (bag, or entry index when feature values are present).
template <int D, bool kHasVals>
__device__ inline void add_entry(const BwdArgs &a, uint32_t p, int sub, Acc &acc) {
  float x = 1.f;
  if (kHasVals) {
    x = a.vals[p];
    p = (uint32_t)a.bag_of[p];
  }
  const uint32_t b = p / (uint32_t)a.F;
  const float4 gp = a.g_pool ? ld4_stream(a.g_pool + (int64_t)p * D + sub * 4) : f4zero();
  const float4 as = a.g_fm ? ld4(a.A_sum + (int64_t)b * D + sub * 4) : f4zero();
  const float gf = a.g_fm ? a.g_fm[b] : 0.f;
  const float gl = a.g_lr ? a.g_lr[b] : 0.f;
  const double xd = (double)x;
  const double xg = xd * (double)gf;
  acc.v[0] += xd * (double)gp.x + xg * (double)as.x;
  acc.v[1] += xd * (double)gp.y + xg * (double)as.y;
  acc.v[2] += xd * (double)gp.z + xg * (double)as.z;
  acc.v[3] += xd * (double)gp.w + xg * (double)as.w;
  acc.s2 += xd * xg;
  acc.gw += xd * (double)gl;
}

// (4a) one lane group per segment; long segments are left to the chunked path.  The segment's
// bounds, row and first payload arrive together; the row state and the first entry's upstream
// gradients are then fetched together, so a one-entry segment costs two memory round trips.
// The kernel waits on memory for most of its time, so a fifth wave per SIMD is worth more than registers: it is
// compiled for five (96 vector registers; at the 120 it would take by itself four fit), and gathers two entries'
// gradient rows at a time instead of four, which is what lets it fit almost without spilling.  Measured at the large
// table: 18.2 -> 16.5 ms; six waves (80 registers, 68 bytes of spill) lose that again.
// kSecond: an optimizer with a second state array (Adam, FTRL) may be in use.
template <int D, bool kHasVals, bool kSecond>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(5, 5))) void k_short_update(const BwdArgs a) {
  constexpr int G = D / 4;
  constexpr int U = 2;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int sub = (int)(gid % G);
  const int64_t ngroups = (int64_t)gridDim.x * blockDim.x / G;
  const int64_t n_uniq = a.ctrl->n_uniq;
  // grid-stride over the segments: the grid is sized on the host for the chip, not for the (device-side) segment count.
  // The bounds, row and first payload of the lane group's next segment are requested while the current one is being
  // worked on, which takes one of the two dependent round trips per segment off the critical path.
  int64_t u = gid / G;
  int i0_n = 0, i1_n = 0, row_n = 0;
  uint32_t p0_n = 0;
  if (u < n_uniq) { i0_n = a.seg_off[u]; i1_n = a.seg_off[u + 1]; row_n = a.uniq_rows[u]; p0_n = a.first_pay[u]; }
  for (; u < n_uniq; u += ngroups) {
    const int i0 = i0_n, i1 = i1_n;
    const int row = row_n;
    const uint32_t p0 = p0_n;
    {
      const int64_t un = u + ngroups;
      if (un < n_uniq) { i0_n = a.seg_off[un]; i1_n = a.seg_off[un + 1]; row_n = a.uniq_rows[un]; p0_n = a.first_pay[un]; }
    }
    const int len = i1 - i0;
    if (len > kShortMax) continue;
    Acc acc = acc_zero();
    if (G >= U) {
      // The payloads of the next G entries are fetched lane by lane in the same round trip as the row state and
      // the first entry's gradients, so a segment of up to G+1 entries costs 2 + ceil((len-1)/U) round trips.
      uint32_t mine = (1 + sub < len) ? a.pay_sorted[i0 + 1 + sub] : 0u;
      float myx = 1.f;
      const RowState st = load_row<D, kSecond>(a, row, sub);
      add_entry<D, kHasVals>(a, p0, sub, acc);
      const int glane = (int)(threadIdx.x & (kWave - 1)) - sub;       // first lane of this group in the wave
      for (int base = 1; base < len; base += G) {
        if (base > 1) mine = (base + sub < len) ? a.pay_sorted[i0 + base + sub] : 0u;
        if (kHasVals) {
          const bool have = base + sub < len;
          myx = have ? a.vals[mine] : 1.f;
          mine = have ? (uint32_t)a.bag_of[mine] : 0u;
        }
        const int cnt = min(G, len - base);
        for (int j0 = 0; j0 < cnt; j0 += U) {
          uint32_t bag[U];
          bool live[U];
          float x[U];
#pragma unroll
          for (int k = 0; k < U; ++k) {
            live[k] = j0 + k < cnt;
            bag[k] = __shfl(mine, glane + ((j0 + k) & (G - 1)), kWave);
            x[k] = kHasVals ? __shfl(myx, glane + ((j0 + k) & (G - 1)), kWave) : 1.f;
          }
          accumulate_batch<D, U>(a, bag, live, x, sub, acc);
        }
      }
      apply_row<D, kSecond>(a, u, row, sub, st, acc);
    } else {
      const RowState st = load_row<D, kSecond>(a, row, sub);
      add_entry<D, kHasVals>(a, p0, sub, acc);
      reduce_entries<D, kHasVals, 2>(a, i0 + 1, i1, sub, acc);
      apply_row<D, kSecond>(a, u, row, sub, st, acc);
    }
  }
}

// (4b) one wave per chunk of a long segment: the chunk is split evenly over the wave's lane
// groups, the groups' sums are combined with cross-lane shuffles, and the wave writes
// partials[c] = (s1[D], s2, gw, 0, 0) in double -- or, when the segment has no other chunk (33 .. 512
// entries, most long segments), updates the row at once
template <int D, bool kHasVals>
__global__ __launch_bounds__(kBlock) void k_long_partial(const BwdArgs a) {
  constexpr int G = D / 4;
  constexpr int NG = kWave / G;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t c = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  if (c >= a.ctrl->n_chunks) return;                          // uniform per wave
  const int g = lane / G, sub = lane % G;
  const int j = a.chunk_owner[c];
  const int u = a.long_seg[j];
  const int c_lo = a.seg_off[u] + (int)(c - a.long_c0[j]) * kChunk;
  const int c_hi = min(c_lo + kChunk, a.seg_off[u + 1]);
  const int per = (c_hi - c_lo + NG - 1) / NG;
  const int i0 = min(c_lo + g * per, c_hi), i1 = min(i0 + per, c_hi);
  Acc acc = acc_zero();
  reduce_entries<D, kHasVals, 4, true>(a, i0, i1, sub, acc);
#pragma unroll
  for (int m = G; m < kWave; m <<= 1) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc.v[k] += __shfl_xor(acc.v[k], m, kWave);
    acc.s2 += __shfl_xor(acc.s2, m, kWave);
    acc.gw += __shfl_xor(acc.gw, m, kWave);
  }
  if (g == 0) {
    if (a.seg_off[u + 1] - a.seg_off[u] <= kChunk) {
      // the segment is this one chunk: the wave holds its whole sum and updates the row itself
      const int row = a.uniq_rows[u];
      apply_row<D>(a, u, row, sub, load_row<D>(a, row, sub), acc);
    } else {
      double *p = a.partials + c * (D + 4);
      *reinterpret_cast<double2 *>(p + sub * 4) = make_double2(acc.v[0], acc.v[1]);
      *reinterpret_cast<double2 *>(p + sub * 4 + 2) = make_double2(acc.v[2], acc.v[3]);
      if (sub == 0) *reinterpret_cast<double2 *>(p + D) = make_double2(acc.s2, acc.gw);
    }
  }
}

// (4b') Segments of more than kMidFan chunks (rows that take a sizeable share of a skewed batch): one wave per
// group of kMidFan consecutive chunk partials adds them up in place, into the group's first slot, so that the
// per-segment combine below walks nch / kMidFan terms instead of nch.  Lane groups take the group's partials
// in strides and are combined by the same xor tree as in k_long_partial.
template <int D>
__global__ __launch_bounds__(kBlock) void k_long_mid(const BwdArgs a) {
  constexpr int G = D / 4;
  constexpr int NG = kWave / G;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t gi = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  if (gi >= a.ctrl->n_groups) return;                         // uniform per wave
  const int j = a.group_seg[gi];
  const int u = a.long_seg[j];
  const int nch = (a.seg_off[u + 1] - a.seg_off[u] + kChunk - 1) / kChunk;
  const int64_t c = a.group_c[gi];
  const int rel = (int)(c - a.long_c0[j]);
  const int cnt = min(kMidFan, nch - rel);
  const int g = lane / G, sub = lane % G;
  Acc acc = acc_zero();
  for (int k = g; k < cnt; k += NG) {
    const double *p = a.partials + (c + k) * (D + 4);
    const double2 lo = *reinterpret_cast<const double2 *>(p + sub * 4);
    const double2 hi = *reinterpret_cast<const double2 *>(p + sub * 4 + 2);
    const double2 t = *reinterpret_cast<const double2 *>(p + D);
    acc.v[0] += lo.x; acc.v[1] += lo.y; acc.v[2] += hi.x; acc.v[3] += hi.y;
    acc.s2 += t.x; acc.gw += t.y;                             // the same two values in every lane group's sub lanes
  }
#pragma unroll
  for (int m = G; m < kWave; m <<= 1) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc.v[k] += __shfl_xor(acc.v[k], m, kWave);
    acc.s2 += __shfl_xor(acc.s2, m, kWave);
    acc.gw += __shfl_xor(acc.gw, m, kWave);
  }
  // every partial of the group has been read by this wave's loads above (the shuffles waited for them)
  if (g == 0) {
    double *p = a.partials + c * (D + 4);
    *reinterpret_cast<double2 *>(p + sub * 4) = make_double2(acc.v[0], acc.v[1]);
    *reinterpret_cast<double2 *>(p + sub * 4 + 2) = make_double2(acc.v[2], acc.v[3]);
    if (sub == 0) *reinterpret_cast<double2 *>(p + D) = make_double2(acc.s2, acc.gw);
  }
}

// (4c) one workgroup per long segment of several chunks: lane groups stride over the chunk partials, an
// LDS tree combines the groups, group 0 updates the row
template <int D>
__global__ __launch_bounds__(kBlock) void k_long_final(const BwdArgs a) {
  constexpr int G = D / 4;
  constexpr int NGB = kBlock / G;           // lane groups per workgroup
  __shared__ double red[NGB][D + 4];
  const int grp = threadIdx.x / G, sub = threadIdx.x % G;
  const long long NM = a.ctrl->n_multi;      // one-chunk segments were updated by the wave that reduced their chunk
  for (int64_t jj = blockIdx.x; jj < NM; jj += gridDim.x) {
    const int j = a.multi_seg[jj];
    const int u = a.long_seg[j];
    const int nch = (a.seg_off[u + 1] - a.seg_off[u] + kChunk - 1) / kChunk;
    const double *p0 = a.partials + (int64_t)a.long_c0[j] * (D + 4);
    const int step = nch > kMidFan ? kMidFan : 1;      // k_long_mid left one sum per kMidFan chunks
    Acc acc = acc_zero();
    for (int c = grp * step; c < nch; c += NGB * step) {
      const double *p = p0 + (int64_t)c * (D + 4);
      const double2 lo = *reinterpret_cast<const double2 *>(p + sub * 4);
      const double2 hi = *reinterpret_cast<const double2 *>(p + sub * 4 + 2);
      acc.v[0] += lo.x; acc.v[1] += lo.y; acc.v[2] += hi.x; acc.v[3] += hi.y;
      if (sub == 0) {
        const double2 t = *reinterpret_cast<const double2 *>(p + D);
        acc.s2 += t.x; acc.gw += t.y;
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) red[grp][sub * 4 + k] = acc.v[k];
    if (sub == 0) { red[grp][D] = acc.s2; red[grp][D + 1] = acc.gw; }
    __syncthreads();
    for (int h = NGB / 2; h >= 1; h >>= 1) {
      if (grp < h) {
#pragma unroll
        for (int k = 0; k < 4; ++k) red[grp][sub * 4 + k] += red[grp + h][sub * 4 + k];
        if (sub == 0) { red[grp][D] += red[grp + h][D]; red[grp][D + 1] += red[grp + h][D + 1]; }
      }
      __syncthreads();
    }
    if (grp == 0) {
      Acc tot;
#pragma unroll
      for (int k = 0; k < 4; ++k) tot.v[k] = red[0][sub * 4 + k];
      tot.s2 = red[0][D];
      tot.gw = red[0][D + 1];
      const int row = a.uniq_rows[u];
      apply_row<D>(a, u, row, sub, load_row<D>(a, row, sub), tot);
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(kBlock) void k_export(const BwdArgs a) {
  const long long U = a.ctrl->n_uniq;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < U; u += stride) {
    const int row = a.uniq_rows[u];
    if (a.uniq_rows_out) a.uniq_rows_out[u] = row;
    if (a.uniq_keys_out) a.uniq_keys_out[u] = a.row_keys[row];
    if (a.counts_out) a.counts_out[u] = a.seg_off[u + 1] - a.seg_off[u];
  }
}

__global__ void k_set_i64(int64_t *p, int64_t v) { *p = v; }

inline unsigned blocks_for(int64_t threads, int64_t cap = 1ll << 30) {
  int64_t g = (threads + kBlock - 1) / kBlock;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (unsigned)g;
}

template <int D, bool kHasVals>
void launch_update(const BwdArgs &a, hipStream_t s) {
  constexpr int G = D / 4;
  const int64_t max_long = a.n / (kShortMax + 1) + 1;
  const int64_t max_chunks = a.n / kChunk + max_long + 1;
  {
    ProfScope ps(KID_SHORT_UPDATE, s);
    const bool second = a.opt_emb == DES_OPT_ADAM || a.opt_w == DES_OPT_ADAM || a.opt_w == DES_OPT_FTRL;
    const dim3 grid(blocks_for(a.n * G, kShortGrid)), block(kBlock);
    if (second) hipLaunchKernelGGL((k_short_update<D, kHasVals, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_short_update<D, kHasVals, false>), grid, block, 0, s, a);
  }
  {
    ProfScope ps(KID_LONG_PARTIAL, s);
    hipLaunchKernelGGL((k_long_partial<D, kHasVals>), dim3(blocks_for(max_chunks * kWave)), dim3(kBlock), 0, s, a);
  }
  {
    ProfScope ps(KID_LONG_FINAL, s);
    const int64_t max_multi = a.n / (kChunk + 1) + 1, max_groups = 3 * (a.n / ((int64_t)kChunk * kMidFan)) + 4;
    if (a.n > (int64_t)kChunk * kMidFan)          // a smaller batch cannot hold a segment of that many chunks
      hipLaunchKernelGGL(k_long_mid<D>, dim3(blocks_for(max_groups * kWave)), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL(k_long_final<D>, dim3((unsigned)(max_multi < 8192 ? max_multi : 8192)), dim3(kBlock), 0, s, a);
  }
}

template <int D>
void launch_update_v(const BwdArgs &a, hipStream_t s) {
  if (a.vals) launch_update<D, true>(a, s); else launch_update<D, false>(a, s);
}

struct Layout {
  size_t key_a, key_b, pay_a, pay_b, bag_of, seg_off, uniq_rows, first_pay, head_sums, long_seg, long_c0, multi_seg, group_seg,
      group_c, chunk_owner, partials, sort_scratch, total;
};

Layout layout_for(int D, int64_t n) {
  const size_t m = (size_t)(n > 0 ? n : 1);
  const size_t max_long = m / (kShortMax + 1) + 1, max_chunks = m / kChunk + max_long + 1;
  Layout L;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
  L.key_a = take(m * 4); L.key_b = take(m * 4); L.pay_a = take(m * 4); L.pay_b = take(m * 4);
  L.bag_of = take(m * 4);
  L.seg_off = take((m + 1) * 4); L.uniq_rows = take(m * 4); L.first_pay = take(m * 4);
  L.head_sums = take(((m + kHeadTile - 1) / kHeadTile + 1) * 4);
  L.long_seg = take(max_long * 4); L.long_c0 = take(max_long * 4);
  L.multi_seg = take((m / (kChunk + 1) + 1) * 4);
  const size_t max_groups = 3 * (m / ((size_t)kChunk * kMidFan)) + 4;   // sum of ceil(chunks / kMidFan) over those segments
  L.group_seg = take(max_groups * 4); L.group_c = take(max_groups * 4);
  L.chunk_owner = take(max_chunks * 4);
  L.partials = take(max_chunks * (size_t)(D + 4) * 8);
  L.sort_scratch = take(sort_scratch_bytes(n));
  L.total = o;
  return L;
}

int bits_for(uint64_t max_value) {
  int b = 1;
  while (b < 32 && (max_value >> b) != 0) ++b;
  return b;
}

// Row-sorting half of the backward pass: CSR -> (row, bag) pairs, sort by row, segment heads, split into
// short and long segments.  Needs the batch and its rows only, not the gradients.  Returns which sort
// buffer holds the sorted pairs.
int sort_stage(des_table *t, BwdArgs &a, const Layout &L, hipStream_t s) {
  char *ws = t->ws;
  const int64_t n = a.n;
  uint32_t *key_a = (uint32_t *)(ws + L.key_a), *pay_a = (uint32_t *)(ws + L.pay_a);
  {
    ProfScope ps(KID_EXPAND, s);
    const dim3 grid(blocks_for(a.nbags, 1 << 20)), block(kBlock);     // one workgroup per kBlock bags
    if (a.vals) hipLaunchKernelGGL(k_expand<true>, grid, block, 0, s, a, key_a, pay_a);
    else hipLaunchKernelGGL(k_expand<false>, grid, block, 0, s, a, key_a, pay_a);
  }
  SortBuffers sb{key_a, (uint32_t *)(ws + L.key_b), pay_a, (uint32_t *)(ws + L.pay_b)};
  const int side = radix_sort_u32_pairs(sb, n, bits_for((uint64_t)t->cfg.capacity_rows), ws + L.sort_scratch, s);
  a.key_sorted = (uint32_t *)(ws + (side ? L.key_b : L.key_a));
  a.pay_sorted = (uint32_t *)(ws + (side ? L.pay_b : L.pay_a));
  {
    ProfScope ps(KID_HEADS, s);
    const int64_t nb = (n + kHeadTile - 1) / kHeadTile;
    hipLaunchKernelGGL(k_heads_count, dim3((unsigned)nb), dim3(kBlock), 0, s, a);
    if (nb > kHeadsSelfPrefix) {                  // many tiles: one device-wide scan of the counts
      exclusive_scan_u32(a.head_sums, nb, a.head_sums + nb, ws + L.sort_scratch, s);
      hipLaunchKernelGGL(k_heads_finish, dim3(1), dim3(1), 0, s, a, (const uint32_t *)(a.head_sums + nb));
      hipLaunchKernelGGL(k_heads_write<false>, dim3((unsigned)nb), dim3(kBlock), 0, s, a);
    } else {
      hipLaunchKernelGGL(k_heads_write<true>, dim3((unsigned)nb), dim3(kBlock), 0, s, a);
    }
  }
  {
    ProfScope ps(KID_CLASSIFY, s);
    hipLaunchKernelGGL(k_classify, dim3((unsigned)((n + kHeadTile - 1) / kHeadTile)), dim3(kBlock), 0, s, a);
    const int64_t max_long = n / (kShortMax + 1) + 1;
    hipLaunchKernelGGL(k_chunk_owner, dim3((unsigned)(max_long < 65536 ? max_long : 65536)), dim3(kBlock), 0, s, a);
  }
  return side;
}

void batch_args(des_table *t, const des_batch_t *b, const int32_t *rows, const Layout &L, BwdArgs &a) {
  char *ws = t->ws;
  a = BwdArgs{};
  a.offsets = b->offsets; a.vals = b->vals; a.rows = rows;
  a.n = b->nnz; a.nbags = b->B * (int64_t)b->F; a.F = b->F;
  a.missing = (uint32_t)t->cfg.capacity_rows;
  a.emb = t->cfg.emb; a.w = t->cfg.w; a.acc_emb = t->cfg.acc_emb; a.acc_w = t->cfg.acc_w;
  a.acc2_emb = t->cfg.acc2_emb; a.acc2_w = t->cfg.acc2_w;
  a.row_keys = t->cfg.row_keys; a.ctrl = t->ctrl;
  a.bag_of = (int32_t *)(ws + L.bag_of);
  a.seg_off = (int32_t *)(ws + L.seg_off); a.uniq_rows = (int32_t *)(ws + L.uniq_rows);
  a.first_pay = (uint32_t *)(ws + L.first_pay);
  a.head_sums = (uint32_t *)(ws + L.head_sums);
  a.long_seg = (int32_t *)(ws + L.long_seg); a.long_c0 = (uint32_t *)(ws + L.long_c0);
  a.multi_seg = (int32_t *)(ws + L.multi_seg);
  a.group_seg = (int32_t *)(ws + L.group_seg); a.group_c = (uint32_t *)(ws + L.group_c);
  a.chunk_owner = (int32_t *)(ws + L.chunk_owner); a.partials = (double *)(ws + L.partials);
}

__global__ void k_report_n_uniq(const Ctrl *ctrl, int64_t *out) { *out = ctrl->n_uniq; }

}  // namespace

size_t backward_ws_bytes(int D, int64_t max_n) { return layout_for(D, max_n).total; }

des_status_t backward_prepare_launch(des_table *t, const des_batch_t *b, const int32_t *rows, hipStream_t s) {
  t->prep.valid = false;
  if (b->nnz == 0) return DES_OK;
  const Layout L = layout_for(t->cfg.dim, b->nnz);
  BwdArgs a;
  batch_args(t, b, rows, L, a);
  const int side = sort_stage(t, a, L, s);
  if (hipGetLastError() != hipSuccess) return DES_ERR_DEVICE;
  t->prep.valid = true;
  t->prep.offsets = b->offsets; t->prep.rows = rows; t->prep.vals = b->vals;
  t->prep.nnz = b->nnz; t->prep.B = b->B; t->prep.F = b->F; t->prep.side = side;
  return DES_OK;
}

des_status_t backward_launch(des_table *t, const des_batch_t *b, const int32_t *rows, const des_backward_io_t *io,
                             const des_optimizer_t *opt, hipStream_t s) {
  const int64_t n = b->nnz;
  const int D = t->cfg.dim;
  const bool prepared = t->prep.valid && t->prep.offsets == b->offsets && t->prep.rows == rows &&
                        t->prep.vals == b->vals && t->prep.nnz == n && t->prep.B == b->B && t->prep.F == b->F;
  t->prep.valid = false;                          // the update consumes the sorted form
  if (n == 0) {
    if (io->n_uniq_out) hipLaunchKernelGGL(k_set_i64, dim3(1), dim3(1), 0, s, io->n_uniq_out, (int64_t)0);
    return DES_OK;
  }
  const Layout L = layout_for(D, n);
  char *ws = t->ws;
  BwdArgs a;
  batch_args(t, b, rows, L, a);
  a.g_lr = io->g_lr; a.g_fm = io->g_fm; a.A_sum = io->A_sum; a.g_pool = io->g_pool;
  a.opt_emb = opt->opt_emb; a.opt_w = opt->opt_w; a.lr = opt->lr; a.eps = opt->eps;
  a.b1 = opt->beta1; a.b2 = opt->beta2;
  const double t_step = (double)(opt->step > 0 ? opt->step : 1);
  a.c1 = (float)(1.0 / (1.0 - pow((double)opt->beta1, t_step)));
  a.c2 = (float)(1.0 / (1.0 - pow((double)opt->beta2, t_step)));
  a.f_alpha = opt->ftrl_alpha; a.f_beta = opt->ftrl_beta; a.f_l1 = opt->ftrl_l1; a.f_l2 = opt->ftrl_l2;
  a.uniq_rows_out = io->uniq_rows_out; a.uniq_keys_out = io->uniq_keys_out; a.counts_out = io->counts_out;
  a.merged_out = io->merged_out; a.n_uniq_out = io->n_uniq_out;
  if (prepared) {
    a.key_sorted = (uint32_t *)(ws + (t->prep.side ? L.key_b : L.key_a));
    a.pay_sorted = (uint32_t *)(ws + (t->prep.side ? L.pay_b : L.pay_a));
    if (io->n_uniq_out) hipLaunchKernelGGL(k_report_n_uniq, dim3(1), dim3(1), 0, s, t->ctrl, io->n_uniq_out);
  } else {
    sort_stage(t, a, L, s);
  }
  switch (D) {
    case 4: launch_update_v<4>(a, s); break;
    case 8: launch_update_v<8>(a, s); break;
    case 16: launch_update_v<16>(a, s); break;
    case 32: launch_update_v<32>(a, s); break;
    case 64: launch_update_v<64>(a, s); break;
    case 128: launch_update_v<128>(a, s); break;
    case 256: launch_update_v<256>(a, s); break;
    default: return DES_ERR_INVALID_ARG;
  }
  if (io->uniq_rows_out || io->uniq_keys_out || io->counts_out) {
    ProfScope ps(KID_EXPORT, s);
    hipLaunchKernelGGL(k_export, dim3(blocks_for(n, 1 << 16)), dim3(kBlock), 0, s, a);
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // namespace des
