// Device-wide exclusive scan and stable LSD radix sort for gfx950 (wave64).
//
// Both are plain multi-kernel primitives without inter-workgroup waiting: every kernel's
// workgroups are independent, so every wave reaches its exit whatever the dispatch order.
#include "des_internal.h"

namespace des {

namespace {

constexpr int kScanItems = 8;                       // items per thread in the scan kernels
constexpr int kScanTile = kBlock * kScanItems;
constexpr int kSortItems = 16;                      // items per thread in the sort kernels
constexpr int kSortTile = kBlock * kSortItems;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxDigitBits = 9;                    // widest radix digit of one pass
constexpr int kMaxRadix = 1 << kMaxDigitBits;

template <typename T>
__device__ inline T wave_inclusive_scan(T v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    T o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  return v;
}

// Exclusive prefix of v over the workgroup (thread order); total = sum over the workgroup.
template <typename T>
__device__ inline T block_exclusive_scan(T v, T *lds /*[kWavesPerBlock]*/, T &total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  T inc = wave_inclusive_scan(v);
  if (lane == kWave - 1) lds[wave] = inc;
  __syncthreads();
  T base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) {
    T x = lds[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + inc - v;
}

// The thread's kScanItems consecutive values in 16-byte accesses when they all exist (the arrays scanned here are
// the library's own, 256-byte aligned); values past n read as zero.
template <typename T>
__device__ inline void load_items(const T *__restrict__ data, int64_t base, int64_t n, T (&item)[kScanItems]) {
  constexpr int kPer = 16 / sizeof(T);
  static_assert(kScanItems % kPer == 0, "whole 16-byte accesses");
  if (base + kScanItems <= n) {
#pragma unroll
    for (int q = 0; q < kScanItems / kPer; ++q) {
      const uint4 raw = *reinterpret_cast<const uint4 *>(data + base + q * kPer);
      const T *t = reinterpret_cast<const T *>(&raw);
#pragma unroll
      for (int j = 0; j < kPer; ++j) item[q * kPer + j] = t[j];
    }
  } else {
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) item[i] = base + i < n ? data[base + i] : (T)0;
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_scan_reduce(const T *__restrict__ data, int64_t n, T *__restrict__ sums) {
  __shared__ T lds[kWavesPerBlock];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  T v = 0;
  T item[kScanItems];
  load_items(data, base, n, item);
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) v += item[i];
  T total;
  block_exclusive_scan(v, lds, total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// One workgroup scans the per-tile sums in place (exclusive) and stores the grand total.
template <typename T>
__global__ __launch_bounds__(kBlock) void k_scan_sums(T *__restrict__ sums, int64_t nb, T *__restrict__ total_out) {
  __shared__ T lds[kWavesPerBlock];
  T carry = 0;
  for (int64_t base = 0; base < nb; base += kBlock) {
    const int64_t i = base + threadIdx.x;
    T v = i < nb ? sums[i] : (T)0;
    T total;
    T ex = block_exclusive_scan(v, lds, total);
    if (i < nb) sums[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0 && total_out) *total_out = carry;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_scan_apply(T *__restrict__ data, int64_t n, const T *__restrict__ sums) {
  __shared__ T lds[kWavesPerBlock];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  T item[kScanItems];
  T v = 0;
  load_items(data, base, n, item);
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) v += item[i];
  T total;
  T run = sums[blockIdx.x] + block_exclusive_scan(v, lds, total);
  if (base + kScanItems <= n) {
    constexpr int kPer = 16 / sizeof(T);
#pragma unroll
    for (int q = 0; q < kScanItems / kPer; ++q) {
      uint4 raw;
      T *t = reinterpret_cast<T *>(&raw);
#pragma unroll
      for (int j = 0; j < kPer; ++j) { t[j] = run; run += item[q * kPer + j]; }
      *reinterpret_cast<uint4 *>(data + base + q * kPer) = raw;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
      if (base + i < n) data[base + i] = run;
      run += item[i];
    }
  }
}

template <typename T>
void exclusive_scan(T *data, int64_t n, T *total_out, void *scratch, hipStream_t s) {
  if (n <= 0) return;
  const int64_t nb = (n + kScanTile - 1) / kScanTile;
  T *sums = (T *)scratch;
  hipLaunchKernelGGL(k_scan_reduce<T>, dim3((unsigned)nb), dim3(kBlock), 0, s, data, n, sums);
  hipLaunchKernelGGL(k_scan_sums<T>, dim3(1), dim3(kBlock), 0, s, sums, nb, total_out);
  hipLaunchKernelGGL(k_scan_apply<T>, dim3((unsigned)nb), dim3(kBlock), 0, s, data, n, sums);
}

// ---------------------------------------------------------------------------------------
// Radix sort.  One workgroup owns a tile of kSortTile consecutive items; wave w owns the w-th
// quarter of the tile and walks it in rounds of 64, so "wave, round, lane" is item order.

// Digit counts of kHistTiles consecutive tiles per workgroup: all keys of the workgroup are requested before the
// first is counted, and the counts of one digit leave as one contiguous run of kHistTiles values.  Pays once
// there are enough tiles to fill the chip with such workgroups (0.84 -> 0.74 ms over four passes of 1.05e8
// keys; a loss at 8e6 keys, which keep one tile per workgroup).
constexpr int kHistManyTiles = 8192;
template <typename KeyT, int kHistTiles>
__global__ __launch_bounds__(kBlock) void k_radix_hist(const KeyT *__restrict__ keys, int64_t n,
                                                        const long long *__restrict__ n_dev, int shift, int bits,
                                                        uint32_t *__restrict__ hist, int nblocks) {
  __shared__ uint32_t cnt[kHistTiles][kMaxRadix];
  const int64_t n_eff = n_dev ? (int64_t)min((long long)n, *n_dev) : n;
  const int radix = 1 << bits;
  const int blk0 = blockIdx.x * kHistTiles;
  const uint32_t mask = (1u << bits) - 1u;
  KeyT key[kHistTiles][kSortItems];
  // the keys are requested before the counters are cleared, so that the barrier is passed while they travel
#pragma unroll
  for (int j = 0; j < kHistTiles; ++j) {
    const int64_t base = (int64_t)(blk0 + j) * kSortTile;
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
      const int64_t idx = base + (int64_t)i * kBlock + threadIdx.x;
      key[j][i] = idx < n_eff ? keys[idx] : (KeyT)0;
    }
  }
  for (int i = threadIdx.x; i < kHistTiles * kMaxRadix; i += kBlock) (&cnt[0][0])[i] = 0;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kHistTiles; ++j) {
    const int64_t base = (int64_t)(blk0 + j) * kSortTile;
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
      const int64_t idx = base + (int64_t)i * kBlock + threadIdx.x;
      if (idx < n_eff) atomicAdd(&cnt[j][(uint32_t)(key[j][i] >> shift) & mask], 1u);
    }
  }
  __syncthreads();
  const int tiles = min(kHistTiles, nblocks - blk0);
  for (int i = threadIdx.x; i < radix * kHistTiles; i += kBlock) {
    const int d = i / kHistTiles, j = i % kHistTiles;
    if (j < tiles) hist[(size_t)d * nblocks + blk0 + j] = cnt[j][d];
  }
}

// Scatter of one pass.  The tile is first put in digit order inside LDS (rank of an item = items of
// smaller digits in the tile + items of its digit in earlier waves + earlier rounds of its wave +
// lower lanes of its round, which is item order, so the pass is stable); then consecutive threads
// write consecutive sorted items, so the items of one digit leave as one contiguous run instead of
// one 4-byte store per lane.
template <typename KeyT, bool kHasPayload>
__global__ __launch_bounds__(kBlock) void k_radix_scatter(const KeyT *__restrict__ keys_in,
                                                           const uint32_t *__restrict__ pay_in,
                                                           KeyT *__restrict__ keys_out, uint32_t *__restrict__ pay_out,
                                                           int64_t n, const long long *__restrict__ n_dev, int shift,
                                                           int bits, const uint32_t *__restrict__ offsets, int nblocks) {
  __shared__ uint32_t cnt[kWavesPerBlock][kMaxRadix];   // per wave and digit: count, then start inside the digit's run
  __shared__ uint32_t dig_base[kMaxRadix];              // first sorted index of the digit inside the tile
  __shared__ uint32_t gofs[kMaxRadix];                  // where the tile's run of the digit starts in the output
  __shared__ uint32_t scan_lds[kWavesPerBlock];
  __shared__ KeyT skey[kSortTile];                      // the sorted keys; afterwards reused for the payloads
  static_assert(sizeof(KeyT) >= sizeof(uint32_t), "payloads are staged in the key buffer");
  const int64_t n_eff = n_dev ? (int64_t)min((long long)n, *n_dev) : n;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t tile = (int64_t)blockIdx.x * kSortTile;
  if (tile >= n_eff) return;                         // uniform per workgroup
  const int tile_n = (int)min((int64_t)kSortTile, n_eff - tile);
  const int radix = 1 << bits;
  const uint32_t mask = (1u << bits) - 1u;
  const unsigned long long lane_lt = (1ull << lane) - 1ull;
  const int64_t wbase = tile + (int64_t)wave * (kSortItems * kWave);
  KeyT key[kSortItems];
  uint32_t pay[kSortItems];
  uint32_t rank[kSortItems];
  // the tile's items are requested first, so that their latency overlaps the fetch of the run offsets
#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const int64_t idx = wbase + r * kWave + lane;
    const bool live = idx < n_eff;
    key[r] = live ? keys_in[idx] : (KeyT)0;
    if (kHasPayload) pay[r] = live ? pay_in[idx] : 0u;
  }
  for (int d = threadIdx.x; d < radix; d += kBlock) {
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) cnt[w][d] = 0;
    gofs[d] = offsets[(size_t)d * nblocks + blockIdx.x];
  }
  __syncthreads();

#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const int64_t idx = wbase + r * kWave + lane;
    const bool live = idx < n_eff;
    const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
    // lanes of this wave holding the same digit
    unsigned long long peers = __ballot(live);
    for (int bit = 0; bit < bits; ++bit) {
      const bool one = (d >> bit) & 1u;
      const unsigned long long bal = __ballot(one);
      peers &= one ? bal : ~bal;
    }
    const uint32_t before = (uint32_t)__popcll(peers & lane_lt);
    uint32_t prev = 0;
    if (live) prev = cnt[wave][d];
    // every lane has read its counter before the group leaders below overwrite them:
    // the wave executes the load and the store as two instructions in program order
    __builtin_amdgcn_wave_barrier();
    if (live && before == 0) cnt[wave][d] = prev + (uint32_t)__popcll(peers);
    __builtin_amdgcn_wave_barrier();
    rank[r] = prev + before;
  }
  __syncthreads();
  // per digit: exclusive prefix over the waves; then exclusive prefix of the digit totals over the digits
  // (two digits per thread: kMaxRadix <= 2 * kBlock)
  static_assert(kMaxRadix <= 2 * kBlock, "two digits per thread");
  uint32_t tot[2] = {0u, 0u};
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int d = threadIdx.x * 2 + j;
    if (d < radix) {
      uint32_t run = 0;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        const uint32_t c = cnt[w][d];
        cnt[w][d] = run;
        run += c;
      }
      tot[j] = run;
    }
  }
  uint32_t total;
  const uint32_t ex = block_exclusive_scan<uint32_t>(tot[0] + tot[1], scan_lds, total);
  if (threadIdx.x * 2 < radix) dig_base[threadIdx.x * 2] = ex;
  if (threadIdx.x * 2 + 1 < radix) dig_base[threadIdx.x * 2 + 1] = ex + tot[0];
  __syncthreads();
  uint32_t li[kSortItems];
#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const int64_t idx = wbase + r * kWave + lane;
    li[r] = 0;
    if (idx < n_eff) {
      const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
      li[r] = dig_base[d] + cnt[wave][d] + rank[r];
      skey[li[r]] = key[r];
    }
  }
  __syncthreads();
  // keys out; every thread remembers where its sorted items went, for the payloads that follow
  constexpr int kOut = kSortTile / kBlock;
  uint32_t pos[kOut];
#pragma unroll
  for (int j = 0; j < kOut; ++j) {
    const int i = threadIdx.x + j * kBlock;
    pos[j] = 0;
    if (i < tile_n) {
      const KeyT k = skey[i];
      const uint32_t d = (uint32_t)(k >> shift) & mask;
      pos[j] = gofs[d] + ((uint32_t)i - dig_base[d]);
      keys_out[pos[j]] = k;
    }
  }
  if (kHasPayload) {
    uint32_t *spay = reinterpret_cast<uint32_t *>(skey);
    __syncthreads();                                   // all keys read before the buffer is overwritten
#pragma unroll
    for (int r = 0; r < kSortItems; ++r)
      if (wbase + r * kWave + lane < n_eff) spay[li[r]] = pay[r];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kOut; ++j) {
      const int i = threadIdx.x + j * kBlock;
      if (i < tile_n) pay_out[pos[j]] = spay[i];
    }
  }
}

inline int64_t sort_blocks(int64_t n) { return (n + kSortTile - 1) / kSortTile; }

template <typename KeyT, bool kHasPayload>
int radix_sort(SortBuffers buf, int64_t n, const long long *n_dev, int bits, void *scratch, hipStream_t s,
               int kid_hist, int kid_scan, int kid_scatter) {
  if (n <= 0 || bits <= 0) return 0;
  const int nblocks = (int)sort_blocks(n);
  uint32_t *hist = (uint32_t *)scratch;
  void *scan_scratch = (char *)scratch + align_up((size_t)kMaxRadix * nblocks * sizeof(uint32_t), 256);
  const int npass = (bits + kMaxDigitBits - 1) / kMaxDigitBits;
  const int per = (bits + npass - 1) / npass;
  KeyT *kin = (KeyT *)buf.keys_a, *kout = (KeyT *)buf.keys_b;
  uint32_t *pin = buf.pay_a, *pout = buf.pay_b;
  int side = 0;
  for (int p = 0; p < npass; ++p) {
    const int shift = p * per;
    const int b = (bits - shift) < per ? (bits - shift) : per;
    {
      ProfScope ps(kid_hist, s);
      if (nblocks >= kHistManyTiles)
        hipLaunchKernelGGL((k_radix_hist<KeyT, 4>), dim3((nblocks + 3) / 4), dim3(kBlock), 0, s, kin, n, n_dev, shift, b, hist,
                           nblocks);
      else
        hipLaunchKernelGGL((k_radix_hist<KeyT, 1>), dim3(nblocks), dim3(kBlock), 0, s, kin, n, n_dev, shift, b, hist, nblocks);
    }
    {
      ProfScope ps(kid_scan, s);
      exclusive_scan<uint32_t>(hist, (int64_t)(1 << b) * nblocks, nullptr, scan_scratch, s);
    }
    {
      ProfScope ps(kid_scatter, s);
      hipLaunchKernelGGL((k_radix_scatter<KeyT, kHasPayload>), dim3(nblocks), dim3(kBlock), 0, s, kin, pin, kout, pout,
                         n, n_dev, shift, b, hist, nblocks);
    }
    KeyT *tk = kin; kin = kout; kout = tk;
    uint32_t *tp = pin; pin = pout; pout = tp;
    side ^= 1;
  }
  return side;
}

}  // namespace

size_t scan_scratch_bytes(int64_t n) {
  const int64_t nb = (n + kScanTile - 1) / kScanTile;
  return align_up((size_t)(nb + 1) * sizeof(unsigned long long), 256);
}

size_t sort_scratch_bytes(int64_t n) {
  const int64_t nblocks = sort_blocks(n > 0 ? n : 1);
  return align_up((size_t)kMaxRadix * nblocks * sizeof(uint32_t), 256) + scan_scratch_bytes(kMaxRadix * nblocks);
}

void exclusive_scan_u32(uint32_t *data, int64_t n, uint32_t *total_out, void *scratch, hipStream_t s) {
  exclusive_scan<uint32_t>(data, n, total_out, scratch, s);
}

void exclusive_scan_u64(unsigned long long *data, int64_t n, unsigned long long *total_out, void *scratch,
                        hipStream_t s) {
  exclusive_scan<unsigned long long>(data, n, total_out, scratch, s);
}

int radix_sort_u32_pairs(SortBuffers buf, int64_t n, int bits, void *scratch, hipStream_t s) {
  return radix_sort<uint32_t, true>(buf, n, nullptr, bits, scratch, s, KID_SORT_HIST, KID_SORT_SCAN, KID_SORT_SCATTER);
}

}  // namespace des
