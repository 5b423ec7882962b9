// First fully-connected layer of the DNN tower under DES (Section 4.3, Eq. dnn_bmm / dnn_des).
//
// The concatenated pooled embeddings V [B, F*D] and the layer weights W [F*D, H] are both cut
// along the field dimension; shard s owns the fields f with f mod K == s and its sub-operator is
// M1(V_s, W_s) = V_s^T W_s, a [B,H] partial that the aggregation sums over the shards.  Backward:
// the gradient dY of the aggregate reaches every shard unchanged (Section 3.2.2), each shard
// forms the gradient of its own field columns (dY W_s^T, which is the upstream gradient of the
// pooled embeddings) and of its own weight rows (V_s dY).
//
// This is the one dense contraction of the path, so it runs on the matrix cores: fp32 MFMA
// (v_mfma_f32_32x32x2f32, fp32 accumulate), 128x128 output tile per workgroup, four waves in a
// 2x2 arrangement of 64x64, 16-deep k tiles staged in LDS k-major so both operands are read with
// conflict-free 32-lane rows, next tile prefetched into registers during the MFMAs.
//
// One kernel serves the three products through operand strides and a sliced k range:
//   forward   C_s[B,H]   = sum over the shard's fields of pool[:, f, :] x W[f*D:(f+1)*D, :]
//   g_pool    C[B,F*D]   = dY x W^T
//   dW        C_z[F*D,H] = pool[z-th slice of samples]^T x dY[slice]   (split over samples, summed after)
#include "des_internal.h"

namespace des {
namespace {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDA = BM + 4, LDB = BN + 4;    // LDS row pitches (floats)
constexpr int kFlushTiles = 8;               // 128 products per first-level run
constexpr long long kTwoLevelDepth = 1024;

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
  const float *A, *B;
  float *C;
  long long a_rs, a_cs, b_rs, b_cs;   // element strides: A(m,k) = A[m*a_rs + k*a_cs], B(k,n) = B[k*b_rs + n*b_cs]
  int M, N;
  long long c_rs;                     // C(m,n) = C[slice*c_slice + m*c_rs + n]
  long long c_slice;
  // k range of slice z: blocks [base, base + blk_len) for base = k_begin + z*k_shift, += blk_stride, below k_limit
  long long k_begin, k_shift, blk_len, blk_stride, k_limit;
};

__device__ inline float4 ld4g(const float *p) { return *reinterpret_cast<const float4 *>(p); }

// Loads the part of a 128 x 16 operand tile this thread stages: two float4 (eight floats).
// kKContig: the k index is the contiguous one in memory (float4 along k), else the m/n index is.
template <bool kKContig>
__device__ inline void load_tile(const float *__restrict__ P, long long rs, long long cs, int mn0, int MN,
                                 long long k0, long long kend, float4 (&r)[2]) {
  // whole tile inside the operand (the same answer for every thread): plain 16-byte loads, no per-element guards
  if (mn0 + BM <= MN && k0 + BK <= kend) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = threadIdx.x + i * kBlock;
      r[i] = kKContig ? ld4g(P + (long long)(mn0 + idx / 4) * rs + k0 + (idx % 4) * 4)
                      : ld4g(P + (k0 + idx / 32) * cs + mn0 + (idx % 32) * 4);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = threadIdx.x + i * kBlock;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (kKContig) {
      const int mn = mn0 + idx / 4;
      const long long k = k0 + (idx % 4) * 4;
      if (mn < MN) {
        const float *p = P + (long long)mn * rs + k;            // cs == 1
        if (k + 3 < kend) { const float4 t = ld4g(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
        else { for (int j = 0; j < 4; ++j) if (k + j < kend) v[j] = p[j]; }
      }
    } else {
      const long long k = k0 + idx / 32;
      const int mn = mn0 + (idx % 32) * 4;
      if (k < kend) {
        const float *p = P + k * cs + mn;                         // rs == 1
        if (mn + 3 < MN) { const float4 t = ld4g(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
        else { for (int j = 0; j < 4; ++j) if (mn + j < MN) v[j] = p[j]; }
      }
    }
    r[i] = make_float4(v[0], v[1], v[2], v[3]);
  }
}

// Writes the staged registers into the k-major LDS tile T[BK][LD].
template <bool kKContig, int LD>
__device__ inline void store_tile(float *__restrict__ T, const float4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = threadIdx.x + i * kBlock;
    if (kKContig) {
      const int mn = idx / 4, k = (idx % 4) * 4;
      T[(k + 0) * LD + mn] = r[i].x;
      T[(k + 1) * LD + mn] = r[i].y;
      T[(k + 2) * LD + mn] = r[i].z;
      T[(k + 3) * LD + mn] = r[i].w;
    } else {
      const int k = idx / 32, mn = (idx % 32) * 4;
      *reinterpret_cast<float4 *>(&T[k * LD + mn]) = r[i];
    }
  }
}

template <bool kAKContig, bool kBKContig, bool kTwoLevel>
__global__ __launch_bounds__(kBlock) void k_gemm(const GemmArgs g) {
  __shared__ __align__(16) float As[BK * LDA];
  __shared__ __align__(16) float Bs[BK * LDB];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int z = blockIdx.z;
  // kTwoLevel (long contractions; the weight gradient sums over the whole batch): two-level fp32
  // summation.  The matrix cores accumulate runs of kFlushTiles*BK products from zero and each run is
  // then added into `total`, so small products are never added to a large running sum.  Short
  // contractions keep the single accumulator and the registers that saves.
  f32x16 acc[2][2], total[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; total[i][j][r] = 0.f; }
  int run = 0;

  const int lrow = lane & 31, lk = lane >> 5;     // MFMA operand: row/column within the 32-block, k within the pair
  for (long long base = g.k_begin + (long long)z * g.k_shift; base < g.k_limit; base += g.blk_stride) {
    const long long kend = min(base + g.blk_len, g.k_limit);
    float4 ra[2], rb[2];
    load_tile<kAKContig>(g.A, g.a_rs, g.a_cs, m0, g.M, base, kend, ra);
    load_tile<kBKContig>(g.B, g.b_cs, g.b_rs, n0, g.N, base, kend, rb);   // for B the "row" index is n
    for (long long k0 = base; k0 < kend; k0 += BK) {
      __syncthreads();                              // previous tile fully consumed
      store_tile<kAKContig, LDA>(As, ra);
      store_tile<kBKContig, LDB>(Bs, rb);
      __syncthreads();
      if (k0 + BK < kend) {                         // prefetch the next tile while this one is multiplied
        load_tile<kAKContig>(g.A, g.a_rs, g.a_cs, m0, g.M, k0 + BK, kend, ra);
        load_tile<kBKContig>(g.B, g.b_cs, g.b_rs, n0, g.N, k0 + BK, kend, rb);
      }
      // operands of step kk+2 are read from LDS before the MFMAs of step kk are issued
      float a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = As[lk * LDA + wm * 64 + i * 32 + lrow];
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = Bs[lk * LDB + wn * 64 + j * 32 + lrow];
#pragma unroll
      for (int kk = 0; kk < BK; kk += 2) {
        float an[2] = {0.f, 0.f}, bn[2] = {0.f, 0.f};
        if (kk + 2 < BK) {
#pragma unroll
          for (int i = 0; i < 2; ++i) an[i] = As[(kk + 2 + lk) * LDA + wm * 64 + i * 32 + lrow];
#pragma unroll
          for (int j = 0; j < 2; ++j) bn[j] = Bs[(kk + 2 + lk) * LDB + wn * 64 + j * 32 + lrow];
        }
        __builtin_amdgcn_sched_barrier(0);       // keep the reads above the MFMAs: the scheduler would sink them to their use
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i) { a[i] = an[i]; b[i] = bn[i]; }
      }
      if (kTwoLevel && ++run == kFlushTiles) {
        run = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            total[i][j] += acc[i][j];
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
          }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) total[i][j] += acc[i][j];
  // accumulator element r of a 32x32 block sits at row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
  float *C = g.C + (long long)z * g.c_slice;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + lrow;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 64 + i * 32 + (r >> 2) * 8 + lk * 4 + (r & 3);
        if (row < g.M && col < g.N) C[(long long)row * g.c_rs + col] = total[i][j][r];
      }
    }
}

// `depth`: products summed per output element of one slice; above kTwoLevelDepth the two-level kernel runs.
template <bool kAKContig, bool kBKContig>
des_status_t launch(const GemmArgs &g, int slices, long long depth, int kid, hipStream_t s) {
  const dim3 grid((unsigned)((g.N + BN - 1) / BN), (unsigned)((g.M + BM - 1) / BM), (unsigned)slices);
  ProfScope ps(kid, s);
  if (depth > kTwoLevelDepth)
    hipLaunchKernelGGL((k_gemm<kAKContig, kBKContig, true>), grid, dim3(kBlock), 0, s, g);
  else
    hipLaunchKernelGGL((k_gemm<kAKContig, kBKContig, false>), grid, dim3(kBlock), 0, s, g);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

bool al16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace
}  // namespace des

using namespace des;

extern "C" {

des_status_t des_dnn_partial_forward(const float *pool, const float *W, int64_t B, int32_t F, int32_t D, int32_t H,
                                     int32_t K, float *Y_partial, void *stream) {
  if (B < 0 || F < 1 || D < 4 || (D & 3) || H < 4 || (H & 3) || K < 1 || K > 256) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  if (!pool || !W || !Y_partial) return DES_ERR_INVALID_ARG;
  if (B >= 2147483647ll || (int64_t)F * D >= 2147483647ll || !al16(pool) || !al16(W) || !al16(Y_partial))
    return DES_ERR_INVALID_ARG;
  GemmArgs g;
  g.A = pool; g.a_rs = (long long)F * D; g.a_cs = 1;
  g.B = W; g.b_rs = H; g.b_cs = 1;
  g.C = Y_partial; g.M = (int)B; g.N = H; g.c_rs = H; g.c_slice = (long long)B * H;
  // shard s: fields s, s+K, ... = k blocks of length D starting at s*D, K*D apart
  g.k_begin = 0; g.k_shift = D; g.blk_len = D; g.blk_stride = (long long)K * D; g.k_limit = (long long)F * D;
  return launch<true, false>(g, K, (long long)((F + K - 1) / K) * D, KID_DNN_FORWARD, (hipStream_t)stream);
}

des_status_t des_dnn_backward_bytes(int64_t B, int32_t F, int32_t D, int32_t H, size_t *workspace_bytes) {
  if (!workspace_bytes || B < 0 || F < 1 || D < 4 || H < 4) return DES_ERR_INVALID_ARG;
  *workspace_bytes = (size_t)16 * F * D * H * sizeof(float);    // up to 16 sample slices of dW
  return DES_OK;
}

des_status_t des_dnn_backward(const float *pool, const float *W, const float *dY, int64_t B, int32_t F, int32_t D,
                              int32_t H, float *g_pool, float *dW, void *workspace, size_t workspace_bytes,
                              void *stream) {
  if (B < 0 || F < 1 || D < 4 || (D & 3) || H < 4 || (H & 3)) return DES_ERR_INVALID_ARG;
  if (!g_pool && !dW) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;            // g_pool is empty; dW would be all zero and is left untouched
  if (!pool || !W || !dY) return DES_ERR_INVALID_ARG;
  if (B >= 2147483647ll || (int64_t)F * D >= 2147483647ll || !al16(pool) || !al16(W) || !al16(dY) ||
      (g_pool && !al16(g_pool)) || (dW && !al16(dW)) || !al16(workspace))
    return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const long long FD = (long long)F * D;
  if (g_pool) {                                   // g_pool[B, F*D] = dY[B,H] x W^T: B(k=h, n=j) = W[j*H + h]
    GemmArgs g;
    g.A = dY; g.a_rs = H; g.a_cs = 1;
    g.B = W; g.b_rs = 1; g.b_cs = H;
    g.C = g_pool; g.M = (int)B; g.N = (int)FD; g.c_rs = FD; g.c_slice = 0;
    g.k_begin = 0; g.k_shift = 0; g.blk_len = H; g.blk_stride = (1ll << 40); g.k_limit = H;
    des_status_t st = launch<true, true>(g, 1, H, KID_DNN_GPOOL, s);
    if (st != DES_OK) return st;
  }
  if (dW) {                                       // dW[F*D, H] = pool^T x dY, split over slices of samples
    const long long tiles = ((FD + BM - 1) / BM) * ((H + BN - 1) / BN);
    // Slices of samples: enough workgroups to fill the chip, chosen so that the last round of resident
    // workgroups (two per CU for the two-level kernel, 256 CUs) is as full as possible; fewer slices win ties
    // (less partial-sum traffic).  At most 16 slices, at least BK samples each.
    int Z = 1;
    {
      const long long per_round = 2 * 256;
      double best = -1.0;
      for (int z = 1; z <= 16 && (long long)z * BK <= (B > BK ? B : BK); ++z) {
        const long long blocks = tiles * z, rounds = (blocks + per_round - 1) / per_round;
        const double fill = (double)blocks / (double)(rounds * per_round);
        if (fill > best + 0.02) { best = fill; Z = z; }
      }
    }
    long long chunk = ((B + Z - 1) / Z + BK - 1) / BK * BK;
    Z = (int)((B + chunk - 1) / chunk);
    if (Z > 1 && (!workspace || workspace_bytes < (size_t)Z * FD * H * sizeof(float))) return DES_ERR_WORKSPACE;
    GemmArgs g;
    g.A = pool; g.a_rs = 1; g.a_cs = FD;          // A(m=j, k=b) = pool[b*FD + j]
    g.B = dY; g.b_rs = H; g.b_cs = 1;
    g.C = Z > 1 ? (float *)workspace : dW; g.M = (int)FD; g.N = H; g.c_rs = H; g.c_slice = FD * H;
    g.k_begin = 0; g.k_shift = chunk; g.blk_len = chunk; g.blk_stride = (1ll << 40); g.k_limit = B;
    des_status_t st = launch<false, false>(g, Z, chunk, KID_DNN_DW, s);
    if (st != DES_OK) return st;
    if (Z > 1) return des_aggregate_partials((const float *)workspace, Z, FD * H, dW, stream);
  }
  return DES_OK;
}

}  // extern "C"
