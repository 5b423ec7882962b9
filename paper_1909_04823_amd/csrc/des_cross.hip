// DCN cross layer under DES (Section 4, the paragraph on DCN; the layer itself is the cited DCN paper's
// x_{l+1} = x_0 (x_l^T w_l) + b_l + x_l with vectors of length d = F*D).
//
// w_l is cut along d like the fields it multiplies (column f*D+c goes with field f, shard f mod K,
// Section 5).  Sub-operator: the dot product over a shard's columns, one scalar per sample and shard
// (k_cross_partial).  Aggregation: the sum of the K scalars (des_aggregate_partials).  Remaining operator:
// y = x_0 * s + b + x_l, the same on every process (k_cross_apply).  Backward (Section 3.2.2): the gradient
// of the aggregated scalar, g_s[b] = <g_y[b], x_0[b]>, reaches every sub-operator unchanged.
//
// Everything here streams [B,d] arrays once; the kernels are bound by HBM.  Sums run in double in a fixed
// order (lane-strided partial sums combined by an xor tree; batch sums as per-slice partials added in slice
// order), so results do not depend on scheduling.
#include "des_internal.h"

namespace des {
namespace {

constexpr int kMaxCrossSlices = 256;   // row slices of the weight- and bias-gradient sums
constexpr int kCrossGridTarget = 2048; // workgroups the gradient kernel aims for

// P[s,b] = sum over the fields f = s, s+K, ... and the D columns of each of xl[b,f,:] * w[f,:].
// A group of G lanes per (sample, shard): lane t takes the float4s t, t+G, ... of the shard's columns.
template <int G>
__global__ __launch_bounds__(kBlock) void k_cross_partial(const float *__restrict__ xl, const float *__restrict__ w,
                                                           int64_t B, int F, int D4, int K, float *__restrict__ P) {
  const int64_t gid = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
  const int t = threadIdx.x % G;
  const int64_t stride = (int64_t)gridDim.x * kBlock / G;
  const int64_t row4 = (int64_t)F * D4;                       // float4s per sample
  for (int64_t item = gid; item < B * K; item += stride) {    // uniform per group; groups never straddle waves
    const int64_t b = item / K;
    const int s = (int)(item % K);
    const int nf = s < F ? (F - s + K - 1) / K : 0;           // fields of this shard
    const int m_end = nf * D4;
    double acc = 0.0;
#pragma unroll 4
    for (int m = t; m < m_end; m += G) {
      const int f = s + K * (m / D4);
      const int64_t q = (int64_t)f * D4 + (m % D4);
      const float4 xv = reinterpret_cast<const float4 *>(xl)[b * row4 + q];
      const float4 wv = reinterpret_cast<const float4 *>(w)[q];
      acc += ((double)xv.x * (double)wv.x + (double)xv.y * (double)wv.y) +
             ((double)xv.z * (double)wv.z + (double)xv.w * (double)wv.w);
    }
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
    if (t == 0) P[(int64_t)s * B + b] = (float)acc;
  }
}

// y[b,j] = x0[b,j] * s[b] + bias[j] + xl[b,j], four columns per thread.
__global__ __launch_bounds__(kBlock) void k_cross_apply(const float *__restrict__ x0, const float *__restrict__ xl,
                                                         const float *__restrict__ s, const float *__restrict__ bias,
                                                         int64_t B, int64_t d4, float *__restrict__ y) {
  const int64_t n4 = B * d4;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
#pragma unroll 2
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const int64_t b = i / d4, q = i % d4;
    const float4 a = reinterpret_cast<const float4 *>(x0)[i];
    const float4 x = reinterpret_cast<const float4 *>(xl)[i];
    const float4 c = reinterpret_cast<const float4 *>(bias)[q];
    const double sv = (double)s[b];
    float4 o;
    o.x = (float)((double)a.x * sv + (double)c.x + (double)x.x);
    o.y = (float)((double)a.y * sv + (double)c.y + (double)x.y);
    o.z = (float)((double)a.z * sv + (double)c.z + (double)x.z);
    o.w = (float)((double)a.w * sv + (double)c.w + (double)x.w);
    reinterpret_cast<float4 *>(y)[i] = o;
  }
}

// g_s[b] = <g_y[b,:], x0[b,:]>, one wave per sample.
__global__ __launch_bounds__(kBlock) void k_cross_gs(const float *__restrict__ g_y, const float *__restrict__ x0,
                                                      int64_t B, int64_t d4, float *__restrict__ g_s) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wstride = (int64_t)gridDim.x * (kBlock / kWave);
  for (int64_t b = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave; b < B; b += wstride) {
    double acc = 0.0;
#pragma unroll 4
    for (int64_t q = lane; q < d4; q += kWave) {
      const float4 g = reinterpret_cast<const float4 *>(g_y)[b * d4 + q];
      const float4 a = reinterpret_cast<const float4 *>(x0)[b * d4 + q];
      acc += ((double)g.x * (double)a.x + (double)g.y * (double)a.y) + ((double)g.z * (double)a.z + (double)g.w * (double)a.w);
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
    if (lane == 0) g_s[b] = (float)acc;
  }
}

// The elementwise gradients and the batch sums of one slice of rows.  grid (blocks of 256 float4 columns,
// slices); a thread owns four columns, walks the slice's rows and keeps its eight sums in double:
//   g_xl = g_y + g_s[b] * w,   g_x0 (+)= g_y * s[b],   dw += g_s[b] * xl,   db += g_y.
// partial[slice][0][:] = dw sums, partial[slice][1][:] = db sums.
// kFold: the layer's input is x0 itself, so g_xl is one more share of x0's gradient and is added into g_x0
// instead of being written.
template <bool kAccumulate, bool kFold>
__global__ __launch_bounds__(kBlock) void k_cross_grad(const float *__restrict__ xl, const float *__restrict__ w,
                                                        const float *__restrict__ s, const float *__restrict__ g_s,
                                                        const float *g_y, int64_t B, int64_t d4,
                                                        int64_t rows_per_slice, float *g_xl, float *g_x0,
                                                        double *__restrict__ partial) {
  const int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (q >= d4) return;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slice;
  const int64_t r1 = min(B, r0 + rows_per_slice);
  const float4 wv = reinterpret_cast<const float4 *>(w)[q];
  double dw[4] = {0.0, 0.0, 0.0, 0.0}, db[4] = {0.0, 0.0, 0.0, 0.0};
  constexpr int U = 4;
  for (int64_t r = r0; r < r1; r += U) {
    float4 g[U], x[U], old[U];
    float gs[U], sv[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const bool live = r + k < r1;
      const int64_t i = (live ? r + k : r) * d4 + q;
      g[k] = reinterpret_cast<const float4 *>(g_y)[i];
      x[k] = reinterpret_cast<const float4 *>(xl)[i];
      if (kAccumulate) old[k] = reinterpret_cast<const float4 *>(g_x0)[i];
      gs[k] = g_s[live ? r + k : r];
      sv[k] = s[live ? r + k : r];
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (r + k >= r1) break;
      const int64_t i = (r + k) * d4 + q;
      const double gd = (double)gs[k], sd = (double)sv[k];
      float4 o, z;
      o.x = (float)((double)g[k].x + gd * (double)wv.x);
      o.y = (float)((double)g[k].y + gd * (double)wv.y);
      o.z = (float)((double)g[k].z + gd * (double)wv.z);
      o.w = (float)((double)g[k].w + gd * (double)wv.w);
      const double f = kFold ? sd + 1.0 : sd;            // g*s + g when the input gradient is folded in
      z.x = (float)((kAccumulate ? (double)old[k].x : 0.0) + (double)g[k].x * f + (kFold ? gd * (double)wv.x : 0.0));
      z.y = (float)((kAccumulate ? (double)old[k].y : 0.0) + (double)g[k].y * f + (kFold ? gd * (double)wv.y : 0.0));
      z.z = (float)((kAccumulate ? (double)old[k].z : 0.0) + (double)g[k].z * f + (kFold ? gd * (double)wv.z : 0.0));
      z.w = (float)((kAccumulate ? (double)old[k].w : 0.0) + (double)g[k].w * f + (kFold ? gd * (double)wv.w : 0.0));
      if (!kFold) reinterpret_cast<float4 *>(g_xl)[i] = o;
      reinterpret_cast<float4 *>(g_x0)[i] = z;
      dw[0] += gd * (double)x[k].x; dw[1] += gd * (double)x[k].y; dw[2] += gd * (double)x[k].z; dw[3] += gd * (double)x[k].w;
      db[0] += (double)g[k].x; db[1] += (double)g[k].y; db[2] += (double)g[k].z; db[3] += (double)g[k].w;
    }
  }
  const int64_t d = d4 * 4;
  double *p = partial + (int64_t)blockIdx.y * 2 * d + q * 4;
#pragma unroll
  for (int k = 0; k < 4; ++k) { p[k] = dw[k]; p[d + k] = db[k]; }
}

// Backward of the sub-operator alone, for the gradient g_s[b] of the aggregated scalar:
//   g_xl[b,j] = g_s[b] * w[j],   dw[j] = sum_b g_s[b] * xl[b,j]   (partial[slice][0][:]; the db half stays unused).
__global__ __launch_bounds__(kBlock) void k_cross_subop_grad(const float *__restrict__ xl, const float *__restrict__ w,
                                                              const float *__restrict__ g_s, int64_t B, int64_t d4,
                                                              int64_t rows_per_slice, float *__restrict__ g_xl,
                                                              double *__restrict__ partial) {
  const int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (q >= d4) return;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slice;
  const int64_t r1 = min(B, r0 + rows_per_slice);
  const float4 wv = reinterpret_cast<const float4 *>(w)[q];
  double dw[4] = {0.0, 0.0, 0.0, 0.0};
  constexpr int U = 4;
  for (int64_t r = r0; r < r1; r += U) {
    float4 x[U];
    float gs[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int64_t rr = r + k < r1 ? r + k : r;
      x[k] = reinterpret_cast<const float4 *>(xl)[rr * d4 + q];
      gs[k] = g_s[rr];
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (r + k >= r1) break;
      const double gd = (double)gs[k];
      if (g_xl)
        reinterpret_cast<float4 *>(g_xl)[(r + k) * d4 + q] =
            make_float4((float)(gd * (double)wv.x), (float)(gd * (double)wv.y), (float)(gd * (double)wv.z),
                        (float)(gd * (double)wv.w));
      dw[0] += gd * (double)x[k].x; dw[1] += gd * (double)x[k].y; dw[2] += gd * (double)x[k].z; dw[3] += gd * (double)x[k].w;
    }
  }
  double *p = partial + (int64_t)blockIdx.y * 2 * (d4 * 4) + q * 4;
#pragma unroll
  for (int k = 0; k < 4; ++k) p[k] = dw[k];
}

// dw[j], db[j] = sums over the slices, in slice order (db null: only the dw half is summed).
__global__ __launch_bounds__(kBlock) void k_cross_final(const double *__restrict__ partial, int slices, int64_t d,
                                                         float *__restrict__ dw, float *__restrict__ db) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= (db ? 2 * d : d)) return;
  double a = 0.0;
  for (int sl = 0; sl < slices; ++sl) a += partial[(int64_t)sl * 2 * d + j];
  if (j < d) dw[j] = (float)a; else db[j - d] = (float)a;
}

inline unsigned blocks_for(int64_t threads, int64_t cap) {
  int64_t g = (threads + kBlock - 1) / kBlock;
  return (unsigned)(g < 1 ? 1 : (g > cap ? cap : g));
}

inline int cross_slices(int64_t B, int64_t d) {
  const int64_t col_blocks = (d / 4 + kBlock - 1) / kBlock;
  int64_t sl = kCrossGridTarget / (col_blocks > 0 ? col_blocks : 1);
  if (sl > kMaxCrossSlices) sl = kMaxCrossSlices;
  if (sl > B) sl = B;
  return (int)(sl < 1 ? 1 : sl);
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace
}  // namespace des

using namespace des;

extern "C" {

des_status_t des_cross_partial(const float *xl, const float *w, int64_t B, int32_t F, int32_t D, int32_t K, float *P,
                               void *stream) {
  if (B < 0 || F < 1 || D < 4 || (D & 3) || K < 1 || (int64_t)F * D > (1ll << 30)) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  if (!xl || !w || !P || !aligned16(xl) || !aligned16(w)) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int D4 = D / 4;
  int G = 1;
  while (G < 16 && G * 2 <= D4) G *= 2;
  const unsigned grid = blocks_for(B * K * G, 1 << 20);
  ProfScope ps(KID_CROSS_PARTIAL, s);
  switch (G) {
    case 1: hipLaunchKernelGGL(k_cross_partial<1>, dim3(grid), dim3(kBlock), 0, s, xl, w, B, F, D4, K, P); break;
    case 2: hipLaunchKernelGGL(k_cross_partial<2>, dim3(grid), dim3(kBlock), 0, s, xl, w, B, F, D4, K, P); break;
    case 4: hipLaunchKernelGGL(k_cross_partial<4>, dim3(grid), dim3(kBlock), 0, s, xl, w, B, F, D4, K, P); break;
    case 8: hipLaunchKernelGGL(k_cross_partial<8>, dim3(grid), dim3(kBlock), 0, s, xl, w, B, F, D4, K, P); break;
    default: hipLaunchKernelGGL(k_cross_partial<16>, dim3(grid), dim3(kBlock), 0, s, xl, w, B, F, D4, K, P); break;
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_cross_apply(const float *x0, const float *xl, const float *s_in, const float *bias, int64_t B,
                             int64_t d, float *y, void *stream) {
  if (B < 0 || d < 4 || (d & 3)) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  if (!x0 || !xl || !s_in || !bias || !y || !aligned16(x0) || !aligned16(xl) || !aligned16(bias) || !aligned16(y))
    return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_CROSS_APPLY, s);
  hipLaunchKernelGGL(k_cross_apply, dim3(blocks_for(B * (d / 4), 1 << 18)), dim3(kBlock), 0, s, x0, xl, s_in, bias, B,
                     d / 4, y);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_cross_backward_bytes(int64_t B, int64_t d, size_t *bytes) {
  if (!bytes || B < 0 || d < 4 || (d & 3)) return DES_ERR_INVALID_ARG;
  const int64_t rows = B > 0 ? B : 1;
  *bytes = align_up((size_t)rows * sizeof(float), 256) + (size_t)cross_slices(rows, d) * 2 * (size_t)d * sizeof(double);
  return DES_OK;
}

des_status_t des_cross_backward(const float *x0, const float *xl, const float *w, const float *s_in, const float *g_y,
                                int64_t B, int64_t d, float *g_xl, float *g_x0, int32_t accumulate_g_x0, float *dw,
                                float *db, void *workspace, size_t workspace_bytes, void *stream) {
  if (B < 0 || d < 4 || (d & 3)) return DES_ERR_INVALID_ARG;
  if (!dw || !db) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  size_t need = 0;
  des_cross_backward_bytes(B, d, &need);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return DES_ERR_WORKSPACE;
  float *g_s = (float *)workspace;
  double *partial = (double *)((char *)workspace + align_up((size_t)(B > 0 ? B : 1) * sizeof(float), 256));
  if (B == 0) {                                         // empty batch: the sums are zero
    ProfScope ps(KID_CROSS_GRAD, s);
    hipLaunchKernelGGL(k_cross_final, dim3(blocks_for(2 * d, 1 << 20)), dim3(kBlock), 0, s, partial, 0, d, dw, db);
    return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
  }
  if (!x0 || !xl || !w || !s_in || !g_y || !g_x0) return DES_ERR_INVALID_ARG;
  if (!aligned16(x0) || !aligned16(xl) || !aligned16(w) || !aligned16(g_y) || !aligned16(g_xl) || !aligned16(g_x0))
    return DES_ERR_INVALID_ARG;
  const int64_t d4 = d / 4;
  const int slices = cross_slices(B, d);
  const int64_t rows_per_slice = (B + slices - 1) / slices;
  ProfScope ps(KID_CROSS_GRAD, s);
  hipLaunchKernelGGL(k_cross_gs, dim3(blocks_for(B * kWave, 1 << 16)), dim3(kBlock), 0, s, g_y, x0, B, d4, g_s);
  const dim3 grid((unsigned)((d4 + kBlock - 1) / kBlock), (unsigned)slices);
#define DES_CROSS_GRAD(ACC, FOLD)                                                                                    \
  hipLaunchKernelGGL((k_cross_grad<ACC, FOLD>), grid, dim3(kBlock), 0, s, xl, w, s_in, g_s, g_y, B, d4, rows_per_slice, \
                     g_xl, g_x0, partial)
  if (g_xl) { if (accumulate_g_x0) DES_CROSS_GRAD(true, false); else DES_CROSS_GRAD(false, false); }
  else      { if (accumulate_g_x0) DES_CROSS_GRAD(true, true);  else DES_CROSS_GRAD(false, true); }
#undef DES_CROSS_GRAD
  hipLaunchKernelGGL(k_cross_final, dim3(blocks_for(2 * d, 1 << 20)), dim3(kBlock), 0, s, partial, slices, d, dw, db);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_cross_partial_backward(const float *xl, const float *w, const float *g_s, int64_t B, int64_t d,
                                        float *g_xl, float *dw, void *workspace, size_t workspace_bytes, void *stream) {
  if (B < 0 || d < 4 || (d & 3) || !dw) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  size_t need = 0;
  des_cross_backward_bytes(B, d, &need);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return DES_ERR_WORKSPACE;
  double *partial = (double *)((char *)workspace + align_up((size_t)(B > 0 ? B : 1) * sizeof(float), 256));
  ProfScope ps(KID_CROSS_GRAD, s);
  if (B == 0) {
    hipLaunchKernelGGL(k_cross_final, dim3(blocks_for(d, 1 << 20)), dim3(kBlock), 0, s, partial, 0, d, dw, (float *)nullptr);
    return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
  }
  if (!xl || !w || !g_s || !aligned16(xl) || !aligned16(w) || !aligned16(g_xl)) return DES_ERR_INVALID_ARG;
  const int64_t d4 = d / 4;
  const int slices = cross_slices(B, d);
  const int64_t rows_per_slice = (B + slices - 1) / slices;
  const dim3 grid((unsigned)((d4 + kBlock - 1) / kBlock), (unsigned)slices);
  hipLaunchKernelGGL(k_cross_subop_grad, grid, dim3(kBlock), 0, s, xl, w, g_s, B, d4, rows_per_slice, g_xl, partial);
  hipLaunchKernelGGL(k_cross_final, dim3(blocks_for(d, 1 << 20)), dim3(kBlock), 0, s, partial, slices, d, dw, (float *)nullptr);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // extern "C"
