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
#pragma unroll 8
  for (int sl = 0; sl < slices; ++sl) a += partial[(int64_t)sl * 2 * d + j];
  if (j < d) dw[j] = (float)a; else db[j - d] = (float)a;
}

// ---- the whole cross network at once -----------------------------------------------------------
// Every cross layer adds a multiple of x_0 and a bias to its input, so by induction
//   x_l[b,:] = gamma_l[b] * x_0[b,:] + c_l[:],   gamma_0 = 1, gamma_{l+1} = gamma_l + s_l,   c_l = b_0 + ... + b_{l-1},
//   s_l[b]   = <x_l[b], w_l> = gamma_l[b] * t_l[b] + <c_l, w_l>,          t_k[b] = <x_0[b], u_k>,
// with u_0..u_{n-1} the layers' weights and u_n the output unit's weights on x_n.  The only contact with the
// [B,d] data is the m = n+1 dot products t_k, all of them sub-operators on x_0 (cut along d, one scalar per
// sample, shard and vector, summed by the aggregation): one pass over x_0 instead of four per layer, and under
// DES one exchange of m scalars per sample for the whole network.  The rest of the forward pass is a
// recurrence on scalars.  Backward, for the gradient g[b] of the logit term <x_n, u_n>:
//   g_s_l = g t_n + sum_{l'>l} g_s_l' t_l'                    (gradient of s_l; every g_{x_l} is a combination of the u_k)
//   beta_l = g_s_l gamma_l (l < n),  beta_n = g gamma_n
//   g_x0[b,:] = sum_k beta_k[b] u_k                           (rank m)
//   du_k = sum_b beta_k[b] x_0[b,:] + c_k G_k,   G_l = sum_b g_s_l,  G_n = sum_b g
//   db_l = u_n G_n + sum_{l'>l} u_l' G_l'
// which is a second pass over x_0 fused with the update of x_0's gradient.
constexpr int kCrossNetMax = 8;        // most vectors u_k (seven layers and the output unit's)

// P[s,b,k] = sum over the columns j of shard s of x0[b,j] * U[k,j]; a group of G lanes per (kNetRows samples,
// shard), so that every float4 of U fetched from the caches serves several samples.
constexpr int kNetRows = 4;
template <int M>
__global__ __launch_bounds__(kBlock) void k_cross_net_partial(const float *__restrict__ x0, const float *__restrict__ U,
                                                               int64_t B, int F, int D4, int K, int G,
                                                               float *__restrict__ P) {
  const int64_t gid = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
  const int t = threadIdx.x % G;
  const int64_t stride = (int64_t)gridDim.x * kBlock / G;
  const int64_t row4 = (int64_t)F * D4;
  const int64_t n_items = ((B + kNetRows - 1) / kNetRows) * K;
  for (int64_t item = gid; item < n_items; item += stride) {
    const int64_t b0 = (item / K) * kNetRows;
    const int s = (int)(item % K);
    const int nf = s < F ? (F - s + K - 1) / K : 0;
    const int m_end = nf * D4;
    double acc[kNetRows][M];
#pragma unroll
    for (int r = 0; r < kNetRows; ++r)
#pragma unroll
      for (int k = 0; k < M; ++k) acc[r][k] = 0.0;
    for (int i = t; i < m_end; i += G) {
      const int f = s + K * (i / D4);
      const int64_t q = (int64_t)f * D4 + (i % D4);
      float4 xv[kNetRows];
#pragma unroll
      for (int r = 0; r < kNetRows; ++r)
        xv[r] = reinterpret_cast<const float4 *>(x0)[min(b0 + r, B - 1) * row4 + q];
#pragma unroll
      for (int k = 0; k < M; ++k) {
        const float4 uv = reinterpret_cast<const float4 *>(U)[k * row4 + q];
        const double ux = (double)uv.x, uy = (double)uv.y, uz = (double)uv.z, uw = (double)uv.w;
#pragma unroll
        for (int r = 0; r < kNetRows; ++r)
          acc[r][k] += ((double)xv[r].x * ux + (double)xv[r].y * uy) + ((double)xv[r].z * uz + (double)xv[r].w * uw);
      }
    }
    for (int o = G / 2; o > 0; o >>= 1) {
#pragma unroll
      for (int r = 0; r < kNetRows; ++r)
#pragma unroll
        for (int k = 0; k < M; ++k) acc[r][k] += __shfl_xor(acc[r][k], o, kWave);
    }
    if (t == 0) {
#pragma unroll
      for (int r = 0; r < kNetRows; ++r)
        if (b0 + r < B)
#pragma unroll
          for (int k = 0; k < M; ++k) P[((int64_t)s * B + b0 + r) * M + k] = (float)acc[r][k];
    }
  }
}

// c_k[j] = bias[0][j] + ... + bias[k-1][j]
__device__ inline double bias_prefix(const float *__restrict__ bias, int64_t d, int k, int64_t j) {
  double c = 0.0;
  for (int l = 0; l < k; ++l) c += (double)bias[(int64_t)l * d + j];
  return c;
}

// kappa[k] = <c_k, u_k>; one workgroup per k.
__global__ __launch_bounds__(kBlock) void k_cross_net_kappa(const float *__restrict__ U, const float *__restrict__ bias,
                                                             int64_t d, double *__restrict__ kappa) {
  __shared__ double red[kBlock];
  const int k = blockIdx.x;
  double acc = 0.0;
#pragma unroll 8
  for (int64_t j = threadIdx.x; j < d; j += kBlock) acc += bias_prefix(bias, d, k, j) * (double)U[(int64_t)k * d + j];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int h = kBlock / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) kappa[k] = red[0];
}

// gamma[b,0] = 1, gamma[b,l+1] = gamma[b,l] + s_l[b], c[b] = gamma[b,n] t[b,n] + kappa[n]; one thread per sample.
__global__ __launch_bounds__(kBlock) void k_cross_net_scalars(const float *__restrict__ t, const double *__restrict__ kappa,
                                                               int64_t B, int n, float *__restrict__ gamma,
                                                               float *__restrict__ c) {
  const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (b >= B) return;
  const int m = n + 1;
  double gam = 1.0;
  for (int l = 0; l < n; ++l) {
    gamma[b * m + l] = (float)gam;
    gam += gam * (double)t[b * m + l] + kappa[l];
  }
  gamma[b * m + n] = (float)gam;
  c[b] = (float)(gam * (double)t[b * m + n] + kappa[n]);
}

// beta[b,k] and, per workgroup, the sums of g_s_l and g over its samples (Gpart[block][k], double).
__global__ __launch_bounds__(kBlock) void k_cross_net_beta(const float *__restrict__ t, const float *__restrict__ gamma,
                                                            const float *__restrict__ g, int64_t B, int n,
                                                            float *__restrict__ beta, double *__restrict__ Gpart) {
  __shared__ double red[kBlock];
  const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int m = n + 1;
  double gs[kCrossNetMax];
#pragma unroll
  for (int k = 0; k < kCrossNetMax; ++k) gs[k] = 0.0;
  if (b < B) {
    const double gb = (double)g[b];
#pragma unroll
    for (int k = 0; k < kCrossNetMax; ++k)
      if (k == n) gs[k] = gb;                               // slot n carries g itself
#pragma unroll
    for (int l = kCrossNetMax - 2; l >= 0; --l) {
      if (l < n) {
        double a = gb * (double)t[b * m + n];
#pragma unroll
        for (int lp = 1; lp < kCrossNetMax - 1; ++lp)
          if (lp > l && lp < n) a += gs[lp] * (double)t[b * m + lp];
        gs[l] = a;
      }
    }
#pragma unroll
    for (int k = 0; k < kCrossNetMax; ++k)
      if (k <= n) beta[b * m + k] = (float)(gs[k] * (double)gamma[b * m + k]);
  }
#pragma unroll
  for (int k = 0; k < kCrossNetMax; ++k) {
    if (k > n) break;                                       // uniform
    red[threadIdx.x] = gs[k];
    __syncthreads();
    for (int h = kBlock / 2; h > 0; h >>= 1) {
      if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
      __syncthreads();
    }
    if (threadIdx.x == 0) Gpart[(int64_t)blockIdx.x * m + k] = red[0];
    __syncthreads();
  }
}

// Gsum[k] = sum over the workgroups' partials: one wave per k, lane i adds the partials i, i+64, ... in order,
// an xor tree adds the lanes.
__global__ __launch_bounds__(kWave) void k_cross_net_gsum(const double *__restrict__ Gpart, int64_t nblk, int m,
                                                           double *__restrict__ Gsum) {
  const int k = blockIdx.x;
  double a = 0.0;
#pragma unroll 4
  for (int64_t i = threadIdx.x; i < nblk; i += kWave) a += Gpart[i * m + k];
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) a += __shfl_xor(a, o, kWave);
  if (threadIdx.x == 0) Gsum[k] = a;
}

// The pass over x0 of the backward: g_x0[b,j] (+)= sum_k beta[b,k] U[k,j] and the slice's part of
// S[k,j] = sum_b beta[b,k] x0[b,j].  grid (blocks of 256 float4 columns, slices); partial[slice][k][:].
template <int M, bool kAccumulate>
__global__ __launch_bounds__(kBlock) void k_cross_net_grad(const float *__restrict__ x0, const float *__restrict__ U,
                                                            const float *__restrict__ beta, int64_t B, int64_t d4,
                                                            int64_t rows_per_slice, float *g_x0,
                                                            double *__restrict__ partial) {
  const int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (q >= d4) return;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slice;
  const int64_t r1 = min(B, r0 + rows_per_slice);
  float4 u[M];
  double S[M][4];
#pragma unroll
  for (int k = 0; k < M; ++k) {
    u[k] = reinterpret_cast<const float4 *>(U)[k * d4 + q];
    S[k][0] = S[k][1] = S[k][2] = S[k][3] = 0.0;
  }
  constexpr int UR = 4;
  for (int64_t r = r0; r < r1; r += UR) {
    float4 x[UR], old[UR];
#pragma unroll
    for (int i = 0; i < UR; ++i) {
      const int64_t rr = r + i < r1 ? r + i : r;
      x[i] = reinterpret_cast<const float4 *>(x0)[rr * d4 + q];
      if (kAccumulate) old[i] = reinterpret_cast<const float4 *>(g_x0)[rr * d4 + q];
    }
#pragma unroll
    for (int i = 0; i < UR; ++i) {
      if (r + i >= r1) break;
      double z[4] = {0.0, 0.0, 0.0, 0.0};
      if (kAccumulate) { z[0] = old[i].x; z[1] = old[i].y; z[2] = old[i].z; z[3] = old[i].w; }
#pragma unroll
      for (int k = 0; k < M; ++k) {
        const double bk = (double)beta[(r + i) * M + k];      // the same address for the whole workgroup
        z[0] += bk * (double)u[k].x; z[1] += bk * (double)u[k].y; z[2] += bk * (double)u[k].z; z[3] += bk * (double)u[k].w;
        S[k][0] += bk * (double)x[i].x; S[k][1] += bk * (double)x[i].y; S[k][2] += bk * (double)x[i].z; S[k][3] += bk * (double)x[i].w;
      }
      reinterpret_cast<float4 *>(g_x0)[(r + i) * d4 + q] = make_float4((float)z[0], (float)z[1], (float)z[2], (float)z[3]);
    }
  }
  const int64_t d = d4 * 4;
#pragma unroll
  for (int k = 0; k < M; ++k) {
    double *p = partial + ((int64_t)blockIdx.y * M + k) * d + q * 4;
    p[0] = S[k][0]; p[1] = S[k][1]; p[2] = S[k][2]; p[3] = S[k][3];
  }
}

// dU[k,j] = sum over the slices of S + c_k[j] G_k;  dbias[l,j] = U[n,j] G_n + sum_{l'>l} U[l',j] G_l'.
__global__ __launch_bounds__(kBlock) void k_cross_net_final(const double *__restrict__ partial, int slices,
                                                             const double *__restrict__ Gsum, const float *__restrict__ U,
                                                             const float *__restrict__ bias, int64_t d, int n,
                                                             float *__restrict__ dU, float *__restrict__ dbias) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  const int m = n + 1;
  for (int k = 0; k < m; ++k) {
    double a = 0.0;
#pragma unroll 8
    for (int sl = 0; sl < slices; ++sl) a += partial[((int64_t)sl * m + k) * d + j];
    dU[(int64_t)k * d + j] = (float)(a + bias_prefix(bias, d, k, j) * Gsum[k]);
  }
  double tail = (double)U[(int64_t)n * d + j] * Gsum[n];      // u_n G_n + sum over the layers above l
  for (int l = n - 1; l >= 0; --l) {
    dbias[(int64_t)l * d + j] = (float)tail;
    tail += (double)U[(int64_t)l * d + j] * Gsum[l];
  }
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

// ---- whole cross network ----
struct NetLayout { size_t kappa, gsum, beta, gpart, partial, total; int slices; int64_t nblk; };
static NetLayout net_layout(int64_t B, int64_t d, int n) {
  const int m = n + 1;
  const int64_t rows = B > 0 ? B : 1;
  NetLayout L;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
  L.nblk = (rows + kBlock - 1) / kBlock;
  L.slices = cross_slices(rows, d);
  L.kappa = take(kCrossNetMax * sizeof(double));
  L.gsum = take(kCrossNetMax * sizeof(double));
  L.beta = take((size_t)rows * m * sizeof(float));
  L.gpart = take((size_t)L.nblk * m * sizeof(double));
  L.partial = take((size_t)L.slices * m * (size_t)d * sizeof(double));
  L.total = o;
  return L;
}

des_status_t des_cross_net_bytes(int64_t B, int64_t d, int32_t n_layers, size_t *bytes) {
  if (!bytes || B < 0 || d < 4 || (d & 3) || n_layers < 0 || n_layers + 1 > kCrossNetMax) return DES_ERR_INVALID_ARG;
  *bytes = net_layout(B, d, n_layers).total;
  return DES_OK;
}

des_status_t des_cross_net_partial(const float *x0, const float *U, int64_t B, int32_t F, int32_t D, int32_t m,
                                   int32_t K, float *P, void *stream) {
  if (B < 0 || F < 1 || D < 4 || (D & 3) || K < 1 || m < 1 || m > kCrossNetMax || (int64_t)F * D > (1ll << 30))
    return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  if (!x0 || !U || !P || !aligned16(x0) || !aligned16(U)) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int D4 = D / 4;
  int G = 1;
  while (G < 16 && G * 2 <= D4) G *= 2;
  const unsigned grid = blocks_for((B + kNetRows - 1) / kNetRows * K * G, 1 << 20);
  ProfScope ps(KID_CROSS_PARTIAL, s);
#define DES_NET_PARTIAL(M) \
  case M: hipLaunchKernelGGL(k_cross_net_partial<M>, dim3(grid), dim3(kBlock), 0, s, x0, U, B, F, D4, K, G, P); break
  switch (m) {
    DES_NET_PARTIAL(1); DES_NET_PARTIAL(2); DES_NET_PARTIAL(3); DES_NET_PARTIAL(4);
    DES_NET_PARTIAL(5); DES_NET_PARTIAL(6); DES_NET_PARTIAL(7); DES_NET_PARTIAL(8);
  }
#undef DES_NET_PARTIAL
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_cross_net_forward(const float *t, const float *U, const float *bias, int64_t B, int64_t d,
                                   int32_t n_layers, float *gamma, float *c, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  if (B < 0 || d < 4 || (d & 3) || n_layers < 0 || n_layers + 1 > kCrossNetMax) return DES_ERR_INVALID_ARG;
  if (B == 0) return DES_OK;
  if (!t || !U || (n_layers > 0 && !bias) || !gamma || !c) return DES_ERR_INVALID_ARG;
  const NetLayout L = net_layout(B, d, n_layers);
  if (!workspace || workspace_bytes < L.total || ((uintptr_t)workspace & 255u)) return DES_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  double *kappa = (double *)((char *)workspace + L.kappa);
  ProfScope ps(KID_CROSS_APPLY, s);
  hipLaunchKernelGGL(k_cross_net_kappa, dim3(n_layers + 1), dim3(kBlock), 0, s, U, bias, d, kappa);
  hipLaunchKernelGGL(k_cross_net_scalars, dim3(blocks_for(B, 1 << 30)), dim3(kBlock), 0, s, t, kappa, B, n_layers, gamma, c);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_cross_net_backward(const float *x0, const float *U, const float *bias, const float *t,
                                    const float *gamma, const float *g, int64_t B, int64_t d, int32_t n_layers,
                                    float *g_x0, int32_t accumulate_g_x0, float *dU, float *dbias, void *workspace,
                                    size_t workspace_bytes, void *stream) {
  if (B < 0 || d < 4 || (d & 3) || n_layers < 0 || n_layers + 1 > kCrossNetMax) return DES_ERR_INVALID_ARG;
  if (!dU || (n_layers > 0 && (!dbias || !bias)) || !U) return DES_ERR_INVALID_ARG;
  const NetLayout L = net_layout(B, d, n_layers);
  if (!workspace || workspace_bytes < L.total || ((uintptr_t)workspace & 255u)) return DES_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)workspace;
  float *beta = (float *)(ws + L.beta);
  double *gpart = (double *)(ws + L.gpart), *gsum = (double *)(ws + L.gsum), *partial = (double *)(ws + L.partial);
  const int m = n_layers + 1;
  const int64_t d4 = d / 4;
  ProfScope ps(KID_CROSS_GRAD, s);
  if (B == 0) {                                          // empty batch: every sum is zero
    hipLaunchKernelGGL(k_cross_net_gsum, dim3(m), dim3(kWave), 0, s, gpart, (int64_t)0, m, gsum);
    hipLaunchKernelGGL(k_cross_net_final, dim3(blocks_for(d, 1 << 20)), dim3(kBlock), 0, s, partial, 0, gsum, U, bias, d,
                       n_layers, dU, dbias);
    return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
  }
  if (!x0 || !t || !gamma || !g || !g_x0 || !aligned16(x0) || !aligned16(U) || !aligned16(g_x0)) return DES_ERR_INVALID_ARG;
  hipLaunchKernelGGL(k_cross_net_beta, dim3((unsigned)L.nblk), dim3(kBlock), 0, s, t, gamma, g, B, n_layers, beta, gpart);
  hipLaunchKernelGGL(k_cross_net_gsum, dim3(m), dim3(kWave), 0, s, gpart, L.nblk, m, gsum);
  const int64_t rows_per_slice = (B + L.slices - 1) / L.slices;
  const dim3 grid((unsigned)((d4 + kBlock - 1) / kBlock), (unsigned)L.slices);
#define DES_NET_GRAD(M)                                                                                                  \
  case M:                                                                                                                \
    if (accumulate_g_x0)                                                                                                 \
      hipLaunchKernelGGL((k_cross_net_grad<M, true>), grid, dim3(kBlock), 0, s, x0, U, beta, B, d4, rows_per_slice, g_x0, \
                         partial);                                                                                       \
    else                                                                                                                 \
      hipLaunchKernelGGL((k_cross_net_grad<M, false>), grid, dim3(kBlock), 0, s, x0, U, beta, B, d4, rows_per_slice,      \
                         g_x0, partial);                                                                                 \
    break
  switch (m) {
    DES_NET_GRAD(1); DES_NET_GRAD(2); DES_NET_GRAD(3); DES_NET_GRAD(4);
    DES_NET_GRAD(5); DES_NET_GRAD(6); DES_NET_GRAD(7); DES_NET_GRAD(8);
  }
#undef DES_NET_GRAD
  hipLaunchKernelGGL(k_cross_net_final, dim3(blocks_for(d, 1 << 20)), dim3(kBlock), 0, s, partial, L.slices, gsum, U, bias,
                     d, n_layers, dU, dbias);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // extern "C"