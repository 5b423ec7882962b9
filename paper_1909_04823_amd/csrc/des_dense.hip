// The dense remainder of a DES model step: what runs on every process, identically, after the
// aggregated weights-rich operators (Section 3.2.1) -- the hidden-layer epilogue fused into the
// aggregation, the output unit with the mean log-loss (Section 4.1: sigmoid output; Section 6
// reports log loss), their backward passes and the optimizer step of the dense parameters.
// All of it is streaming, elementwise or column-reduction work bound by HBM; sums over the batch
// are taken in double in a fixed order (per-slice partials, then one pass over the slices), so
// results do not depend on scheduling.
#include <mutex>
#include "des_internal.h"

namespace des {
namespace {

constexpr int kMaxSlices = 64;        // row slices of a column reduction
constexpr int kHeadBlocks = 1024;     // workgroups of the output-unit kernel (each keeps one loss partial)

// Library-owned scratch of des_bias_act_backward_static: the per-slice column partials of layers up to
// kStaticMaxH wide (2 MiB per GPU, held until the process ends).  Every GPU has its own copy of the array at
// its own address; in host code the array's name is only a handle for hipGetSymbolAddress, never a pointer.
constexpr int kStaticMaxH = 4096;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) double scratch[(size_t)kMaxSlices * kStaticMaxH];
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
des_status_t static_scratch(double **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DES_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DES_ERR_DEVICE;
    g_scratch_ptr[dev] = static_cast<double *>(p);
  }
  *out = g_scratch_ptr[dev];
  return DES_OK;
}

inline unsigned blocks_for(int64_t n, int64_t cap) {
  int64_t g = (n + kBlock - 1) / kBlock;
  return (unsigned)(g < 1 ? 1 : (g > cap ? cap : g));
}

// out[b,h] = act( sum_s P[s,b,h] + bias[h] ), four columns per thread, shard sum in double.
__global__ __launch_bounds__(kBlock) void k_aggregate_bias_act(const float *__restrict__ P, int K, int64_t rows,
                                                                int H, const float *__restrict__ bias, int relu,
                                                                float *__restrict__ out) {
  const int64_t n4 = rows * H / 4, n = rows * H;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const int h = (int)((i * 4) % H);
    double a[4] = {0.0, 0.0, 0.0, 0.0};
    if (bias) {
      const float4 bv = *reinterpret_cast<const float4 *>(bias + h);
      a[0] = bv.x; a[1] = bv.y; a[2] = bv.z; a[3] = bv.w;
    }
    // bias first or last makes no difference to the double sum beyond its last bit; the rounding to
    // fp32 happens once, below
#pragma unroll 8
    for (int s = 0; s < K; ++s) {
      const float4 p = *reinterpret_cast<const float4 *>(P + (int64_t)s * n + i * 4);
      a[0] += (double)p.x; a[1] += (double)p.y; a[2] += (double)p.z; a[3] += (double)p.w;
    }
    float4 o = make_float4((float)a[0], (float)a[1], (float)a[2], (float)a[3]);
    if (relu) { o.x = fmaxf(o.x, 0.f); o.y = fmaxf(o.y, 0.f); o.z = fmaxf(o.z, 0.f); o.w = fmaxf(o.w, 0.f); }
    *reinterpret_cast<float4 *>(out + i * 4) = o;
  }
}

// Column sums over a slice of rows.  kMode 0: v = dA[r,c] where A[r,c] > 0 (or everywhere without
// relu), written to dZ and summed.  kMode 1: v = g[r] * A[r,c], summed only.
// grid (column blocks of 64, slices); lane = column, the four waves take rows r = begin + wave, +4, ...
template <int kMode>
__global__ __launch_bounds__(kBlock) void k_column_partials(const float *__restrict__ A, const float *dA,
                                                             const float *__restrict__ g, int64_t rows, int H,
                                                             int relu, int64_t rows_per_slice, float *dZ,
                                                             double *__restrict__ partial) {
  __shared__ double red[kBlock];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int c = blockIdx.x * kWave + lane;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slice;
  const int64_t r1 = min(rows, r0 + rows_per_slice);
  double acc = 0.0;
  if (c < H) {
    for (int64_t r = r0 + wave; r < r1; r += kBlock / kWave) {
      const int64_t i = r * H + c;
      if (kMode == 0) {
        const float v = (!relu || A[i] > 0.f) ? dA[i] : 0.f;
        dZ[i] = v;
        acc += (double)v;
      } else {
        acc += (double)g[r] * (double)A[i];
      }
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (wave == 0 && c < H)
    partial[(int64_t)blockIdx.y * H + c] = (red[lane] + red[lane + kWave]) + (red[lane + 2 * kWave] + red[lane + 3 * kWave]);
}

// out[c] = sum over the slices of partial[s,c], in slice order.
__global__ __launch_bounds__(kBlock) void k_column_final(const double *__restrict__ partial, int slices, int H,
                                                          float *__restrict__ out) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= H) return;
  double a = 0.0;
  for (int s = 0; s < slices; ++s) a += partial[(int64_t)s * H + c];
  out[c] = (float)a;
}

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Output unit: one wave per sample (grid-stride).  logit = b0 + A_lr + fm2 + <a, w_out> in double;
// p, the sample's log-loss log(1+e^z) - y z in its overflow-free form, g = (p - y)/B; da = g * w_out.
// Lane 0 of each wave keeps running sums of loss and g; the workgroup writes one partial of each.
__global__ __launch_bounds__(kBlock) void k_head(const float *__restrict__ A_lr, const float *__restrict__ fm2,
                                                  const float *__restrict__ a, const float *__restrict__ w_out,
                                                  const float *__restrict__ b0, const float *__restrict__ labels,
                                                  int64_t B, int H, float *__restrict__ logit_out,
                                                  float *__restrict__ p_out, float *__restrict__ g_logit,
                                                  float *__restrict__ da, double *__restrict__ partial) {
  __shared__ double red[2 * (kBlock / kWave)];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t wstride = (int64_t)gridDim.x * (kBlock / kWave);
  const double bias = b0 ? (double)b0[0] : 0.0;
  double loss_acc = 0.0, g_acc = 0.0;
  for (int64_t b = (int64_t)blockIdx.x * (kBlock / kWave) + wave; b < B; b += wstride) {
    double dot = 0.0;
    if (a)
      for (int h = lane; h < H; h += kWave) dot += (double)a[b * H + h] * (double)w_out[h];
    dot = wave_sum(dot);
    double z = bias + dot;
    if (A_lr) z += (double)A_lr[b];
    if (fm2) z += (double)fm2[b];
    const double y = (double)labels[b];
    const double p = 1.0 / (1.0 + exp(-z));
    const double gd = (p - y) / (double)B;
    const float gf = (float)gd;
    if (lane == 0) {
      loss_acc += (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z))) - y * z;
      g_acc += gd;
      if (logit_out) logit_out[b] = (float)z;
      if (p_out) p_out[b] = (float)p;
      g_logit[b] = gf;
    }
    if (a && da)
      for (int h = lane; h < H; h += kWave) da[b * H + h] = (float)(gd * (double)w_out[h]);
  }
  if (lane == 0) { red[wave] = loss_acc; red[kBlock / kWave + wave] = g_acc; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double l = 0.0, gs = 0.0;
    for (int w = 0; w < kBlock / kWave; ++w) { l += red[w]; gs += red[kBlock / kWave + w]; }
    partial[blockIdx.x] = l;
    partial[gridDim.x + blockIdx.x] = gs;
  }
}

// loss = (sum of the loss partials)/B, db0 = sum of the g partials; one wave, fixed order.
__global__ __launch_bounds__(kWave) void k_head_final(const double *__restrict__ partial, int nblocks, int64_t B,
                                                       float *__restrict__ loss_out, float *__restrict__ db0_out) {
  double l = 0.0, gs = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += kWave) { l += partial[i]; gs += partial[nblocks + i]; }
  l = wave_sum(l);
  gs = wave_sum(gs);
  if (threadIdx.x == 0) {
    if (loss_out) loss_out[0] = (float)(l / (double)B);
    if (db0_out) db0_out[0] = (float)gs;
  }
}

// One optimizer step on every coordinate of a dense array, in double, state and weight stored in fp32.
__global__ __launch_bounds__(kBlock) void k_dense_update(float *__restrict__ theta, const float *__restrict__ grad,
                                                          float *__restrict__ s1, float *__restrict__ s2, int64_t n,
                                                          const des_optimizer_t o, double c1, double c2) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const double G = (double)grad[i], w = (double)theta[i];
    if (o.opt_emb == DES_OPT_SGD) {
      theta[i] = (float)(w - (double)o.lr * G);
    } else if (o.opt_emb == DES_OPT_ADAGRAD) {
      const double acc = (double)s1[i] + G * G;
      theta[i] = (float)(w - (double)o.lr * G / (sqrt(acc) + (double)o.eps));
      s1[i] = (float)acc;
    } else if (o.opt_emb == DES_OPT_ADAM) {       // c1 = 1 - beta1^t, c2 = 1 - beta2^t from the host
      const double m = (double)o.beta1 * (double)s1[i] + (1.0 - (double)o.beta1) * G;
      const double v = (double)o.beta2 * (double)s2[i] + (1.0 - (double)o.beta2) * G * G;
      theta[i] = (float)(w - (double)o.lr * (m / c1) / (sqrt(v / c2) + (double)o.eps));
      s1[i] = (float)m;
      s2[i] = (float)v;
    } else {                                      // FTRL-Proximal: s1 = n, s2 = z
      const double n0 = (double)s1[i], n1 = n0 + G * G;
      const double sigma = (sqrt(n1) - sqrt(n0)) / (double)o.ftrl_alpha;
      const double z = (double)s2[i] + G - sigma * w;
      const double l1 = (double)o.ftrl_l1;
      const double wn = fabs(z) <= l1 ? 0.0
                                      : -(z - (z > 0.0 ? l1 : -l1)) /
                                            (((double)o.ftrl_beta + sqrt(n1)) / (double)o.ftrl_alpha + (double)o.ftrl_l2);
      theta[i] = (float)wn;
      s1[i] = (float)n1;
      s2[i] = (float)z;
    }
  }
}

bool al16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
bool al8(const void *p) { return ((uintptr_t)p & 7u) == 0; }

int slices_for(int64_t rows) {
  int64_t s = (rows + 255) / 256;                 // at least 256 rows per slice
  return (int)(s < 1 ? 1 : (s > kMaxSlices ? kMaxSlices : s));
}

template <int kMode>
des_status_t column_sums(const float *A, const float *dA, const float *g, int64_t rows, int H, int relu, float *dZ,
                         float *out, double *partial, hipStream_t s) {
  const int slices = slices_for(rows);
  const int64_t per = (rows + slices - 1) / slices;
  {
    ProfScope ps(KID_COLUMN_PARTIALS, s);
    hipLaunchKernelGGL((k_column_partials<kMode>), dim3((unsigned)((H + kWave - 1) / kWave), (unsigned)slices),
                       dim3(kBlock), 0, s, A, dA, g, rows, H, relu, per, dZ, partial);
  }
  {
    ProfScope ps(KID_COLUMN_FINAL, s);
    hipLaunchKernelGGL(k_column_final, dim3((unsigned)((H + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, partial,
                       slices, H, out);
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // namespace
}  // namespace des

using namespace des;

extern "C" {

des_status_t des_dense_workspace_bytes(int32_t H_max, size_t *workspace_bytes) {
  if (!workspace_bytes || H_max < 0) return DES_ERR_INVALID_ARG;
  const size_t cols = (size_t)kMaxSlices * (size_t)H_max, head = 2 * (size_t)kHeadBlocks;
  *workspace_bytes = sizeof(double) * (cols > head ? cols : head);
  return DES_OK;
}

des_status_t des_aggregate_bias_act(const float *P, int32_t K, int64_t rows, int32_t H, const float *bias,
                                    int32_t relu, float *out, void *stream) {
  if (K < 1 || rows < 0 || H < 4 || (H & 3)) return DES_ERR_INVALID_ARG;
  if (rows == 0) return DES_OK;
  if (!P || !out || !al16(P) || !al16(out) || !al16(bias)) return DES_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_AGG_BIAS_ACT, s);
  hipLaunchKernelGGL(k_aggregate_bias_act, dim3(blocks_for(rows * H / 4, 1 << 20)), dim3(kBlock), 0, s, P, K, rows, H,
                     bias, relu, out);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_bias_act_backward(const float *A, const float *dA, int64_t rows, int32_t H, int32_t relu, float *dZ,
                                   float *dbias, void *workspace, size_t workspace_bytes, void *stream) {
  if (rows < 0 || H < 1) return DES_ERR_INVALID_ARG;
  if (!A || !dA || !dZ || !dbias || !workspace || !al8(workspace)) return DES_ERR_INVALID_ARG;
  if (workspace_bytes < sizeof(double) * (size_t)kMaxSlices * (size_t)H) return DES_ERR_WORKSPACE;
  return column_sums<0>(A, dA, nullptr, rows, H, relu, dZ, dbias, (double *)workspace, (hipStream_t)stream);
}

des_status_t des_bias_act_backward_static(const float *A, const float *dA, int64_t rows, int32_t H, int32_t relu,
                                          float *dZ, float *dbias, void *stream) {
  if (rows < 0 || H < 1) return DES_ERR_INVALID_ARG;
  if (!A || !dA || !dZ || !dbias) return DES_ERR_INVALID_ARG;
  if (H > kStaticMaxH) return DES_ERR_WORKSPACE;      // wider than the library's own scratch holds
  double *partial = nullptr;
  const des_status_t st = static_scratch(&partial);
  if (st != DES_OK) return st;
  // every partial the final pass reads is written by the first pass of the same call: nothing to clear
  return column_sums<0>(A, dA, nullptr, rows, H, relu, dZ, dbias, partial, (hipStream_t)stream);
}

des_status_t des_head(const float *A_lr, const float *fm2, const float *a, const float *w_out, const float *b0,
                      const float *labels, int64_t B, int32_t H, float *logit_out, float *p_out, float *loss_out,
                      float *g_logit, float *da, float *dw_out, float *db0_out, void *workspace,
                      size_t workspace_bytes, void *stream) {
  if (B < 1 || !labels || !g_logit || !workspace || !al8(workspace)) return DES_ERR_INVALID_ARG;
  if ((a != nullptr) != (w_out != nullptr) || (a && H < 1) || (dw_out && !a)) return DES_ERR_INVALID_ARG;
  size_t need = sizeof(double) * 2 * (size_t)kHeadBlocks;
  if (dw_out && sizeof(double) * (size_t)kMaxSlices * (size_t)H > need) need = sizeof(double) * (size_t)kMaxSlices * (size_t)H;
  if (workspace_bytes < need) return DES_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  int64_t nb = (B + kBlock / kWave - 1) / (kBlock / kWave);
  if (nb > kHeadBlocks) nb = kHeadBlocks;
  {
    ProfScope ps(KID_HEAD, s);
    hipLaunchKernelGGL(k_head, dim3((unsigned)nb), dim3(kBlock), 0, s, A_lr, fm2, a, w_out, b0, labels, B, H, logit_out,
                       p_out, g_logit, da, (double *)workspace);
    hipLaunchKernelGGL(k_head_final, dim3(1), dim3(kWave), 0, s, (const double *)workspace, (int)nb, B, loss_out,
                       db0_out);
  }
  if (hipGetLastError() != hipSuccess) return DES_ERR_DEVICE;
  if (dw_out)      // dw_out[h] = sum_b g[b] * a[b,h]; reuses the workspace after the head's partials were consumed
    return column_sums<1>(a, nullptr, g_logit, B, H, 0, nullptr, dw_out, (double *)workspace, s);
  return DES_OK;
}

des_status_t des_dense_update(float *theta, const float *grad, float *s1, float *s2, int64_t n,
                              const des_optimizer_t *optimizer, void *stream) {
  if (n < 0 || !optimizer) return DES_ERR_INVALID_ARG;
  const des_optimizer_t &o = *optimizer;
  const int opt = o.opt_emb;
  if (opt != DES_OPT_SGD && opt != DES_OPT_ADAGRAD && opt != DES_OPT_ADAM && opt != DES_OPT_FTRL) return DES_ERR_INVALID_ARG;
  if (n == 0) return DES_OK;
  if (!theta || !grad) return DES_ERR_INVALID_ARG;
  if (opt != DES_OPT_SGD && !s1) return DES_ERR_INVALID_ARG;
  if ((opt == DES_OPT_ADAM || opt == DES_OPT_FTRL) && !s2) return DES_ERR_INVALID_ARG;
  if (opt == DES_OPT_ADAM && o.step < 1) return DES_ERR_INVALID_ARG;
  if (opt == DES_OPT_FTRL && !(o.ftrl_alpha > 0.f)) return DES_ERR_INVALID_ARG;
  double c1 = 1.0, c2 = 1.0;
  if (opt == DES_OPT_ADAM) {
    c1 = 1.0 - pow((double)o.beta1, (double)o.step);
    c2 = 1.0 - pow((double)o.beta2, (double)o.step);
  }
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_DENSE_UPDATE, s);
  hipLaunchKernelGGL(k_dense_update, dim3(blocks_for(n, 1 << 16)), dim3(kBlock), 0, s, theta, grad, s1, s2, n, o, c1, c2);
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // extern "C"
