// Measurement aids: kernels that perform nothing but the table accesses of a step, on the same index streams and
// with the same lane mapping and access instructions as the real kernels.  Their rates are what this GPU delivers
// for these access patterns (random rows of D floats through L2 / Infinity Cache / HBM) with no arithmetic, no LDS
// and no other traffic in the way, i.e. the ceiling the forward gather and the row update are measured against
// where the published 8 TB/s of streaming bandwidth is not the limit that applies.
#include "des_internal.h"

namespace des {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

// Forward-pass pattern: entry e reads row rows[e] (D floats, D/4 adjacent lanes with one 16-byte load each), U rows
// in flight per lane group, entries taken in batch order.  Every wave leaves one float so the loads are live.
template <int D>
__global__ __launch_bounds__(kBlock) void k_ceiling_gather(const float *__restrict__ emb, int64_t stride,
                                                            const float *__restrict__ w, int64_t w_stride, int64_t n_rows,
                                                            const int32_t *__restrict__ rows, int64_t n,
                                                            float *__restrict__ sink) {
  constexpr int G = D / 4;
  constexpr int U = 8;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int sub = (int)(gid % G);
  const int64_t group = gid / G, ngroups = (int64_t)gridDim.x * blockDim.x / G;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  // a lane group takes U consecutive entries at a time, the groups stride over the batch
  for (int64_t e0 = group * U; e0 < n; e0 += ngroups * U) {
    int32_t r[U];
    float4 v[U];
#pragma unroll
    for (int i = 0; i < U; ++i) r[i] = e0 + i < n ? rows[e0 + i] : -1;
#pragma unroll
    for (int i = 0; i < U; ++i)
      v[i] = (r[i] >= 0 && r[i] < n_rows) ? *reinterpret_cast<const float4 *>(emb + (int64_t)r[i] * stride + sub * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    float wv[U];
#pragma unroll
    for (int i = 0; i < U; ++i)       // the LR weight of the row, fetched by one lane of the group as in the forward pass
      wv[i] = (w && sub == (G > 1 ? 1 : 0) && r[i] >= 0 && r[i] < n_rows) ? w[(int64_t)r[i] * w_stride] : 0.f;
#pragma unroll
    for (int i = 0; i < U; ++i) { acc.x += v[i].x + wv[i]; acc.y += v[i].y; acc.z += v[i].z; acc.w += v[i].w; }
  }
  float t = acc.x + acc.y + acc.z + acc.w;
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) t += __shfl_xor(t, o, kWave);
  if ((threadIdx.x & (kWave - 1)) == 0) sink[gid / kWave] = t;
}

// Update pattern: segment u reads the D floats of row uniq_rows[u] in two arrays (weights, optimizer state) with
// streaming loads and writes both back with streaming stores, one lane group per row, rows ascending.  `zero` is 0
// at run time (the compiler cannot know), so the arrays keep their contents.
template <int D>
__global__ __launch_bounds__(kBlock) void k_ceiling_update(float *emb, float *acc, int64_t stride, int64_t n_rows,
                                                            const int32_t *__restrict__ uniq_rows, int64_t n_uniq, float zero) {
  constexpr int G = D / 4;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int sub = (int)(gid % G);
  const int64_t ngroups = (int64_t)gridDim.x * blockDim.x / G;
  for (int64_t u = gid / G; u < n_uniq; u += ngroups) {
    const int64_t row = uniq_rows[u];
    if (row < 0 || row >= n_rows) continue;            // rows outside the table are skipped, not trusted
    v4f *pv = reinterpret_cast<v4f *>(emb + row * stride + sub * 4);
    v4f *pa = reinterpret_cast<v4f *>(acc + row * stride + sub * 4);
    v4f v = __builtin_nontemporal_load(pv), s = __builtin_nontemporal_load(pa);
    v += zero;
    s += zero;
    __builtin_nontemporal_store(v, pv);
    __builtin_nontemporal_store(s, pa);
  }
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

constexpr int kGatherGrid = 8192;     // workgroups of the gather kernel (grid-stride)
constexpr int kUpdateGrid = 65536;    // most workgroups of the update kernel, as in the real one

}  // namespace
}  // namespace des

using namespace des;

extern "C" {

des_status_t des_ceiling_gather_bytes(size_t *sink_bytes) {
  if (!sink_bytes) return DES_ERR_INVALID_ARG;
  *sink_bytes = (size_t)kGatherGrid * (kBlock / kWave) * sizeof(float);
  return DES_OK;
}

des_status_t des_ceiling_gather(const float *emb, int32_t D, int64_t stride, const float *w, int64_t w_stride, int64_t n_rows,
                                const int32_t *rows, int64_t n, float *sink, size_t sink_bytes, void *stream) {
  if (!emb || !rows || !sink || n < 0 || n_rows < 1 || !aligned16(emb) || ((uintptr_t)rows & 3u) || ((uintptr_t)sink & 3u))
    return DES_ERR_INVALID_ARG;
  if (stride < D || (stride & 3) || ((uintptr_t)w & 3u) || (w && w_stride < 1)) return DES_ERR_INVALID_ARG;
  if (sink_bytes < (size_t)kGatherGrid * (kBlock / kWave) * sizeof(float)) return DES_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_CEILING_GATHER, s);
  const dim3 grid(kGatherGrid), block(kBlock);
  switch (D) {
    case 4: hipLaunchKernelGGL(k_ceiling_gather<4>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    case 8: hipLaunchKernelGGL(k_ceiling_gather<8>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    case 16: hipLaunchKernelGGL(k_ceiling_gather<16>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    case 32: hipLaunchKernelGGL(k_ceiling_gather<32>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    case 64: hipLaunchKernelGGL(k_ceiling_gather<64>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    case 128: hipLaunchKernelGGL(k_ceiling_gather<128>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    case 256: hipLaunchKernelGGL(k_ceiling_gather<256>, grid, block, 0, s, emb, stride, w, w_stride, n_rows, rows, n, sink); break;
    default: return DES_ERR_INVALID_ARG;
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t des_ceiling_update(float *emb, float *acc, int32_t D, int64_t stride, int64_t n_rows, const int32_t *uniq_rows,
                                int64_t n_uniq, void *stream) {
  if (!emb || !acc || !uniq_rows || n_uniq < 0 || n_rows < 1 || !aligned16(emb) || !aligned16(acc) || ((uintptr_t)uniq_rows & 3u))
    return DES_ERR_INVALID_ARG;
  if (stride < D || (stride & 3)) return DES_ERR_INVALID_ARG;
  if (n_uniq == 0) return DES_OK;
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps(KID_CEILING_UPDATE, s);
  int64_t blocks = (n_uniq * (D / 4) + kBlock - 1) / kBlock;
  if (blocks > kUpdateGrid) blocks = kUpdateGrid;
  const dim3 grid((unsigned)blocks), block(kBlock);
  const float zero = 0.f;
  switch (D) {
    case 4: hipLaunchKernelGGL(k_ceiling_update<4>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    case 8: hipLaunchKernelGGL(k_ceiling_update<8>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    case 16: hipLaunchKernelGGL(k_ceiling_update<16>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    case 32: hipLaunchKernelGGL(k_ceiling_update<32>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    case 64: hipLaunchKernelGGL(k_ceiling_update<64>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    case 128: hipLaunchKernelGGL(k_ceiling_update<128>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    case 256: hipLaunchKernelGGL(k_ceiling_update<256>, grid, block, 0, s, emb, acc, stride, n_rows, uniq_rows, n_uniq, zero); break;
    default: return DES_ERR_INVALID_ARG;
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // extern "C"
