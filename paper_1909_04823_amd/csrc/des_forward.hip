// Forward sub-operators of every logical shard in one pass over the batch:
//   LR  M1 (Section 4.1, Eq. lr_m1), FM M1 and M2 (Section 4.2, Eq. fm_m1m2) and the per-field
//   pooled embeddings (Section 4.3).
//
// Mapping: 1, 2 or 4 wave64s per sample.  A row of D floats is read by G = D/4 adjacent lanes
// as one 16-byte load each, so a wave holds 64/G "lane groups" that each fetch a different row
// at the same time.  Every group owns a contiguous range of the sample's bags and walks its
// entries in CSR order in chunks of G: lane i of the group loads the metadata of entry i of
// the chunk (row, key -> shard, value, bag found in the sample's offsets staged in LDS) and
// publishes it in LDS, from where the group reads entry j with one broadcast read; the row
// gathers of a chunk are issued back to back.  The running bag sum stays in registers (the
// pooled output is written once per bag, already summed over shards).  The per-shard FM / LR
// partials of the sample live in LDS ([K][D+2] doubles per sample: D columns, then the sum of
// squares and the LR sum) and are updated with LDS atomics, because the entries of one shard are
// scattered over all groups.  A lane owns columns 4*sub..4*sub+3 of a row but the LDS copy is
// stored column-permuted (column 4*sub+k at k*G+sub) with a row pitch of D+2 doubles, so that the
// 64 lanes of one atomic instruction spread over the LDS banks instead of piling onto a few.
//
// Accumulation is in double, inputs and outputs are fp32: a sample's sum of several hundred
// signed terms cancels, and fp32 accumulation alone would exceed the 1e-5 relative bound
// against an exact reference.
#include "des_internal.h"

namespace des {
namespace {

struct FwdArgs {
  const float *emb, *w;
  const uint64_t *keys;
  const int32_t *offsets;
  const float *vals;
  const int32_t *rows;
  float *P_lr, *P_sum, *P_sq, *pool;
  int64_t B;
  int F, K, policy;
  int acc_doubles;      // LDS doubles per sample for the accumulators
  int lds_per_sample;   // LDS doubles per sample in total (accumulators + staged offsets)
  int wps;              // waves per sample: 1, 2 or 4
};

__device__ inline float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ inline void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }

// Cross-lane move of a double with a DPP control word (VALU, does not use the LDS pipe).
template <int kCtrl>
__device__ inline double dpp_f64(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, kCtrl, 0xF, 0xF, true);
  hi = __builtin_amdgcn_update_dpp(0, hi, kCtrl, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}

// Sum of q over the G adjacent lanes of a lane group (every lane gets the total).
template <int G>
__device__ inline double group_sum(double q) {
  if (G >= 2) q += dpp_f64<0xB1>(q);     // quad_perm [1,0,3,2]
  if (G >= 4) q += dpp_f64<0x4E>(q);     // quad_perm [2,3,0,1]
  if (G >= 8) q += dpp_f64<0x141>(q);    // row_half_mirror: pairs the two quads of 8 lanes
  if (G >= 16) q += dpp_f64<0x140>(q);   // row_mirror: pairs the two halves of 16 lanes
#pragma unroll
  for (int m = 16; m < G; m <<= 1) q += __shfl_xor(q, m, kWave);
  return q;
}

// kByKey: shard of an entry = hash of its ID (entries of a bag scatter over the shards: one LDS update per
// entry).  Otherwise the field partition of Section 5: a bag belongs to shard f mod K as a whole, so its sums
// are formed in registers and the shard's accumulators take one update per bag.
// kHasVals: the batch carries feature values; without them every x is 1 and the products with x are left out.
template <int D, bool kByKey, bool kHasVals>
__global__ __launch_bounds__(kBlock) void k_forward(const FwdArgs a) {
  extern __shared__ __align__(16) double lds[];
  constexpr int G = D / 4;                 // lanes per row = entries per chunk
  constexpr int NG = kWave / G;            // lane groups per wave
  constexpr int U = G >= 16 ? 8 : (G < 4 ? G : 4);   // row gathers in flight per lane (measured: 8 pays from D = 64 on)
  constexpr int kLrLane = G > 1 ? 1 : 0;   // lane of a group that fetches and adds the LR weight
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / G, sub = lane % G;
  const int K = a.K, F = a.F, wps = a.wps;
  const int local = wave / wps, wis = wave % wps;         // sample slot in the workgroup, wave in sample
  // LDS: one 16-byte metadata slot per thread, then per sample the accumulators and offsets
  int4 *meta = reinterpret_cast<int4 *>(lds) + wave * kWave;
  constexpr int P = D + 2;                                // row pitch: D columns, sum of squares, LR sum
  double *sum = lds + 2 * kBlock + (size_t)local * a.lds_per_sample;   // [K][P]
  int *offs = reinterpret_cast<int *>(sum + a.acc_doubles);   // [F+1]
  const int64_t b = (int64_t)blockIdx.x * (kBlock / kWave / wps) + local;
  const bool active = b < a.B;
  const bool need_fm = a.P_sum != nullptr, need_lr = a.P_lr != nullptr, need_pool = a.pool != nullptr;
  const bool need_v = need_fm || need_pool;
  constexpr bool by_key = kByKey;
  const int tis = wis * kWave + lane, nts = wps * kWave;  // thread in sample, threads per sample

  for (int i = tis; i < a.acc_doubles; i += nts) sum[i] = 0.0;
  if (active)
    for (int i = tis; i <= F; i += nts) offs[i] = a.offsets[b * F + i];
  __syncthreads();

  if (active) {
    const int gg = wis * NG + g, ngt = wps * NG;
    const int f0 = (int)(((int64_t)F * gg) / ngt), f1 = (int)(((int64_t)F * (gg + 1)) / ngt);
    const int e0 = offs[f0], e1 = offs[f1];
    int cur = f0;                                         // bag whose sum is being accumulated
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    double bag_sq = 0.0, bag_lr = 0.0;                    // field partition: this lane's share of the bag's scalars
    bool bag_dirty = false;
    float *pool_row = need_pool ? a.pool + (b * F) * (int64_t)D + sub * 4 : nullptr;
    // closes bag `cur`: pooled sum out; under the field partition also the bag's contribution to its shard
    auto close_bag = [&]() {
      if (need_pool)
        st4(pool_row + (int64_t)cur * D, make_float4((float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]));
      if (!kByKey && bag_dirty) {
        const int s = cur % K;
        if (need_fm) {
          double *dst = sum + s * P + sub;
#pragma unroll
          for (int k = 0; k < 4; ++k) atomicAdd(dst + k * G, acc[k]);
          const double q = group_sum<G>(bag_sq);
          if (sub == 0) atomicAdd(sum + s * P + D, q);
        }
        if (need_lr && sub == kLrLane) atomicAdd(sum + s * P + D + 1, bag_lr);
        bag_sq = 0.0;
        bag_lr = 0.0;
        bag_dirty = false;
      }
      acc[0] = acc[1] = acc[2] = acc[3] = 0.0;
    };

    // metadata of entry e0 + sub of the first chunk; later chunks are fetched one chunk ahead
    int r_n = -1;
    uint64_t key_n = 0;
    float x_n = 1.f;
    {
      const int my = e0 + sub;
      if (my < e1) {
        r_n = a.rows[my];
        if (by_key) key_n = a.keys[my];
        if (kHasVals) x_n = a.vals[my];
      }
    }
    for (int e = e0; e < e1; e += G) {
      const int my = e + sub;
      const int r_l = r_n;
      const uint64_t key_l = key_n;
      const float x_l = x_n;
      {                                                   // prefetch the next chunk's metadata
        const int nx = my + G;
        r_n = -1;
        if (nx < e1) {
          r_n = a.rows[nx];
          if (by_key) key_n = a.keys[nx];
          if (kHasVals) x_n = a.vals[nx];
        }
      }
      // bag of this lane's entry: the largest f with offs[f] <= my.  Entries are walked in order,
      // so it is at or shortly after the bag of the last processed entry: a few linear steps,
      // then a binary search for the rare long run of empty bags.
      int bag_l = cur;
      if (my < e1) {
        int lo = cur;
#pragma unroll
        for (int step = 0; step < 4; ++step)
          if (offs[lo + 1] <= my) ++lo;
        if (offs[lo + 1] <= my) {
          int hi = f1;
          ++lo;
          while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (offs[mid] <= my) lo = mid; else hi = mid;
          }
        }
        bag_l = lo;
      }
      const int sh_l = by_key ? (int)((uint32_t)(mix64(key_l) >> 32) % (uint32_t)K) : bag_l % K;
      // publish (row, bag, shard, value) of this lane's entry; the group then reads entry j of the
      // chunk from slot j with one broadcast LDS read.  Same wave, program order: no barrier needed.
      meta[lane] = make_int4(r_l, bag_l, sh_l, __float_as_int(x_l));
      const int cnt = min(G, e1 - e);
#pragma unroll
      for (int j0 = 0; j0 < G; j0 += U) {
        if (j0 < cnt) {
          int4 md[U];
          float4 v[U];
          float wv[U];
#pragma unroll
          for (int i = 0; i < U; ++i) {
            md[i] = meta[g * G + j0 + i];
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            wv[i] = 0.f;
            if (j0 + i < cnt && md[i].x >= 0) {
              if (need_v) v[i] = ld4(a.emb + (int64_t)md[i].x * D + sub * 4);
              if (need_lr && sub == kLrLane) wv[i] = a.w[md[i].x];
            }
          }
#pragma unroll
          for (int i = 0; i < U; ++i) {
            if (j0 + i < cnt) {
              const int bag = md[i].y, s = md[i].z;
              while (cur < bag) {                          // close finished (possibly empty) bags
                close_bag();
                ++cur;
              }
              if (md[i].x >= 0) {
                const double xd = kHasVals ? (double)__int_as_float(md[i].w) : 1.0;
                const double xv[4] = {kHasVals ? xd * (double)v[i].x : (double)v[i].x, kHasVals ? xd * (double)v[i].y : (double)v[i].y,
                                      kHasVals ? xd * (double)v[i].z : (double)v[i].z, kHasVals ? xd * (double)v[i].w : (double)v[i].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[k] += xv[k];
                if (!kByKey) {
                  bag_sq += xv[0] * xv[0] + xv[1] * xv[1] + xv[2] * xv[2] + xv[3] * xv[3];
                  bag_lr += xd * (double)wv[i];
                  bag_dirty = true;
                  continue;
                }
                double q = 0.0;
                if (need_fm) {
                  double *dst = sum + s * P + sub;
#pragma unroll
                  for (int k = 0; k < 4; ++k) atomicAdd(dst + k * G, xv[k]);
                  q = group_sum<G>(xv[0] * xv[0] + xv[1] * xv[1] + xv[2] * xv[2] + xv[3] * xv[3]);
                }
                // one LDS instruction for both scalars: lane 0 adds the sum of squares, lane kLrLane
                // the LR term (the same lane when a row is a single lane wide)
                if (kLrLane == 0) {
                  if (need_fm && sub == 0) atomicAdd(sum + s * P + D, q);
                  if (need_lr && sub == 0) atomicAdd(sum + s * P + D + 1, xd * (double)wv[i]);
                } else if ((sub == 0 && need_fm) || (sub == kLrLane && need_lr)) {
                  atomicAdd(sum + s * P + D + sub, sub == 0 ? q : xd * (double)wv[i]);
                }
              }
            }
          }
        }
      }
    }
    while (cur < f1) {                                    // last bag of the range and empty ones after it
      close_bag();
      ++cur;
    }
  }
  __syncthreads();

  if (active) {
    if (need_fm) {
      for (int idx = tis * 4; idx < K * D; idx += nts * 4) {
        const int s = idx / D, d = idx % D;                 // d = 4*sub: columns d..d+3 sit at k*G + sub
        const double *row = sum + s * P + d / 4;
        st4(a.P_sum + ((int64_t)s * a.B + b) * D + d,
            make_float4((float)row[0], (float)row[G], (float)row[2 * G], (float)row[3 * G]));
      }
      for (int s = tis; s < K; s += nts) a.P_sq[(int64_t)s * a.B + b] = (float)sum[s * P + D];
    }
    if (need_lr)
      for (int s = tis; s < K; s += nts) a.P_lr[(int64_t)s * a.B + b] = (float)sum[s * P + D + 1];
  }
}

// Per-shard pooled partials [K,B,F,D] (small shapes only): one lane group per bag, one pass
// over the bag per shard.
template <int D>
__global__ __launch_bounds__(kBlock) void k_pool_dense(const FwdArgs a, float *__restrict__ P_pool) {
  constexpr int G = D / 4;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t bag = gid / G;
  const int sub = (int)(gid % G);
  const int64_t nbags = a.B * a.F;
  if (bag >= nbags) return;
  const int f = (int)(bag % a.F);
  const int e0 = a.offsets[bag], e1 = a.offsets[bag + 1];
  for (int s = 0; s < a.K; ++s) {
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int e = e0; e < e1; ++e) {
      const int r = a.rows[e];
      if (r < 0) continue;
      const int sh = a.policy == DES_SHARD_KEY_HASH ? (int)((uint32_t)(mix64(a.keys[e]) >> 32) % (uint32_t)a.K)
                                                     : f % a.K;
      if (sh != s) continue;
      const double x = a.vals ? (double)a.vals[e] : 1.0;
      const float4 v = ld4(a.emb + (int64_t)r * D + sub * 4);
      acc[0] += x * (double)v.x; acc[1] += x * (double)v.y; acc[2] += x * (double)v.z; acc[3] += x * (double)v.w;
    }
    st4(P_pool + ((int64_t)s * nbags + bag) * D + sub * 4,
        make_float4((float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]));
  }
}

template <int D>
void launch_forward(bool by_key, bool has_vals, dim3 grid, dim3 block, size_t shmem, hipStream_t s, const FwdArgs &a) {
  if (by_key) {
    if (has_vals) hipLaunchKernelGGL((k_forward<D, true, true>), grid, block, shmem, s, a);
    else hipLaunchKernelGGL((k_forward<D, true, false>), grid, block, shmem, s, a);
  } else {
    if (has_vals) hipLaunchKernelGGL((k_forward<D, false, true>), grid, block, shmem, s, a);
    else hipLaunchKernelGGL((k_forward<D, false, false>), grid, block, shmem, s, a);
  }
}

FwdArgs make_args(des_table *t, const des_batch_t *b, const int32_t *rows) {
  FwdArgs a;
  a.emb = t->cfg.emb; a.w = t->cfg.w;
  a.keys = b->keys; a.offsets = b->offsets; a.vals = b->vals; a.rows = rows;
  a.P_lr = a.P_sum = a.P_sq = a.pool = nullptr;
  a.B = b->B; a.F = b->F; a.K = t->cfg.num_shards; a.policy = t->cfg.shard_policy;
  a.acc_doubles = 0; a.lds_per_sample = 0; a.wps = 1;
  return a;
}

}  // namespace

des_status_t forward_launch(des_table *t, const des_batch_t *b, const int32_t *rows, float *P_lr, float *P_sum,
                            float *P_sq, float *pool, hipStream_t s) {
  if (b->B == 0) return DES_OK;
  FwdArgs a = make_args(t, b, rows);
  a.P_lr = P_lr; a.P_sum = P_sum; a.P_sq = P_sq; a.pool = pool;
  const int D = t->cfg.dim;
  // LDS per sample: K*(D+2) doubles of accumulators plus the sample's F+1 offsets.  Fewer
  // samples per workgroup (more waves per sample) when that is large, so that a CU still holds
  // several workgroups.
  const int64_t acc_doubles = (int64_t)align_up((size_t)a.K * (D + 2), 2);
  const int64_t per_sample = acc_doubles + ((int64_t)b->F + 2) / 2;
  if (per_sample * 8 + 16 * kBlock > 65536) return DES_ERR_INVALID_ARG;   // K*(dim+2) doubles + F+1 ints + 4 KB must fit 64 KB of LDS
  a.acc_doubles = (int)acc_doubles;
  a.lds_per_sample = (int)per_sample;
  int wps = 1;
  while (wps < 4 && (kBlock / kWave / wps) * per_sample * 8 > 40 * 1024) wps *= 2;
  const int64_t entries_per_sample = b->nnz / (b->B > 0 ? b->B : 1);
  if (entries_per_sample >= 2048 && wps < 4) wps = 4;       // very long samples: spread over the workgroup
  a.wps = wps;
  const int spb = kBlock / kWave / wps;
  const dim3 grid((unsigned)((b->B + spb - 1) / spb)), block(kBlock);
  const size_t shmem = 16 * (size_t)kBlock + (size_t)per_sample * 8 * spb;
  const bool by_key = a.policy == DES_SHARD_KEY_HASH;
  ProfScope ps(KID_FORWARD, s);
  switch (D) {
    case 4: launch_forward<4>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    case 8: launch_forward<8>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    case 16: launch_forward<16>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    case 32: launch_forward<32>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    case 64: launch_forward<64>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    case 128: launch_forward<128>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    case 256: launch_forward<256>(by_key, a.vals != nullptr, grid, block, shmem, s, a); break;
    default: return DES_ERR_INVALID_ARG;
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

des_status_t pool_dense_launch(des_table *t, const des_batch_t *b, const int32_t *rows, float *P_pool, hipStream_t s) {
  if (b->B == 0) return DES_OK;
  FwdArgs a = make_args(t, b, rows);
  const int D = t->cfg.dim;
  const int64_t threads = b->B * b->F * (D / 4);
  const dim3 grid((unsigned)((threads + kBlock - 1) / kBlock)), block(kBlock);
  ProfScope ps(KID_POOL_DENSE, s);
  switch (D) {
    case 4: hipLaunchKernelGGL(k_pool_dense<4>, grid, block, 0, s, a, P_pool); break;
    case 8: hipLaunchKernelGGL(k_pool_dense<8>, grid, block, 0, s, a, P_pool); break;
    case 16: hipLaunchKernelGGL(k_pool_dense<16>, grid, block, 0, s, a, P_pool); break;
    case 32: hipLaunchKernelGGL(k_pool_dense<32>, grid, block, 0, s, a, P_pool); break;
    case 64: hipLaunchKernelGGL(k_pool_dense<64>, grid, block, 0, s, a, P_pool); break;
    case 128: hipLaunchKernelGGL(k_pool_dense<128>, grid, block, 0, s, a, P_pool); break;
    case 256: hipLaunchKernelGGL(k_pool_dense<256>, grid, block, 0, s, a, P_pool); break;
    default: return DES_ERR_INVALID_ARG;
  }
  return hipGetLastError() == hipSuccess ? DES_OK : DES_ERR_DEVICE;
}

}  // namespace des
