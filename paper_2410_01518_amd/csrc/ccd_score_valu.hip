// Representative score of Eq. 2 on the vector ALUs: the path for fp32 caches and the plain-ALU
// comparison point for the MFMA kernels.  Two passes over K, because the attention probability of a
// CaP query on a token needs that query's normaliser over ALL cached tokens before the sum over queries
// can be taken:
//   pass 1 (stats): per (unit, token slice, query) running max m and Z = sum 2^(x - m) of the log2-domain
//                   logits x = <q, k_t> * scale * log2(e)        [thread = query, K tile in LDS]
//   merge:          lse2[q] = log2 sum_t 2^x over all slices
//   pass 2 (prob):  u_t = sum_q 2^(x - lse2[q])                  [thread = token, Q tile in LDS]
#include "ccd_common.h"

namespace ccd {

namespace {

constexpr int kThreads = 256;
constexpr int kTokTile = 32;    // tokens of K staged in LDS per step of pass 1
constexpr int kQryTile = 32;    // query rows staged in LDS per step of pass 2

template <typename T, int HD>
__global__ __launch_bounds__(kThreads) void stats_valu_kernel(Dims D, ScorePlan pl, const T* __restrict__ Q,
                                                              const T* __restrict__ K, float2* __restrict__ part) {
  __shared__ float4 Ks[kTokTile][HD / 4];
  __shared__ float2 red[kThreads];
  const int slice = blockIdx.x % pl.n_slices1, unit = D.unit0 + blockIdx.x / pl.n_slices1, tid = threadIdx.x;
  const UnitIdx ui = decode_unit(D, unit);
  const T* Ku = K + kv_offset(D, ui);
  const int t0 = slice * pl.slice1;
  const int t1 = min(D.n, t0 + pl.slice1);

  // Fewer query rows than threads: the threads form kThreads / qw groups that share the tokens of a tile
  // (group g takes the tokens g, g + groups, ...) and merge their (m, Z) pairs at the end of the slice.
  int qw = kThreads;
  while (qw / 2 >= D.GP) qw >>= 1;
  const int groups = kThreads / qw, grp = tid / qw, ql = tid - grp * qw;

  for (int q0 = 0; q0 < D.GP; q0 += qw) {
    const int q = q0 + ql;
    const bool active = q < D.GP;
    float4 qr[HD / 4];
    if (active) {
      const T* qp = Q + q_offset(D, ui, q);
#pragma unroll
      for (int c = 0; c < HD / 4; ++c) qr[c] = load4(qp + 4 * c);
    } else {
#pragma unroll
      for (int c = 0; c < HD / 4; ++c) qr[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float m = -INFINITY, Z = 0.f;
    // sliding window: the first cached token this query sees (0 without a window)
    const int first = D.window > 0 ? max(0, D.win_off + q % D.P) : 0;
    for (int tt = t0; tt < t1; tt += kTokTile) {
      __syncthreads();
      for (int e = tid; e < kTokTile * (HD / 4); e += kThreads) {
        const int t = e / (HD / 4), c = e - t * (HD / 4);
        const int tok = tt + t;
        Ks[t][c] = tok < t1 ? load4(Ku + (int64_t)tok * HD + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      __syncthreads();
      const int nt = min(kTokTile, t1 - tt);
      if (active) {
        for (int t = grp; t < nt; t += groups) {
          if (tt + t < first) continue;
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < HD / 4; ++c) {
            const float4 kk = Ks[t][c];
            acc = fmaf(qr[c].x, kk.x, acc);
            acc = fmaf(qr[c].y, kk.y, acc);
            acc = fmaf(qr[c].z, kk.z, acc);
            acc = fmaf(qr[c].w, kk.w, acc);
          }
          const float x = acc * D.scale_log2;
          if (x > m) {
            Z = Z * fast_exp2(m - x) + 1.f;
            m = x;
          } else {
            Z += fast_exp2(x - m);
          }
        }
      }
    }
    if (groups > 1) {            // (uniform over the workgroup)
      __syncthreads();
      red[tid] = make_float2(m, Z);
      __syncthreads();
      if (grp == 0) {
        for (int g = 1; g < groups; ++g) m = fmaxf(m, red[g * qw + ql].x);
        float z = 0.f;
        for (int g = 0; g < groups; ++g) {
          const float2 v = red[g * qw + ql];
          if (v.y > 0.f) z += v.y * fast_exp2(v.x - m);     // (a group that saw no token holds (-inf, 0))
        }
        Z = z;
      }
    }
    if (active && grp == 0) part[((int64_t)unit * pl.n_slices1 + slice) * D.GP + q] = make_float2(m, Z);
  }
}

// Statistics of the CaP keys' block (causal variant of Eq. 2): query row q = g * P + i sees the CaP keys 0 .. i.
// One workgroup per unit; the result goes behind the slices' statistics in `part`.
template <typename T, int HD>
__global__ __launch_bounds__(kThreads) void cap_block_stats_valu_kernel(Dims D, ScorePlan pl, const T* __restrict__ Q,
                                                                        const T* __restrict__ Kcap,
                                                                        float2* __restrict__ part) {
  __shared__ float4 Ks[kTokTile][HD / 4];
  const int unit = D.unit0 + blockIdx.x, tid = threadIdx.x;
  const UnitIdx ui = decode_unit(D, unit);
  const T* Kc = Kcap + (int64_t)unit * D.P * HD;
  for (int q0 = 0; q0 < D.GP; q0 += kThreads) {
    const int q = q0 + tid;
    const bool active = q < D.GP;
    const int i = q % D.P;                       // CaP position of the query
    float4 qr[HD / 4];
    if (active) {
      const T* qp = Q + q_offset(D, ui, q);
#pragma unroll
      for (int c = 0; c < HD / 4; ++c) qr[c] = load4(qp + 4 * c);
    } else {
#pragma unroll
      for (int c = 0; c < HD / 4; ++c) qr[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float m = -INFINITY, Z = 0.f;
    for (int jj = 0; jj < D.P; jj += kTokTile) {
      __syncthreads();
      for (int e = tid; e < kTokTile * (HD / 4); e += kThreads) {
        const int t = e / (HD / 4), c = e - t * (HD / 4);
        Ks[t][c] = jj + t < D.P ? load4(Kc + (int64_t)(jj + t) * HD + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      __syncthreads();
      const int nt = active ? min(kTokTile, i + 1 - jj) : 0;      // keys jj .. jj + nt - 1 are visible
      for (int t = 0; t < nt; ++t) {
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < HD / 4; ++c) {
          const float4 kk = Ks[t][c];
          acc = fmaf(qr[c].x, kk.x, acc);
          acc = fmaf(qr[c].y, kk.y, acc);
          acc = fmaf(qr[c].z, kk.z, acc);
          acc = fmaf(qr[c].w, kk.w, acc);
        }
        const float x = acc * D.scale_log2;
        if (x > m) {
          Z = Z * fast_exp2(m - x) + 1.f;
          m = x;
        } else {
          Z += fast_exp2(x - m);
        }
      }
    }
    if (active) part[extra_block_index(D, pl, unit, q)] = make_float2(m, Z);
  }
}

__global__ __launch_bounds__(kThreads) void merge_kernel(Dims D, ScorePlan pl, const float2* __restrict__ part,
                                                         float* __restrict__ lse2) {
  const int qblocks = (D.GP + kThreads - 1) / kThreads;
  const int unit = D.unit0 + blockIdx.x / qblocks;
  const int q = (blockIdx.x % qblocks) * kThreads + threadIdx.x;
  if (q >= D.GP) return;
  const float2* p = part + (int64_t)unit * pl.n_slices1 * D.GP + q;
  float M = -INFINITY, Z = 0.f;
  if (pl.cap_block) M = part[extra_block_index(D, pl, unit, q)].x;
  for (int j = 0; j < pl.n_slices1; ++j) M = fmaxf(M, p[(int64_t)j * D.GP].x);
  if (pl.cap_block) {
    const float2 v = part[extra_block_index(D, pl, unit, q)];
    Z = v.y * fast_exp2(v.x - M);
  }
  for (int j = 0; j < pl.n_slices1; ++j) {
    const float2 v = p[(int64_t)j * D.GP];
    if (!(v.y == 0.f)) Z += v.y * fast_exp2(v.x - M);   // a slice may lie outside the query's window: (-inf, 0)
  }
  // a query that sees no key at all (window == P at most, no CaP keys): +inf, every probability comes out 0
  lse2[(int64_t)unit * D.GP + q] = Z == 0.f ? INFINITY : M + __log2f(Z);
}

template <typename T, int HD>
__global__ __launch_bounds__(kThreads) void prob_valu_kernel(Dims D, ScorePlan pl, const T* __restrict__ Q,
                                                             const T* __restrict__ K, const float* __restrict__ lse2,
                                                             float lse_mul, float* __restrict__ u) {
  __shared__ float4 Qs[kQryTile][HD / 4];
  __shared__ float Ls[kQryTile];
  const int unit = D.unit0 + blockIdx.x / pl.n_slices2, tid = threadIdx.x;
  const UnitIdx ui = decode_unit(D, unit);
  const int tok = (blockIdx.x % pl.n_slices2) * kThreads + tid;   // one token per thread
  const bool active = tok < D.n;
  float4 kr[HD / 4];
  if (active) {
    const T* kp = K + kv_offset(D, ui) + (int64_t)tok * HD;
#pragma unroll
    for (int c = 0; c < HD / 4; ++c) kr[c] = load4(kp + 4 * c);
  } else {
#pragma unroll
    for (int c = 0; c < HD / 4; ++c) kr[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float acc_u = 0.f;
  for (int q0 = 0; q0 < D.GP; q0 += kQryTile) {
    __syncthreads();
    for (int e = tid; e < kQryTile * (HD / 4); e += kThreads) {
      const int qi = e / (HD / 4), c = e - qi * (HD / 4);
      const int q = q0 + qi;
      Qs[qi][c] = q < D.GP ? load4(Q + q_offset(D, ui, q) + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (tid < kQryTile) Ls[tid] = (q0 + tid) < D.GP ? lse2[(int64_t)unit * D.GP + q0 + tid] * lse_mul : INFINITY;
    __syncthreads();
    const int nq = min(kQryTile, D.GP - q0);
    for (int qi = 0; qi < nq; ++qi) {
      if (D.window > 0 && tok < D.win_off + (q0 + qi) % D.P) continue;   // outside this query's window
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < HD / 4; ++c) {
        const float4 qq = Qs[qi][c];
        acc = fmaf(qq.x, kr[c].x, acc);
        acc = fmaf(qq.y, kr[c].y, acc);
        acc = fmaf(qq.z, kr[c].z, acc);
        acc = fmaf(qq.w, kr[c].w, acc);
      }
      acc_u += fast_exp2(fmaf(acc, D.scale_log2, -Ls[qi]));
    }
  }
  if (active) u[(int64_t)unit * D.n + tok] = acc_u;
}

}  // namespace

void launch_stats_valu(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s) {
  dim3 grid((unsigned)pl.n_slices1 * D.units_run), block(kThreads);
#define CCD_LAUNCH(T, HD) \
  launch((stats_valu_kernel<T, HD>), grid, block, s, D, pl, (const T*)Q, (const T*)K, part)
  if (D.dtype == 0) { if (D.d == 64) CCD_LAUNCH(float, 64); else CCD_LAUNCH(float, 128); }
  else              { if (D.d == 64) CCD_LAUNCH(uint16_t, 64); else CCD_LAUNCH(uint16_t, 128); }
#undef CCD_LAUNCH
}

void launch_cap_block_stats_valu(const Dims& D, const ScorePlan& pl, const void* Q, const void* K_cap, float2* part,
                                 hipStream_t s) {
  dim3 grid((unsigned)D.units_run), block(kThreads);
#define CCD_LAUNCH(T, HD) \
  launch((cap_block_stats_valu_kernel<T, HD>), grid, block, s, D, pl, (const T*)Q, (const T*)K_cap, part)
  if (D.dtype == 0) { if (D.d == 64) CCD_LAUNCH(float, 64); else CCD_LAUNCH(float, 128); }
  else              { if (D.d == 64) CCD_LAUNCH(uint16_t, 64); else CCD_LAUNCH(uint16_t, 128); }
#undef CCD_LAUNCH
}

void launch_merge(const Dims& D, const ScorePlan& pl, const float2* part, float* lse2, hipStream_t s) {
  dim3 grid((unsigned)((D.GP + kThreads - 1) / kThreads) * D.units_run), block(kThreads);
  launch(merge_kernel, grid, block, s, D, pl, part, lse2);
}

void launch_prob_valu(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const float* lse2, float* u,
                      hipStream_t s) {
  dim3 grid((unsigned)pl.n_slices2 * D.units_run), block(kThreads);
  const float lse_mul = pl.lse_given ? 1.44269504088896340736f : 1.0f;
#define CCD_LAUNCH(T, HD) \
  launch((prob_valu_kernel<T, HD>), grid, block, s, D, pl, (const T*)Q, (const T*)K, lse2, lse_mul, u)
  if (D.dtype == 0) { if (D.d == 64) CCD_LAUNCH(float, 64); else CCD_LAUNCH(float, 128); }
  else              { if (D.d == 64) CCD_LAUNCH(uint16_t, 64); else CCD_LAUNCH(uint16_t, 128); }
#undef CCD_LAUNCH
}

}  // namespace ccd
