// Pooling + NuC lift + final top-k of one unit (Sec. 3.3.3 step 2), as a workgroup-level device function.
#pragma once
#include <float.h>

#include "ccd_common.h"
#include "ccd_topk.h"

namespace ccd {

__device__ __forceinline__ float pooled(const float* __restrict__ u, int t, int n, int w, int mode) {
  if (mode == 0 || w <= 1) return u[t];
  const int r = w >> 1;
  const int lo = max(0, t - r), hi = min(n - 1, t + r);
  if (mode == 1) {
    float m = u[lo];
    for (int j = lo + 1; j <= hi; ++j) m = fmaxf(m, u[j]);
    return m;
  }
  float s = 0.f;
  for (int j = lo; j <= hi; ++j) s += u[j];
  return s / (float)w;
}

// u != nullptr: score <- NuC lift (mask) of pooled u, written to `scores` if that is not null.
// u == nullptr: score <- scores (must not be null).      keep_idx != nullptr: keep_idx <- top-k of score.
// Executed by a whole workgroup of THREADS threads; thread t owns tokens t, t+THREADS, ... (at most KPT of them).
// u_stage (LDS, n floats, or null): the unit's row of u is copied there first, so that the pooling window reads
// LDS instead of issuing a chain of dependent global loads per token.
template <int THREADS, int KPT>
__device__ __forceinline__ void finalize_select_body(const Dims& D, int unit, const float* __restrict__ u,
                                                     const uint8_t* __restrict__ mask, float* scores,
                                                     int32_t* __restrict__ keep_idx, TopkShared<THREADS>& sh,
                                                     float* u_stage) {
  const int tid = threadIdx.x, n = D.n;
  int phase = 0;
  float sc[KPT];
  if (u != nullptr) {
    const float* uu = u + (int64_t)unit * n;
    if (u_stage != nullptr && D.pool_mode != 0 && D.pool_w > 1) {
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const int t = tid + j * THREADS;
        if (t < n) u_stage[t] = uu[t];
      }
      __syncthreads();
      uu = u_stage;
    }
    const bool shared_nov = D.nov_sl == 0 && D.nov_sh == 0;
    const uint8_t* mrow = mask + (int64_t)(shared_nov ? decode_unit(D, unit).b : unit) * n;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int t = tid + j * THREADS;
      sc[j] = -INFINITY;
      if (t < n) {
        float v = pooled(uu, t, n, D.pool_w, D.pool_mode);
        if (fabsf(v) < FLT_MIN) v = 0.f;
        sc[j] = (D.T > 0 && mrow[t]) ? INFINITY : v;
        if (scores != nullptr) scores[(int64_t)unit * n + t] = sc[j];
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int t = tid + j * THREADS;
      sc[j] = t < n ? scores[(int64_t)unit * n + t] : -INFINITY;
    }
  }

  if (keep_idx != nullptr) {
    int32_t* out = keep_idx + (int64_t)unit * D.k;
    uint32_t key[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) key[j] = score_key(sc[j]);
    uint32_t tau, need;
    radix_threshold<THREADS, KPT>([&](int j, int) { return key[j]; }, n, (uint32_t)D.k, sh, phase, tau, need);
    uint32_t eq_base = 0, out_base = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      if (j * THREADS >= n) continue;      // uniform: whole rounds beyond n are skipped
      const int t = tid + j * THREADS;
      const bool eq = t < n && key[j] == tau;
      uint32_t tot;
      const uint32_t erank = block_rank<THREADS>(eq, sh, phase, tot);
      const bool sel = t < n && (key[j] > tau || (eq && eq_base + erank < need));
      eq_base += tot;
      const uint32_t srank = block_rank<THREADS>(sel, sh, phase, tot);
      if (sel) out[out_base + srank] = t;
      out_base += tot;
    }
  }
}

}  // namespace ccd
