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

// Token ownership inside the workgroup.  Striped: thread t owns tokens t, t+THREADS, ... (coalesced global access
// with any KPT).  Blocked: thread t owns the KPT consecutive tokens t*KPT ..: the pooling window of all of them is
// KPT + 2r consecutive values, and ranks in token order need one workgroup scan instead of one per round.
template <int THREADS, int KPT, bool BLOCKED>
__device__ __forceinline__ int owned_token(int tid, int j) { return BLOCKED ? tid * KPT + j : tid + j * THREADS; }

constexpr int kStagePad = 4;   // blocked pooling reads up to 4 tokens before and after a thread's tokens

// Pooled scores of the KPT consecutive tokens of one thread from the LDS copy of the row (token t at
// stage[t + kStagePad]), for windows of at most 2*kStagePad + 1: KPT/4 + 2 vector reads, the rest in registers.
template <int KPT>
__device__ __forceinline__ void pooled_block(float (&out)[KPT], const float* stage, int t0, int n, int w, int mode) {
  static_assert(KPT % 4 == 0, "vector reads of four tokens");
  float win[KPT + 2 * kStagePad];
#pragma unroll
  for (int i = 0; i < KPT / 4 + 2; ++i) {
    const float4 v = *reinterpret_cast<const float4*>(stage + t0 + 4 * i);   // tokens t0 - 4 + 4i ..
    win[4 * i] = v.x; win[4 * i + 1] = v.y; win[4 * i + 2] = v.z; win[4 * i + 3] = v.w;
  }
  const int r = w >> 1;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int t = t0 + j;
    float m = win[j + kStagePad], sum = 0.f;
#pragma unroll
    for (int o = -kStagePad; o <= kStagePad; ++o) {
      const bool in = o >= -r && o <= r && t + o >= 0 && t + o < n;
      const float v = win[j + kStagePad + o];
      m = in ? fmaxf(m, v) : m;
      sum += in ? v : 0.f;
    }
    out[j] = mode == 1 ? m : sum / (float)w;
  }
}

// NuC slots (Sec. 3.3.3 step 1): bit j of the result = the thread's j-th token is among the T tokens of largest
// novelty of the row `nov` (n values).  NaN and -inf never qualify, so fewer than T may be marked; ties go to the lower index.  The
// novelty keys stay in registers; the row is read once.  Every thread of the workgroup must call this.
template <int THREADS, int KPT, bool BLOCKED>
__device__ __forceinline__ uint64_t nuc_slots_of_row(const float* __restrict__ nov, int n, int T,
                                                     TopkShared<THREADS>& sh, int& phase) {
  static_assert(KPT <= 64, "one bit per owned token");
  const int tid = threadIdx.x;
  uint64_t nuc = 0;
  uint32_t key[KPT];
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int t = owned_token<THREADS, KPT, BLOCKED>(tid, j);
    key[j] = t < n ? novelty_key(nov[t]) : 0u;
  }
  uint32_t tau, need;
  radix_threshold<THREADS, KPT, BLOCKED, true>([&](int j, int) { return key[j]; }, n, (uint32_t)max(T, 0), sh, phase, tau, need);
  if (BLOCKED) {
    uint32_t n_eq = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) n_eq += (tid * KPT + j < n && key[j] == tau) ? 1u : 0u;
    uint32_t tot;
    uint32_t eq_rank = block_exclusive_scan<THREADS>(n_eq, sh, phase, tot);
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const bool valid = tid * KPT + j < n, eq = valid && key[j] == tau;
      nuc |= (uint64_t)(valid && (key[j] > tau || (eq && eq_rank < need))) << j;
      eq_rank += eq ? 1u : 0u;
    }
  } else {
    uint32_t eq_base = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      if (j * THREADS >= n) continue;      // uniform: whole rounds beyond n are skipped
      const int t = tid + j * THREADS;
      const bool eq = t < n && key[j] == tau;
      uint32_t tot;
      const uint32_t rank = block_rank<THREADS>(eq, sh, phase, tot);
      nuc |= (uint64_t)(t < n && (key[j] > tau || (eq && eq_base + rank < need))) << j;
      eq_base += tot;
    }
  }
  return nuc;
}

// u != nullptr: score <- pooled u with +inf at the NuC slots of the unit's novelty row (novelty may be null when
// D.T == 0), written to `scores` if that is not null.
// u == nullptr: score <- scores (must not be null).      keep_idx != nullptr: keep_idx <- top-k of score.
// Executed by a whole workgroup of THREADS threads, each owning at most KPT tokens (n <= THREADS * KPT).
// u_stage (LDS, THREADS * KPT + 2 * kStagePad floats, 16-byte aligned, or null): the unit's row of u is copied there
// first, so that the pooling window reads LDS instead of issuing a chain of dependent global loads per token.
// BLOCKED needs u_stage.  keep_lds (BLOCKED only, or null): a second copy of the kept indices, k entries in LDS; it
// may alias u_stage.  Ends without a barrier.
template <int THREADS, int KPT, bool BLOCKED>
__device__ __forceinline__ void finalize_select_body(const Dims& D, int unit, const float* __restrict__ u,
                                                     const float* __restrict__ novelty, float* scores,
                                                     int32_t* __restrict__ keep_idx, TopkShared<THREADS>& sh,
                                                     float* u_stage, int32_t* keep_lds = nullptr) {
  const int tid = threadIdx.x, n = D.n;
  int phase = 0;
  float sc[KPT];
  if (u != nullptr) {
    const float* uu = u + (int64_t)unit * n;
    const bool pooling = D.pool_mode != 0 && D.pool_w > 1;
    const bool stage = u_stage != nullptr && pooling;
    if (stage) {
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const int t = tid + j * THREADS;            // striped copy: coalesced
        if (t < n) u_stage[t + kStagePad] = uu[t];
      }
    }
    // the NuC slots of the row: the workgroup barriers inside also make the staged row visible
    uint64_t nuc = 0;
    if (D.T > 0) {
      nuc = nuc_slots_of_row<THREADS, KPT, BLOCKED>(novelty + nov_offset(D, decode_unit(D, unit)), n, D.T, sh, phase);
    } else if (stage) {
      __syncthreads();
    }
    if (stage) uu = u_stage + kStagePad;
    if (BLOCKED && pooling && D.pool_w <= 2 * kStagePad + 1) {
      pooled_block<KPT>(sc, u_stage, tid * KPT, n, D.pool_w, D.pool_mode);
    } else {
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const int t = owned_token<THREADS, KPT, BLOCKED>(tid, j);
        sc[j] = t < n ? pooled(uu, t, n, D.pool_w, D.pool_mode) : 0.f;
      }
    }
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int t = owned_token<THREADS, KPT, BLOCKED>(tid, j);
      float v = sc[j];
      sc[j] = -INFINITY;
      if (t < n) {
        if (fabsf(v) < FLT_MIN) v = 0.f;
        sc[j] = ((nuc >> j) & 1u) ? INFINITY : v;
        if (scores != nullptr) scores[(int64_t)unit * n + t] = sc[j];
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int t = owned_token<THREADS, KPT, BLOCKED>(tid, j);
      sc[j] = t < n ? scores[(int64_t)unit * n + t] : -INFINITY;
    }
  }

  if (keep_idx != nullptr || keep_lds != nullptr) {
    int32_t* out = keep_idx != nullptr ? keep_idx + (int64_t)unit * D.k : nullptr;
    uint32_t key[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) key[j] = score_key(sc[j]);
    uint32_t tau, need;
    radix_threshold<THREADS, KPT, BLOCKED, false>([&](int j, int) { return key[j]; }, n, (uint32_t)D.k, sh, phase, tau, need);
    if (BLOCKED) {
      // token order is thread order, then j.  A token's place among the kept ones is the number of larger keys
      // before it plus the number of threshold ties before it, capped at `need`: one scan over the two per-thread
      // counts packed into one word (blocked ownership is only used for n <= 32768, so both stay below 2^16)
      uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const bool valid = tid * KPT + j < n;
        n_gt += (valid && key[j] > tau) ? 1u : 0u;
        n_eq += (valid && key[j] == tau) ? 1u : 0u;
      }
      uint32_t tot;
      const uint32_t before = block_exclusive_scan<THREADS>((n_gt << 16) | n_eq, sh, phase, tot);
      uint32_t gt_rank = before >> 16, eq_rank = before & 0xFFFFu;
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const bool valid = tid * KPT + j < n;
        const bool gt = valid && key[j] > tau, eq = valid && key[j] == tau;
        if (gt || (eq && eq_rank < need)) {
          const uint32_t pos = gt_rank + min(eq_rank, need);
          if (out != nullptr) out[pos] = tid * KPT + j;
          if (keep_lds != nullptr) keep_lds[pos] = tid * KPT + j;
        }
        gt_rank += gt ? 1u : 0u;
        eq_rank += eq ? 1u : 0u;
      }
    } else {
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
}

}  // namespace ccd
