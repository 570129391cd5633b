// Per-unit selection kernels: NuC slots (Sec. 3.3.3 step 1), pooling + NuC lift, and the final top-k
// (Sec. 3.3.3 step 2 / App. B "Final Token Selection").  The selection machinery is in ccd_topk.h.
//
// finalize_select_kernel: one workgroup of 1024 threads per unit; thread t owns tokens t, t+1024, ... and keeps
// their scores in registers.  Ballot/popcount prefix counts taken in token order give both the lowest-index
// tie-break and the output slot of every kept token, so keep_idx comes out ascending without a sort.
#include <float.h>

#include "ccd_common.h"
#include "ccd_topk.h"

namespace ccd {

namespace {

constexpr int kSelThreads = 1024;

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

// one workgroup per novelty row: per sequence when novelty is shared by layers and heads, else per unit
__global__ __launch_bounds__(kSelThreads) void nuc_mask_kernel(Dims D, const float* __restrict__ novelty,
                                                               uint8_t* __restrict__ mask) {
  __shared__ TopkShared<kSelThreads> sh;
  const bool shared_nov = D.nov_sl == 0 && D.nov_sh == 0;
  const float* nov = novelty + (shared_nov ? (int64_t)blockIdx.x * D.nov_sb : nov_offset(D, decode_unit(D, blockIdx.x)));
  nuc_mask_job<kSelThreads>(nov, mask + (int64_t)blockIdx.x * D.n, D.n, D.T, sh);
}

// u != nullptr: score <- NuC lift (mask) of pooled u, written to `scores` if that is not null.
// u == nullptr: score <- scores (must not be null).      keep_idx != nullptr: keep_idx <- top-k of score.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void finalize_select_kernel(Dims D, const float* __restrict__ u,
                                                                      const uint8_t* __restrict__ mask, float* scores,
                                                                      int32_t* __restrict__ keep_idx) {
  __shared__ TopkShared<kSelThreads> sh;
  const int unit = D.unit0 + blockIdx.x, tid = threadIdx.x, n = D.n;
  int phase = 0;
  float sc[KPT];
  if (u != nullptr) {
    const float* uu = u + (int64_t)unit * n;
    const bool shared_nov = D.nov_sl == 0 && D.nov_sh == 0;
    const uint8_t* mrow = mask + (int64_t)(shared_nov ? decode_unit(D, unit).b : unit) * n;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int t = tid + j * kSelThreads;
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
      const int t = tid + j * kSelThreads;
      sc[j] = t < n ? scores[(int64_t)unit * n + t] : -INFINITY;
    }
  }

  if (keep_idx != nullptr) {
    int32_t* out = keep_idx + (int64_t)unit * D.k;
    uint32_t key[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) key[j] = score_key(sc[j]);
    uint32_t tau, need;
    radix_threshold<kSelThreads, KPT>([&](int j, int) { return key[j]; }, n, (uint32_t)D.k, sh, phase, tau, need);
    uint32_t eq_base = 0, out_base = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      if (j * kSelThreads >= n) break;
      const int t = tid + j * kSelThreads;
      const bool eq = t < n && key[j] == tau;
      uint32_t tot;
      const uint32_t erank = block_rank<kSelThreads>(eq, sh, phase, tot);
      const bool sel = t < n && (key[j] > tau || (eq && eq_base + erank < need));
      eq_base += tot;
      const uint32_t srank = block_rank<kSelThreads>(sel, sh, phase, tot);
      if (sel) out[out_base + srank] = t;
      out_base += tot;
    }
  }
}

}  // namespace

int select_max_tokens() { return 64 * kSelThreads; }

void launch_nuc_mask(const Dims& D, const float* novelty, uint8_t* mask, hipStream_t s) {
  const bool shared_nov = D.nov_sl == 0 && D.nov_sh == 0;
  hipLaunchKernelGGL(nuc_mask_kernel, dim3(shared_nov ? D.B : D.units), dim3(kSelThreads), 0, s, D, novelty, mask);
}

void launch_finalize_select(const Dims& D, const float* u, const uint8_t* mask, float* scores, int32_t* keep_idx,
                            hipStream_t s) {
  const dim3 grid(D.units_run), block(kSelThreads);
  const int kpt = (D.n + kSelThreads - 1) / kSelThreads;
#define CCD_LAUNCH(KPT) hipLaunchKernelGGL((finalize_select_kernel<KPT>), grid, block, 0, s, D, u, mask, scores, keep_idx)
  if (kpt <= 4) CCD_LAUNCH(4);
  else if (kpt <= 16) CCD_LAUNCH(16);
  else if (kpt <= 32) CCD_LAUNCH(32);
  else CCD_LAUNCH(64);
#undef CCD_LAUNCH
}

}  // namespace ccd
