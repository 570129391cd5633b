// Per-unit selection kernels: NuC slots (Sec. 3.3.3 step 1), pooling + NuC lift, and the final top-k
// (Sec. 3.3.3 step 2 / App. B "Final Token Selection").
//
// Both "top" operations are exact selections with a lowest-index tie-break.  They are done as an MSB-first
// radix select on order-preserving 32-bit keys (four 8-bit digits, histogram in LDS) that yields the threshold
// key tau and the number `need` of tokens equal to tau that still belong to the set; a token is selected iff
// key > tau, or key == tau and fewer than `need` equal tokens precede it.  The "precede" rank and the output
// slot of each kept token come from ballot/popcount prefix counts taken in token order, which also emits
// keep_idx in ascending order without a sort.  One workgroup per unit.
#include <float.h>

#include "ccd_common.h"

namespace ccd {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

struct SelShared {
  uint32_t hist[256];
  uint32_t wave_cnt[kSelWaves];
  uint32_t digit;
  uint32_t remaining;
};

// fp32 -> uint32 with the same order; NaN ranks with -inf and -0 equals +0
__device__ __forceinline__ uint32_t score_key(float x) {
  if (x != x) x = -INFINITY;
  x += 0.0f;
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
// novelty key: NaN and -inf map to 0, strictly below every token that may take a NuC slot
__device__ __forceinline__ uint32_t novelty_key(float x) {
  if (x != x || x == -INFINITY) return 0u;
  return score_key(x);
}

// Exclusive prefix count of `pred` over the workgroup in thread order; `total` receives the workgroup's count.
__device__ __forceinline__ uint32_t block_rank(bool pred, SelShared& sh, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t bal = __ballot(pred);
  const uint32_t r = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 0) sh.wave_cnt[wave] = __popcll(bal);
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const uint32_t c = sh.wave_cnt[w];
    before += (w < wave) ? c : 0u;
    tot += c;
  }
  __syncthreads();
  total = tot;
  return before + r;
}

// Threshold of the kk largest keys among key_of(0..n-1), 1 <= kk <= n.
// On return: #{key > tau} < kk <= #{key >= tau} and need = kk - #{key > tau}.
template <class KeyFn>
__device__ void radix_threshold(KeyFn key_of, int n, uint32_t kk, SelShared& sh, uint32_t& tau, uint32_t& need) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, mask = 0, remaining = kk;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) sh.hist[tid] = 0;
    __syncthreads();
    for (int t = tid; t < n; t += kSelThreads) {
      const uint32_t key = key_of(t);
      if ((key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {
      // lane owns digits 4*lane .. 4*lane+3; suffix sums over lanes give the count of larger digits
      uint32_t h[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) h[j] = sh.hist[4 * tid + j];
      const uint32_t mine = h[0] + h[1] + h[2] + h[3];
      uint32_t suf = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_down(suf, off);
        if (tid + off < 64) suf += o;
      }
      uint32_t excl = suf - mine;
#pragma unroll
      for (int j = 3; j >= 0; --j) {
        const uint32_t incl = excl + h[j];
        if (excl < remaining && remaining <= incl) {
          sh.digit = 4 * tid + j;
          sh.remaining = remaining - excl;
        }
        excl = incl;
      }
    }
    __syncthreads();
    prefix |= sh.digit << shift;
    mask |= 0xFFu << shift;
    remaining = sh.remaining;
  }
  __syncthreads();
  tau = prefix;
  need = remaining;
}

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

// u != nullptr: scores <- NuC lift of pooled u.   keep_idx != nullptr: keep_idx <- top-k of scores.
__global__ __launch_bounds__(kSelThreads) void finalize_select_kernel(Dims D, const float* __restrict__ u,
                                                                      const float* __restrict__ novelty,
                                                                      float* scores, int32_t* __restrict__ keep_idx) {
  __shared__ SelShared sh;
  const int unit = blockIdx.x, tid = threadIdx.x, n = D.n;
  float* sc = scores + (int64_t)unit * n;
  const int rounds = (n + kSelThreads - 1) / kSelThreads;

  if (u != nullptr) {
    const float* uu = u + (int64_t)unit * n;
    const float* nov = novelty + nov_offset(D, decode_unit(D, unit));
    uint32_t T_eff = 0, tau_n = 0xFFFFFFFFu, need_n = 0;
    if (D.T > 0) {
      uint32_t cnt = 0;
      for (int t = tid; t < n; t += kSelThreads) cnt += novelty_key(nov[t]) != 0u;
      // workgroup sum of cnt through the rank helper, one bit at a time would be slow: use LDS atomics
      if (tid == 0) sh.remaining = 0;
      __syncthreads();
      if (cnt) atomicAdd(&sh.remaining, cnt);
      __syncthreads();
      T_eff = min((uint32_t)D.T, sh.remaining);
      __syncthreads();
      if (T_eff > 0) radix_threshold([&](int t) { return novelty_key(nov[t]); }, n, T_eff, sh, tau_n, need_n);
    }
    uint32_t eq_base = 0;
    for (int r = 0; r < rounds; ++r) {
      const int t = r * kSelThreads + tid;
      bool nuc = false;
      if (T_eff > 0) {
        const uint32_t key = t < n ? novelty_key(nov[t]) : 0u;
        const bool eq = t < n && key == tau_n;
        uint32_t tot;
        const uint32_t rank = block_rank(eq, sh, tot);
        nuc = t < n && (key > tau_n || (eq && eq_base + rank < need_n));
        eq_base += tot;
      }
      if (t < n) {
        float v = pooled(uu, t, n, D.pool_w, D.pool_mode);
        if (fabsf(v) < FLT_MIN) v = 0.f;
        sc[t] = nuc ? INFINITY : v;
      }
    }
    __syncthreads();
  }

  if (keep_idx != nullptr) {
    int32_t* out = keep_idx + (int64_t)unit * D.k;
    uint32_t tau, need;
    radix_threshold([&](int t) { return score_key(sc[t]); }, n, (uint32_t)D.k, sh, tau, need);
    uint32_t eq_base = 0, out_base = 0;
    for (int r = 0; r < rounds; ++r) {
      const int t = r * kSelThreads + tid;
      const uint32_t key = t < n ? score_key(sc[t]) : 0u;
      const bool eq = t < n && key == tau;
      uint32_t tot;
      const uint32_t erank = block_rank(eq, sh, tot);
      const bool sel = t < n && (key > tau || (eq && eq_base + erank < need));
      eq_base += tot;
      const uint32_t srank = block_rank(sel, sh, tot);
      if (sel) out[out_base + srank] = t;
      out_base += tot;
    }
  }
}

}  // namespace

void launch_finalize_select(const Dims& D, const float* u, const float* novelty, float* scores, int32_t* keep_idx,
                            hipStream_t s) {
  hipLaunchKernelGGL(finalize_select_kernel, dim3(D.units), dim3(kSelThreads), 0, s, D, u, novelty, scores, keep_idx);
}

}  // namespace ccd
