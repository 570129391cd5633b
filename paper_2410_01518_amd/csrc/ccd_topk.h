// Exact top-k threshold selection inside one workgroup, shared by the NuC-slot job and the final selection.
//
// Keys are order-preserving 32-bit images of fp32 values.  An MSB-first radix select with digits of up to 11 bits
// (LDS histogram, one atomic per candidate key and pass) over the range the keys actually span yields the threshold
// key tau and the number `need` of keys equal to tau that still belong to the k largest: a token is selected iff key > tau, or key == tau and fewer than
// `need` equal tokens precede it in token order (lowest index wins ties).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ccd {

constexpr int kRadixBins = 2048;
constexpr int kCandMax = 256;   // at most this many keys left in the chosen bin: they are ranked directly

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

// Wave-wide inclusive scan in six data-parallel-primitive steps (shifts inside rows of 16 lanes, then the last lane of
// a row broadcast into the following rows): one ALU instruction per step where a cross-lane shuffle takes a round trip
// through the LDS pipeline.  `identity` fills the lanes a step has no source for.
template <class Op>
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, uint32_t identity, Op op) {
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x111, 0xf, 0xf, false));   // row_shr:1
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x112, 0xf, 0xf, false));   // row_shr:2
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x114, 0xf, 0xf, false));   // row_shr:4
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x118, 0xf, 0xf, false));   // row_shr:8
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x142, 0xa, 0xf, false));   // row_bcast:15
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x143, 0xc, 0xf, false));   // row_bcast:31
  return v;
}
// the operation over all 64 lanes, in every lane
template <class Op>
__device__ __forceinline__ uint32_t wave_reduce(uint32_t v, uint32_t identity, Op op) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_scan(v, identity, op), 63);
}

template <int THREADS>
struct TopkShared {
  uint32_t hist[kRadixBins];
  uint32_t wave_sum[2][THREADS / 64];   // ping-pong: one barrier per scan
  uint32_t red[4][THREADS / 64];        // per-wave class counts and key range of radix_threshold
  uint32_t digit, remaining;
  uint32_t bin_count, cand_n;           // keys in the chosen bin; candidates gathered so far
  uint32_t cand_key[kCandMax];          // the keys that share all digits fixed so far, once they are few
};

// Exclusive prefix sum of v over the workgroup in thread order; `total` receives the workgroup's sum.
template <int THREADS>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, TopkShared<THREADS>& sh, int& phase, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_inclusive_scan(v, 0u, [](uint32_t a, uint32_t b) { return a + b; });
  if (lane == 63) sh.wave_sum[phase][wave] = inc;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) {
    const uint32_t c = sh.wave_sum[phase][w];
    before += (w < wave) ? c : 0u;
    tot += c;
  }
  phase ^= 1;
  total = tot;
  return before + inc - v;
}

// Exclusive prefix count of a predicate (ballot/popcount inside the wave).
template <int THREADS>
__device__ __forceinline__ uint32_t block_rank(bool pred, TopkShared<THREADS>& sh, int& phase, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t bal = __ballot(pred);
  const uint32_t r = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 0) sh.wave_sum[phase][wave] = __popcll(bal);
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) {
    const uint32_t c = sh.wave_sum[phase][w];
    before += (w < wave) ? c : 0u;
    tot += c;
  }
  phase ^= 1;
  total = tot;
  return before + r;
}

// Threshold of the kk largest of the keys of tokens 0 .. n-1, 1 <= kk <= n.  Thread tid owns KPT tokens
// (n <= THREADS * KPT): tid + j*THREADS, or tid*KPT + j when BLOCKED; key_of(j, t) returns the key of the thread's
// j-th token t, which the caller holds in registers.
// On return #{key > tau} < kk <= #{key >= tau} and need = kk - #{key > tau}.  Ends with a barrier.
// ABOVE_LOW_ONLY: keys at or below the key of -inf never qualify (novelty: NaN and -inf map to key 0): kk is first
// cut down to the number of other keys, and if none is left nothing is selected (tau = 0xFFFFFFFF, need = 0).
//
// Scores of one row share a few exponents, and a quarter or half of them are the +inf of the NuC slots: the top
// 11 bits of such keys fall into a handful of histogram bins, and a wave's 64 LDS atomics on one address serialise
// (measured: 5.2 us for the first pass against 1.4 us for the later ones).  So the keys are first split into three
// classes by fixed bounds - at or above the key of +inf, at or below the key of -inf, ordinary - with counts and, for
// the ordinary ones, minimum and maximum from one workgroup reduction.  The class that holds the kk-th largest is
// known from the counts; inside it the digits are taken from key - lo over the range hi - lo actually spanned, most
// significant first, 11 bits at a time (fewer passes when the range is narrow, none when it is a single value).
template <int THREADS, int KPT, bool BLOCKED = false, bool ABOVE_LOW_ONLY = false, class KeyFn>
__device__ __forceinline__ void radix_threshold(KeyFn key_of, int n, uint32_t kk, TopkShared<THREADS>& sh, int& phase, uint32_t& tau,
                                uint32_t& need) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int kBinsPerThread = kRadixBins / THREADS;
  constexpr int kWaves = THREADS / 64;
  static_assert(THREADS >= kCandMax, "one thread ranks one candidate");
  constexpr uint32_t kHiFrom = 0xFF800000u;   // score_key(+inf)
  constexpr uint32_t kLoUpTo = 0x007FFFFFu;   // score_key(-inf)

  // class counts and the range of the ordinary keys
  uint32_t c_hi = 0, c_mid = 0, mn = 0xFFFFFFFFu, mx = 0u;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int t = BLOCKED ? tid * KPT + j : tid + j * THREADS;
    if (t < n) {
      const uint32_t key = key_of(j, t);
      const bool hi = key >= kHiFrom, mid = !hi && key > kLoUpTo;
      c_hi += hi ? 1u : 0u;
      c_mid += mid ? 1u : 0u;
      mn = mid ? min(mn, key) : mn;
      mx = mid ? max(mx, key) : mx;
    }
  }
  c_hi = wave_reduce(c_hi, 0u, [](uint32_t a, uint32_t b) { return a + b; });
  c_mid = wave_reduce(c_mid, 0u, [](uint32_t a, uint32_t b) { return a + b; });
  mn = wave_reduce(mn, 0xFFFFFFFFu, [](uint32_t a, uint32_t b) { return min(a, b); });
  mx = wave_reduce(mx, 0u, [](uint32_t a, uint32_t b) { return max(a, b); });
  for (int i = tid; i < kRadixBins; i += THREADS) sh.hist[i] = 0;
  if (lane == 0) {
    sh.red[0][wave] = c_hi;
    sh.red[1][wave] = c_mid;
    sh.red[2][wave] = mn;
    sh.red[3][wave] = mx;
  }
  __syncthreads();                             // wave results and the cleared histogram are visible
  uint32_t n_hi = 0, n_mid = 0;
  mn = 0xFFFFFFFFu;
  mx = 0u;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    n_hi += sh.red[0][w];
    n_mid += sh.red[1][w];
    mn = min(mn, sh.red[2][w]);
    mx = max(mx, sh.red[3][w]);
  }

  if (ABOVE_LOW_ONLY) {
    kk = min(kk, n_hi + n_mid);
    if (kk == 0) {                               // uniform
      __syncthreads();
      tau = 0xFFFFFFFFu;
      need = 0;
      return;
    }
  }
  // the class of the kk-th largest key: candidates are the keys in [lo, hi]; `remaining` of them are wanted
  uint32_t lo, hi, remaining;
  if (kk <= n_hi) {
    lo = kHiFrom; hi = 0xFFFFFFFFu; remaining = kk;
  } else if (kk <= n_hi + n_mid) {
    lo = mn; hi = mx; remaining = kk - n_hi;
  } else {
    lo = 0u; hi = kLoUpTo; remaining = kk - n_hi - n_mid;
  }
  int rem_bits = 32 - __clz(hi - lo);          // bits of key - lo not yet fixed (__clz(0) = 32)
  if (rem_bits == 0) __syncthreads();          // a single candidate value: no pass, but still end with a barrier
  uint32_t prefix = 0;                         // the fixed high bits of tau - lo, as a value (already shifted down)
#pragma unroll 1
  while (rem_bits > 0) {
    const int width = min(11, rem_bits), shift = rem_bits - width;
    const uint32_t dmask = (1u << width) - 1u;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int t = BLOCKED ? tid * KPT + j : tid + j * THREADS;
      if (t < n) {
        const uint32_t key = key_of(j, t);
        const uint32_t rel = key - lo;
        if (key >= lo && key <= hi && (uint32_t)((uint64_t)rel >> rem_bits) == prefix)
          atomicAdd(&sh.hist[(rel >> shift) & dmask], 1u);
      }
    }
    __syncthreads();
    // thread 0 owns the highest bins: prefix sums in thread order are counts of larger digits.  Each thread
    // clears the bins it has read: the histogram is zero again before the next pass adds to it (two barriers on).
    uint32_t h[kBinsPerThread], mine = 0;
#pragma unroll
    for (int i = 0; i < kBinsPerThread; ++i) {
      const int bin = kRadixBins - 1 - (tid * kBinsPerThread + i);
      h[i] = sh.hist[bin];
      sh.hist[bin] = 0;
      mine += h[i];
    }
    uint32_t tot;
    uint32_t excl = block_exclusive_scan<THREADS>(mine, sh, phase, tot);
#pragma unroll
    for (int i = 0; i < kBinsPerThread; ++i) {
      const uint32_t incl = excl + h[i];
      if (excl < remaining && remaining <= incl) {
        sh.digit = kRadixBins - 1 - (tid * kBinsPerThread + i);
        sh.remaining = remaining - excl;
        sh.bin_count = h[i];
        sh.cand_n = 0;
      }
      excl = incl;
    }
    __syncthreads();
    prefix = (prefix << width) | sh.digit;
    remaining = sh.remaining;
    rem_bits = shift;
    const uint32_t n_cand = sh.bin_count;
    if (rem_bits > 0 && n_cand <= (uint32_t)kCandMax) {      // uniform over the workgroup
      // Few keys share the digits fixed so far (the digits are spread over the range, so this is the rule after one
      // pass): gather them and rank them against each other instead of two more histogram passes.
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const int t = BLOCKED ? tid * KPT + j : tid + j * THREADS;
        if (t < n) {
          const uint32_t key = key_of(j, t);
          const uint32_t rel = key - lo;
          if (key >= lo && key <= hi && (uint32_t)((uint64_t)rel >> rem_bits) == prefix)
            sh.cand_key[atomicAdd(&sh.cand_n, 1u)] = key;
        }
      }
      __syncthreads();
      if ((uint32_t)tid < n_cand) {
        const uint32_t mine = sh.cand_key[tid];
        uint32_t gt = 0, ge = 0;
        for (uint32_t i = 0; i < n_cand; ++i) {
          const uint32_t other = sh.cand_key[i];
          gt += other > mine ? 1u : 0u;
          ge += other >= mine ? 1u : 0u;
        }
        if (gt < remaining && remaining <= ge) {             // the threshold key (equal keys write the same values)
          sh.digit = mine;
          sh.remaining = remaining - gt;
        }
      }
      __syncthreads();
      tau = sh.digit;
      need = sh.remaining;
      return;
    }
  }
  tau = lo + prefix;
  need = remaining;
}

}  // namespace ccd
