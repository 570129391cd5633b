// NuC score from the model's logits (Sec. 3.3.2, Eq. 3; App. B "Calculate NuC Score"): the novelty of a token is its
// cross entropy under the model,
//     novelty[r] = log(sum_v exp(z[r][v])) - z[r][label[r]],
// where row r of the logits is the prediction FOR label r (the caller aligns them).  A label outside [0, V) marks a
// token without a prediction: novelty -inf, which never takes a NuC slot.
//
// One workgroup per row.  The row (V elements: 64 KiB - 256 KiB for today's vocabularies) is streamed once, 16 bytes
// per lane and load, each thread keeping a running (maximum, sum of exp2 relative to it) pair that is rescaled only
// per 16-byte chunk; the pairs are merged across the wave by shuffles and across waves through LDS.  The kernel is
// HBM-bound: one exp2, one fma and one add per element against 2 (bf16) or 4 (fp32) bytes read.
#include "ccd_common.h"

namespace ccd {

namespace {

constexpr int kNucThreads = 256;
constexpr int kNucLoads = 4;            // 16-byte loads a thread keeps in flight
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;
constexpr float kLowest = -3.0e38f;     // finite stand-in for "no value yet": keeps (m - m_new) free of inf - inf

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct MaxSum { float m, s; };          // s = sum of 2^((x - m) * log2 e)

__device__ __forceinline__ MaxSum merge(MaxSum a, MaxSum b) {
  const float m = fmaxf(a.m, b.m);
  return {m, a.s * fast_exp2((a.m - m) * kLog2e) + b.s * fast_exp2((b.m - m) * kLog2e)};
}

template <int N>
__device__ __forceinline__ void fold(MaxSum& acc, const float (&x)[N]) {
  float cm = x[0];
#pragma unroll
  for (int i = 1; i < N; ++i) cm = fmaxf(cm, x[i]);
  const float m = fmaxf(acc.m, cm);
  float s = acc.s * fast_exp2((acc.m - m) * kLog2e);
#pragma unroll
  for (int i = 0; i < N; ++i) s += fast_exp2((x[i] - m) * kLog2e);   // difference first: exact for nearby values
  acc.m = m;
  acc.s = s;
}

template <bool BF16>
__global__ __launch_bounds__(kNucThreads) void nuc_from_logits_kernel(const char* __restrict__ logits,
                                                                      const int32_t* __restrict__ labels,
                                                                      float* __restrict__ novelty, int V,
                                                                      int64_t row_stride_bytes) {
  constexpr int kEPC = BF16 ? 8 : 4;                            // elements per 16-byte chunk
  __shared__ MaxSum wave_acc[kNucThreads / 64];
  const int64_t r = blockIdx.x;
  const char* row = logits + r * row_stride_bytes;
  const int label = labels[r];
  const int n_chunks = V / kEPC;
  MaxSum acc{kLowest, 0.f};
  for (int c0 = threadIdx.x; c0 < n_chunks; c0 += kNucThreads * kNucLoads) {
    u32x4 v[kNucLoads];
#pragma unroll
    for (int i = 0; i < kNucLoads; ++i) {
      const int c = c0 + i * kNucThreads;
      if (c < n_chunks) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row) + c);   // read once
    }
#pragma unroll
    for (int i = 0; i < kNucLoads; ++i) {
      if (c0 + i * kNucThreads < n_chunks) {
        float x[kEPC];
        const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        if (BF16) {
#pragma unroll
          for (int j = 0; j < 4; ++j) { x[2 * j] = __uint_as_float(w[j] << 16); x[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u); }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(w[j]);
        }
        fold(acc, x);
      }
    }
  }
  // the last V % kEPC elements, one per thread
  const int t = n_chunks * kEPC + threadIdx.x;
  if (t < V) {
    float x[1];
    x[0] = BF16 ? bf16_bits_to_float(reinterpret_cast<const uint16_t*>(row)[t]) : reinterpret_cast<const float*>(row)[t];
    fold(acc, x);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc = merge(acc, MaxSum{__shfl_xor(acc.m, off), __shfl_xor(acc.s, off)});
  if ((threadIdx.x & 63) == 0) wave_acc[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    MaxSum a = wave_acc[0];
#pragma unroll
    for (int w = 1; w < kNucThreads / 64; ++w) a = merge(a, wave_acc[w]);
    float out = -INFINITY;
    if (label >= 0 && label < V) {
      const float zl = BF16 ? bf16_bits_to_float(reinterpret_cast<const uint16_t*>(row)[label])
                            : reinterpret_cast<const float*>(row)[label];
      out = (a.m + __log2f(a.s) * kLn2) - zl;      // log-sum-exp in natural units, then the label's logit
    }
    novelty[r] = out;
  }
}

}  // namespace

void launch_nuc_from_logits(const void* logits, const int32_t* labels, float* novelty, int64_t rows, int V,
                            int64_t row_stride_elems, int dtype, hipStream_t s) {
  const dim3 grid((unsigned)rows), block(kNucThreads);
  if (dtype == 1)
    launch((nuc_from_logits_kernel<true>), grid, block, s, (const char*)logits, labels, novelty, V,
                       row_stride_elems * 2);
  else
    launch((nuc_from_logits_kernel<false>), grid, block, s, (const char*)logits, labels, novelty, V,
                       row_stride_elems * 4);
}

}  // namespace ccd
