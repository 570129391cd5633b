// CR-RoPE (Sec. 3.5): the pot holds keys BEFORE the rotary embedding; after a distillation the kept keys get the
// rotary embedding of their new positions 0 .. |C|-1.  Dimension i is paired with dimension i + d/2 (the pairing of
// the LLaMA / Mistral models the paper evaluates):
//     y_i       = x_i * cos[p][i] - x_{i+d/2} * sin[p][i]
//     y_{i+d/2} = x_{i+d/2} * cos[p][i] + x_i * sin[p][i]
// Rows are handled 16 bytes per lane, ROWB/16 consecutive lanes per row: the lane that holds x_i .. and the lane that
// holds x_{i+d/2} .. are ROWB/32 lanes apart and swap their words with one cross-lane exchange per 32 bits.
// Arithmetic in fp32 (one multiply and one fma per output), one rounding to the storage type (bf16: nearest even).
#pragma once
#include "ccd_common.h"

namespace ccd {

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  const uint32_t x = __float_as_uint(f);
  if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (x >> 16) | 0x40u;
  return (x + 0x7FFFu + ((x >> 16) & 1u)) >> 16;
}

// cos / sin of the lane's elements of one row: loaded apart from the rotation so that a kernel can have them in
// flight together with the row itself
template <int ROWB, bool BF16>
struct RopeCoef {
  static constexpr int kLanesPerRow = ROWB / 16, kHalf = kLanesPerRow / 2;
  static constexpr int kEPL = BF16 ? 8 : 4;                 // elements per lane
  float c[kEPL], s[kEPL];
  // cos_row / sin_row: the table rows [d/2] of the row's position; lane_in_row: the lane's place among the row's lanes
  __device__ __forceinline__ void load(int lane_in_row, const float* __restrict__ cos_row, const float* __restrict__ sin_row) {
    const int i0 = (lane_in_row % kHalf) * kEPL;            // both lanes of a pair read the same entries
#pragma unroll
    for (int e = 0; e < kEPL; e += 4) {
      const float4 cv = *reinterpret_cast<const float4*>(cos_row + i0 + e);
      const float4 sv = *reinterpret_cast<const float4*>(sin_row + i0 + e);
      c[e] = cv.x; c[e + 1] = cv.y; c[e + 2] = cv.z; c[e + 3] = cv.w;
      s[e] = sv.x; s[e + 1] = sv.y; s[e + 2] = sv.z; s[e + 3] = sv.w;
    }
  }
};

// The lane's 16 bytes of a rotated row.  `x` are the lane's 16 bytes of the source row, `lane_in_row` its place
// among the ROWB/16 lanes of the row.  Both lanes of a pair must call this together (same row: they do).
template <int ROWB, bool BF16>
__device__ __forceinline__ uint4 rope_lane(const uint4& x, int lane_in_row, const RopeCoef<ROWB, BF16>& t) {
  constexpr int kHalf = RopeCoef<ROWB, BF16>::kHalf, kEPL = RopeCoef<ROWB, BF16>::kEPL;
  const bool upper = lane_in_row >= kHalf;                  // this lane holds x_{i+d/2}
  uint4 o;                                                  // the partner's words
  o.x = __shfl_xor(x.x, kHalf);
  o.y = __shfl_xor(x.y, kHalf);
  o.z = __shfl_xor(x.z, kHalf);
  o.w = __shfl_xor(x.w, kHalf);
  float a[kEPL], b[kEPL];
  const uint32_t xw[4] = {x.x, x.y, x.z, x.w}, ow[4] = {o.x, o.y, o.z, o.w};
  if (BF16) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      a[2 * w] = __uint_as_float(xw[w] << 16);  a[2 * w + 1] = __uint_as_float(xw[w] & 0xFFFF0000u);
      b[2 * w] = __uint_as_float(ow[w] << 16);  b[2 * w + 1] = __uint_as_float(ow[w] & 0xFFFF0000u);
    }
  } else {
#pragma unroll
    for (int w = 0; w < 4; ++w) { a[w] = __uint_as_float(xw[w]); b[w] = __uint_as_float(ow[w]); }
  }
  float y[kEPL];
#pragma unroll
  for (int e = 0; e < kEPL; ++e) y[e] = upper ? fmaf(b[e], t.s[e], a[e] * t.c[e]) : fmaf(-b[e], t.s[e], a[e] * t.c[e]);
  uint4 r;
  if (BF16) {
    r.x = f32_to_bf16_bits(y[0]) | (f32_to_bf16_bits(y[1]) << 16);
    r.y = f32_to_bf16_bits(y[2]) | (f32_to_bf16_bits(y[3]) << 16);
    r.z = f32_to_bf16_bits(y[4]) | (f32_to_bf16_bits(y[5]) << 16);
    r.w = f32_to_bf16_bits(y[6]) | (f32_to_bf16_bits(y[7]) << 16);
  } else {
    r.x = __float_as_uint(y[0]); r.y = __float_as_uint(y[1]); r.z = __float_as_uint(y[2]); r.w = __float_as_uint(y[3]);
  }
  return r;
}

}  // namespace ccd
