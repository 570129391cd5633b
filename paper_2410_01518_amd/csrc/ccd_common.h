// Small device helpers shared by the libinfinipot kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ccd_kernels.h"
#include "ccd_launch.h"

namespace ccd {

__device__ __forceinline__ float bf16_bits_to_float(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const uint16_t* p) { return bf16_bits_to_float(*p); }

// four consecutive elements (the address is 8- or 16-byte aligned by construction)
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const uint16_t* p) {
  uint2 r = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                     __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}

// v_exp_f32: 2^x, results below the smallest normal are flushed to zero
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct UnitIdx { int b, l, h; };
__device__ __forceinline__ UnitIdx decode_unit(const Dims& D, int unit) {
  UnitIdx u;
  u.h = unit % D.Hkv;
  int bl = unit / D.Hkv;
  u.l = bl % D.L;
  u.b = bl / D.L;
  return u;
}
__device__ __forceinline__ int64_t kv_offset(const Dims& D, UnitIdx u) {
  return u.b * D.kv_sb + u.l * D.kv_sl + u.h * D.kv_sh;
}
// first element of query row q (0 <= q < G*P) of the group of query heads that shares KV head u.h
__device__ __forceinline__ int64_t q_offset(const Dims& D, UnitIdx u, int q) {
  int g = q / D.P, i = q - g * D.P;
  return u.b * D.q_sb + u.l * D.q_sl + (int64_t)(u.h * D.G + g) * D.q_sh + (int64_t)i * D.d;
}
// where the one extra (max, sum) entry of (unit, query q) lives in `part`, behind the slices of all units: the block of
// the CaP keys on the vector-ALU path, the windowed head on the matrix-core path
__device__ __forceinline__ int64_t extra_block_index(const Dims& D, const ScorePlan& pl, int unit, int q) {
  return ((int64_t)D.units * pl.n_slices1 + unit) * D.GP + q;
}
__device__ __forceinline__ int64_t nov_offset(const Dims& D, UnitIdx u) {
  return u.b * D.nov_sb + u.l * D.nov_sl + u.h * D.nov_sh;
}

}  // namespace ccd
