// Representative score of Eq. 2 for bf16 caches on the matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Same two-pass scheme as the vector-ALU kernels (the normaliser of every CaP query over ALL cached tokens is
// needed before probabilities can be summed over queries); the logits are recomputed in pass 2 rather than kept.
// A workgroup of 4 waves owns one token slice of one unit.  Each wave keeps the fragments of 64 query rows in
// registers for the whole slice; K streams HBM -> LDS by DMA in 32-token tiles (a ring of two batches of three or
// two tiles, XOR-swizzled so that fragment reads are bank-conflict free) and every wave reads each tile.
//
// The 32x32 accumulator tile puts its column index on the lane (lane % 32) and its row index on the register, so
// the operand order is chosen per pass to make the reduction run along registers, never across lanes:
//   pass 1  D[token][query] = Kfrag x Qfrag : each lane owns one query and adds 2^(x - reference) of its 16 token
//           rows to a sum; the reference is fixed per slice (the lane's maximum over the first tile), and a slice
//           whose sums leave the fp32 range is redone with a running maximum;
//   pass 2  D[query][token] = Qfrag x Kfrag : each lane owns one token, adds 2^(x - lse2[query]) of its 16 query
//           rows into partial sums.
// The fragment a lane holds is the same in both roles: the vector with index lane % 32, elements
// 8*(lane/32) .. +7 of each 16-element step of the head dimension.
//
// On this chip the matrix-core time and the vector-ALU time (fma + exp2 + add per logit) of a SIMD add up rather
// than overlap, so a pass costs their sum.  The loop is still software pipelined inside each wave (the MFMAs of tile
// s+1 are issued between the ALU instructions that consume tile s): it hides the LDS reads and the little ALU work
// that does fit under an MFMA.
#include "ccd_score_mfma.h"

namespace ccd {

namespace {

template <int HD, int PASS>
__global__ __launch_bounds__(kMT, 2) void score_pass_kernel(Dims D, ScorePlan pl, const uint16_t* __restrict__ Q,
                                                            const uint16_t* __restrict__ K, float2* __restrict__ part,
                                                            float* __restrict__ u,
                                                            const uint16_t* __restrict__ Kcap,
                                                            float* __restrict__ lse_out) {
  __shared__ ScoreLds<HD, PASS> sm;
  int unit, slice;
  if (!decode_block(D, blockIdx.x, PASS == 1 ? pl.n_slices1 : pl.n_slices2, unit, slice)) return;
  // pass 2 walks the units backwards: the keys pass 1 read last are the ones most likely still held by the
  // memory-side cache
  if (PASS == 2) unit = D.units_run - 1 - unit;
  unit += D.unit0;
  score_pass_body<HD, PASS>(D, pl, unit, slice, Q, K, part, u, Kcap, lse_out, sm);
}

// Sliding attention window: the tokens [0, D.head) that some CaP token does not see.  Those below D.head0 are seen by
// none (score 0, no share in any normaliser); [D.head0, D.head) - at most P + 62 tokens - are seen by some.  Two small
// kernels, one workgroup per unit, outside the two big passes (which start at D.head): statistics before pass 2,
// probabilities (and the zeros) after it.
template <int HD>
struct HeadLds {
  __attribute__((aligned(1024))) uint8_t slot[Tiles<HD>::kSlotBytes];
  float lse_s[kQPerPass];
  float up[4][kMaxSlice];
};

template <int HD>
__global__ __launch_bounds__(kMT) void head_stats_kernel(Dims D, ScorePlan pl, const uint16_t* __restrict__ Q,
                                                         const uint16_t* __restrict__ K, float2* __restrict__ part) {
  __shared__ HeadLds<HD> sm;
  const int unit = D.unit0 + blockIdx.x;
  const UnitIdx ui = decode_unit(D, unit);
  const uint16_t* Ku = K + kv_offset(D, ui);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const float c = D.scale_log2;
  for (int qc = 0; qc < D.GP; qc += kQPerPass) {
    const int q0 = qc + wave * (kQB * 32) + col;
    const MaxSum2 r = stats_sweep_body<HD, true>(Ku, D.head0, D.head, q0 < D.GP ? Q + q_offset(D, ui, q0) : nullptr,
                                              q0 + 32 < D.GP ? Q + q_offset(D, ui, q0 + 32) : nullptr,
                                              (__attribute__((address_space(3))) uint8_t*)sm.slot, c,
                                              D.win_off + q0 % D.P, D.win_off + (q0 + 32) % D.P);
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
      const float m_o = __shfl_xor(r.m[qb], 32), z_o = __shfl_xor(r.Z[qb], 32);
      const float M = fmaxf(r.m[qb], m_o);
      const float z = r.Z[qb] * fast_exp2((r.m[qb] - M) * c) + z_o * fast_exp2((m_o - M) * c);
      const int q = q0 + qb * 32;
      if (half == 0 && q < D.GP) part[extra_block_index(D, pl, unit, q)] = make_float2(M * c, z);
    }
  }
}

template <int HD>
__global__ __launch_bounds__(kMT) void head_prob_kernel(Dims D, const uint16_t* __restrict__ Q,
                                                        const uint16_t* __restrict__ K, const float* __restrict__ lse,
                                                        float lse_mul, float* __restrict__ u) {
  __shared__ HeadLds<HD> sm;
  const int unit = D.unit0 + blockIdx.x;
  const UnitIdx ui = decode_unit(D, unit);
  const uint16_t* Ku = K + kv_offset(D, ui);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, col = lane & 31;
  float* uu = u + (int64_t)unit * D.n;
  for (int qc = 0; qc < D.GP; qc += kQPerPass) {
    const int q = qc + threadIdx.x;
    sm.lse_s[threadIdx.x] = q < D.GP ? lse[(int64_t)unit * D.GP + q] * lse_mul : INFINITY;
    __syncthreads();
    const int q0 = qc + wave * (kQB * 32) + col;
    prob_head_masked<HD>(Ku, D.head0, D.head, q0 < D.GP ? Q + q_offset(D, ui, q0) : nullptr,
                         q0 + 32 < D.GP ? Q + q_offset(D, ui, q0 + 32) : nullptr,
                         (__attribute__((address_space(3))) uint8_t*)sm.slot, D.scale_log2, &sm.lse_s[wave * (kQB * 32)],
                         &sm.up[wave][0], qc + wave * (kQB * 32), D.P, D.win_off);
    for (int t = threadIdx.x; t < D.head - D.head0; t += kMT) {     // the same thread every sweep: no race on u
      const float v = (sm.up[0][t] + sm.up[1][t]) + (sm.up[2][t] + sm.up[3][t]);
      uu[D.head0 + t] = qc == 0 ? v : uu[D.head0 + t] + v;
    }
    if (qc == 0)                                          // tokens no CaP token sees
      for (int t = threadIdx.x; t < D.head0; t += kMT) uu[t] = 0.f;
    __syncthreads();   // lse_s and up are rewritten by the next sweep
  }
}

unsigned stats_grid(const Dims& D, const ScorePlan& pl) { return (unsigned)((D.units_run + 7) / 8 * 8) * pl.n_slices1; }

}  // namespace

int mfma_max_slice() { return kMaxSlice; }

void launch_stats_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s) {
  dim3 grid(stats_grid(D, pl)), block(kMT);
  if (D.d == 64)
    launch((score_pass_kernel<64, 1>), grid, block, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part,
                       (float*)nullptr, (const uint16_t*)nullptr, (float*)nullptr);
  else
    launch((score_pass_kernel<128, 1>), grid, block, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part,
                       (float*)nullptr, (const uint16_t*)nullptr, (float*)nullptr);
}

void launch_head_stats_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s) {
  dim3 grid((unsigned)D.units_run), block(kMT);
  if (D.d == 64)
    launch((head_stats_kernel<64>), grid, block, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part);
  else
    launch((head_stats_kernel<128>), grid, block, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part);
}

void launch_head_prob_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const float* lse, float* u,
                           hipStream_t s) {
  const float lse_mul = pl.lse_given ? 1.44269504088896340736f : 1.0f;
  dim3 grid((unsigned)D.units_run), block(kMT);
  if (D.d == 64)
    launch((head_prob_kernel<64>), grid, block, s, D, (const uint16_t*)Q, (const uint16_t*)K, lse, lse_mul, u);
  else
    launch((head_prob_kernel<128>), grid, block, s, D, (const uint16_t*)Q, (const uint16_t*)K, lse, lse_mul, u);
}

// K_cap (nullable; [units, P, d] bf16): the CaP tokens' own keys join the softmax, causally
void launch_prob_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const void* K_cap,
                      const float2* part, float* u, float* lse_io, hipStream_t s) {
  dim3 grid((unsigned)((D.units_run + 7) / 8 * 8) * pl.n_slices2), block(kMT);
  if (D.d == 64)
    launch((score_pass_kernel<64, 2>), grid, block, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K,
                       const_cast<float2*>(part), u, (const uint16_t*)K_cap, lse_io);
  else
    launch((score_pass_kernel<128, 2>), grid, block, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K,
                       const_cast<float2*>(part), u, (const uint16_t*)K_cap, lse_io);
}

}  // namespace ccd
