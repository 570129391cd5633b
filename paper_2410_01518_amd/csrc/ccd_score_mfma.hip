// Representative score of Eq. 2 for bf16 caches on the matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Same two-pass scheme as the vector-ALU kernels (the normaliser of every CaP query over ALL cached tokens is
// needed before probabilities can be summed over queries); the logits are recomputed in pass 2 rather than kept.
// A workgroup of 4 waves owns one token slice of one unit.  Each wave keeps the fragments of 64 query rows in
// registers for the whole slice; K streams HBM -> LDS by DMA in 32-token tiles (two batches of three tiles,
// XOR-swizzled so that fragment reads are bank-conflict free) and every wave reads each tile.
//
// The 32x32 accumulator tile puts its column index on the lane (lane % 32) and its row index on the register, so
// the operand order is chosen per pass to make the reduction run along registers, never across lanes:
//   pass 1  D[token][query] = Kfrag x Qfrag : each lane owns one query, folds its 16 token rows into a running
//           (max, sum of 2^(x - max)) pair;
//   pass 2  D[query][token] = Qfrag x Kfrag : each lane owns one token, adds 2^(x - lse2[query]) of its 16 query
//           rows into partial sums.
// The fragment a lane holds is the same in both roles: the vector with index lane % 32, elements
// 8*(lane/32) .. +7 of each 16-element step of the head dimension.
//
// The path is bound by the vector ALU (fma + exp2 + add per logit), not by the matrix cores, so the loop is
// software pipelined inside each wave: the MFMAs of tile s+1 are issued between the ALU instructions that
// consume tile s, and the scheduler is told to keep that interleave.
#include "ccd_score_mfma.h"

namespace ccd {

namespace {

template <int HD, int PASS>
__global__ __launch_bounds__(kMT, 2) void score_pass_kernel(Dims D, ScorePlan pl, const uint16_t* __restrict__ Q,
                                                            const uint16_t* __restrict__ K, float2* __restrict__ part,
                                                            float* __restrict__ u) {
  __shared__ ScoreLds<HD, PASS> sm;
  int unit, slice;
  if (!decode_block(D, PASS == 1 ? pl.n_slices1 : pl.n_slices2, unit, slice)) return;
  // pass 2 walks the units backwards: the keys pass 1 read last are the ones most likely still held by the
  // memory-side cache
  if (PASS == 2) unit = D.units_run - 1 - unit;
  unit += D.unit0;
  score_pass_body<HD, PASS>(D, pl, unit, slice, Q, K, part, u, sm);
}

}  // namespace

int mfma_max_slice() { return kMaxSlice; }

void launch_stats_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s) {
  dim3 grid((unsigned)((D.units_run + 7) / 8 * 8) * pl.n_slices1), block(kMT);
  if (D.d == 64)
    hipLaunchKernelGGL((score_pass_kernel<64, 1>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part,
                       (float*)nullptr);
  else
    hipLaunchKernelGGL((score_pass_kernel<128, 1>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part,
                       (float*)nullptr);
}

void launch_prob_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const float2* part, float* u,
                      hipStream_t s) {
  dim3 grid((unsigned)((D.units_run + 7) / 8 * 8) * pl.n_slices2), block(kMT);
  if (D.d == 64)
    hipLaunchKernelGGL((score_pass_kernel<64, 2>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K,
                       const_cast<float2*>(part), u);
  else
    hipLaunchKernelGGL((score_pass_kernel<128, 2>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K,
                       const_cast<float2*>(part), u);
}

}  // namespace ccd
