// Internal launch interface between the C-ABI host code and the HIP kernels of libinfinipot.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ccd {

// Device-side description of one call (a flattened copy of ccd_shape_t plus derived values).
struct Dims {
  int B, L, Hq, Hkv, G, d;
  int n;        // tokens scored (n_valid)
  int n_cap;
  int k, P, T;
  int GP;       // G * P query rows per unit
  int pool_w, pool_mode;
  int dtype;    // 0 fp32, 1 bf16
  int units;    // B * L * Hkv
  int unit0, units_run;   // the range of units one launch covers (a call may be split into chunks)
  float scale_log2;  // logit scale times log2(e): probabilities are computed with exp2
  int score_path;    // the caller's choice of kernels for Eq. 2 (CCD_PATH_*), read by the host-side plan only
  // sliding attention window (0 = none): CaP token i sees cached token t iff t >= win_off + i; tokens below `head`
  // (a multiple of 32, at most n) are hidden from some CaP token, the others are seen by all; tokens below `head0`
  // (a multiple of 32, at most head) are hidden from every CaP token
  int window, win_off, head, head0;
  int64_t kv_sb, kv_sl, kv_sh;
  int64_t q_sb, q_sl, q_sh;
  int64_t nov_sb, nov_sl, nov_sh;
};

struct ScorePlan {
  int use_mfma;   // 1: bf16 matrix-core kernels, 0: vector-ALU kernels
  int slice1;     // tokens per workgroup in the statistics pass
  int n_slices1;
  int slice2;     // tokens per workgroup in the probability pass
  int n_slices2;
  int cap_block;  // 1 (vector-ALU path): `part` also holds the statistics of the CaP keys' block (causal Eq. 2)
  int head_block; // 1 (matrix-core path): `part` also holds the statistics of the windowed head (sliding window)
  int lse_given;  // 1: the caller handed in the natural-log-sum-exp of every query row: no statistics pass
  int unit_kernel;  // 1 (matrix-core path): both passes in one kernel, one workgroup per unit (launch_score_unit)
};

ScorePlan plan_score(const Dims& D, bool cap_keys);

// pass 1: per (unit, slice, query) running maximum and sum of exp2 of the log2-domain logits
void launch_stats_valu(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s);
// merge the per-slice statistics into one log2-sum-exp per (unit, query)
void launch_merge(const Dims& D, const ScorePlan& pl, const float2* part, float* lse2, hipStream_t s);
// pass 2: u[unit, t] = sum over queries of exp2(logit2 - lse2)
// (lse2 in log2 units, or the caller's natural-log-sum-exps when pl.lse_given)
void launch_prob_valu(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const float* lse2, float* u,
                      hipStream_t s);

// the same two passes on the matrix cores (bf16 only)
int mfma_max_slice();   // longest token slice a workgroup of the matrix-core passes can take
void launch_stats_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s);
// (pass 2 merges the per-slice statistics itself: no merge launch on this path)
// K_cap (nullable; [units, P, d], contiguous): the CaP tokens' own keys join the softmax (Eq. 2 read as the model's
// causal attention row: query row g * P + i also sees the CaP keys 0 .. i); their statistics are computed in the
// prologue of pass 2 and merged like one more token slice
// lse_io ([units, G*P]): pl.lse_given: read, the caller's natural-log-sum-exp per query row (`part` is not used
// then); else written when pl.head_block: the final log2-sum-exp per query, for launch_head_prob_mfma
void launch_prob_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const void* K_cap,
                      const float2* part, float* u, float* lse_io, hipStream_t s);
// Both passes in one kernel, one workgroup per unit (bf16, any shape; it pays when the units fill the chip round by
// round).  Same roles of K_cap, lse_io and the windowed head's entry of `part` as in launch_prob_mfma; `part` is not
// used otherwise.
bool score_unit_supported(const Dims& D);
void launch_score_unit(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const void* K_cap,
                       const float2* part, float* u, float* lse_io, hipStream_t s);
// Sliding attention window on the matrix-core path: the first D.head tokens are hidden from some CaP tokens and are
// left out of the two passes above.  launch_head_stats_mfma (before pass 2) leaves their (max, sum) statistics per
// query in the extra entry of `part` (pl.head_block must be 1); launch_head_prob_mfma (after pass 2) writes
// u[unit, 0 .. D.head) from the final log2-sum-exps.
void launch_head_stats_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s);
// (lse in log2 units, or the caller's natural-log ones when pl.lse_given)
void launch_head_prob_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const float* lse, float* u,
                           hipStream_t s);

// The same on the vector-ALU path: statistics of CaP key j under CaP query i for j <= i, written to `part` behind
// the slices of all units (pl.cap_block must be 1; launch_merge then takes them in).  K_cap as above.
void launch_cap_block_stats_valu(const Dims& D, const ScorePlan& pl, const void* Q, const void* K_cap, float2* part,
                                 hipStream_t s);

// NuC slots of the unit's novelty row + pooling + NuC lift -> scores (when `u` != null; novelty may be null when
// D.T == 0), top-k -> keep_idx (when `keep_idx` != null)
void launch_finalize_select(const Dims& D, const float* u, const float* novelty, float* scores,
                            int32_t* keep_idx, hipStream_t s);

// selection and compaction of a unit in one workgroup (rows short enough to be staged in LDS)
bool select_compact_supported(const Dims& D);
// (carry_novelty: the novelty is carried per head and its kept entries are compacted in place like the rows)
void launch_select_compact(const Dims& D, const float* u, float* novelty, bool carry_novelty, float* scores,
                           int32_t* keep_idx, void* K, void* V, const float* rope_cos, const float* rope_sin, void* Krot,
                           hipStream_t s);
// CR-RoPE of the first `count` rows of every unit (Sec. 3.5): Krot[j] = rotary embedding at position j of K[j]
void launch_rope_rows(const Dims& D, const void* K, const float* rope_cos, const float* rope_sin, int count, void* Krot,
                      hipStream_t s);
// NuC score from logits (Eq. 3): novelty[r] = logsumexp(logits[r, :]) - logits[r, labels[r]]
void launch_nuc_from_logits(const void* logits, const int32_t* labels, float* novelty, int64_t rows, int V,
                            int64_t row_stride_elems, int dtype, hipStream_t s);
int select_max_tokens();   // largest n the selection kernel handles

// rows [D.n, D.n + count) of every unit of K and V <- the chunk's rows (K_new, V_new dense [units, count, d]); novelty
// (nullable) likewise from novelty_new [B, count], into every head when it is carried per head
void launch_append(const Dims& D, int count, void* K, void* V, const void* K_new, const void* V_new, float* novelty,
                   const float* novelty_new, bool nov_per_head, hipStream_t s);
void launch_compact(const Dims& D, const void* Ksrc, const void* Vsrc, const int32_t* keep_idx,
                    void* Kdst, void* Vdst, float* novelty, hipStream_t s);

}  // namespace ccd
