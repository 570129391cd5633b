// Per-unit selection kernel: NuC slots (Sec. 3.3.3 step 1), pooling + NuC lift, and the final top-k
// (Sec. 3.3.3 step 2 / App. B "Final Token Selection").  The selection machinery is in ccd_topk.h.
//
// finalize_select_kernel: one workgroup of 1024 threads per unit; every thread keeps the scores of its tokens in
// registers (consecutive tokens for rows of up to 32768 tokens, which are staged in LDS; strided tokens for longer
// rows).  Prefix counts taken in token order give both the lowest-index tie-break and the output slot of every kept
// token, so keep_idx comes out ascending without a sort.
#include "ccd_select_body.h"

namespace ccd {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kStageMaxKpt = 32;   // rows of up to 32768 tokens (128 KiB) are staged in LDS for pooling

template <int KPT>
__global__ __launch_bounds__(kSelThreads) void finalize_select_kernel(Dims D, const float* __restrict__ u,
                                                                      const float* __restrict__ novelty, float* scores,
                                                                      int32_t* __restrict__ keep_idx) {
  __shared__ TopkShared<kSelThreads> sh;
  constexpr bool kStaged = KPT <= kStageMaxKpt;
  __shared__ __attribute__((aligned(16))) float u_stage[kStaged ? KPT * kSelThreads + 2 * kStagePad : 4];
  finalize_select_body<kSelThreads, KPT, kStaged>(D, D.unit0 + blockIdx.x, u, novelty, scores, keep_idx, sh,
                                                  kStaged ? u_stage : nullptr);
}

}  // namespace

int select_max_tokens() { return 64 * kSelThreads; }

void launch_finalize_select(const Dims& D, const float* u, const float* novelty, float* scores, int32_t* keep_idx,
                            hipStream_t s) {
  const dim3 grid(D.units_run), block(kSelThreads);
  const int kpt = (D.n + kSelThreads - 1) / kSelThreads;
#define CCD_LAUNCH(KPT) launch((finalize_select_kernel<KPT>), grid, block, s, D, u, novelty, scores, keep_idx)
  if (kpt <= 4) CCD_LAUNCH(4);
  else if (kpt <= 16) CCD_LAUNCH(16);
  else if (kpt <= 32) CCD_LAUNCH(32);
  else CCD_LAUNCH(64);
#undef CCD_LAUNCH
}

}  // namespace ccd
