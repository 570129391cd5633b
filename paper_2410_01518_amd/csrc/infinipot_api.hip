// Host side of libinfinipot: argument checks, workspace layout and kernel sequencing for the C ABI
// declared in include/infinipot.h.  Everything here runs before any launch; the kernels live in the
// ccd_*.hip files.
#include <cstdlib>
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <vector>

#include "../../include/infinipot.h"
#include "ccd_kernels.h"
#include "ccd_launch.h"

// Workspace of ccd_compress_noalloc: one copy per GPU, held from the moment the library is loaded until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress (scratch_of_current_device below): the address
// it yields is what kernels, copies and memsets take.
static __device__ __align__(256) unsigned char scratch[CCD_NOALLOC_WORKSPACE_BYTES];

namespace ccd {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

enum Need { kNeedQ = 1, kNeedKV = 2, kNeedNov = 4, kNeedFull = 7 };

// Checks the fields a call reads; returns CCD_OK or an error code.
static int check_shape(const ccd_shape_t* s, int need) {
  if (s == nullptr) return CCD_EINVAL;
  if (s->B < 1 || s->L < 1 || s->Hkv < 1) return CCD_EINVAL;
  if (s->n_valid < 1 || s->k < 1 || s->k > s->n_valid) return CCD_EINVAL;
  if ((int64_t)s->B * s->L * s->Hkv > (int64_t)1 << 24) return CCD_EINVAL;
  if (s->n_valid > select_max_tokens()) return CCD_EUNSUPPORTED;
  if (need == 0) return CCD_OK;
  if (s->n_cap < s->n_valid) return CCD_EINVAL;
  if (s->dtype != CCD_FP32 && s->dtype != CCD_BF16) return CCD_EUNSUPPORTED;
  if (s->d != 64 && s->d != 128) return CCD_EUNSUPPORTED;
  const int64_t esz = s->dtype == CCD_FP32 ? 4 : 2;
  if (need & kNeedKV) {
    const int64_t row = (int64_t)s->n_cap * s->d;
    if (s->kv_stride_h < row || s->kv_stride_l < 0 || s->kv_stride_b < 0) return CCD_EINVAL;
    if ((s->kv_stride_b * esz) % 16 || (s->kv_stride_l * esz) % 16 || (s->kv_stride_h * esz) % 16) return CCD_EALIGN;
  }
  if (need & kNeedQ) {
    if (s->Hq < 1 || s->Hq % s->Hkv != 0 || s->P < 1) return CCD_EINVAL;
    if ((int64_t)(s->Hq / s->Hkv) * s->P > (1 << 20)) return CCD_EINVAL;
    if (s->q_stride_h < (int64_t)s->P * s->d || s->q_stride_l < 0 || s->q_stride_b < 0) return CCD_EINVAL;
    if ((s->q_stride_b * esz) % 16 || (s->q_stride_l * esz) % 16 || (s->q_stride_h * esz) % 16) return CCD_EALIGN;
    if (!(s->scale >= 0.f) || isinf(s->scale)) return CCD_EINVAL;
    if (s->pool_mode < CCD_POOL_NONE || s->pool_mode > CCD_POOL_AVG) return CCD_EUNSUPPORTED;
    if (s->pool_w < 1 || s->pool_w % 2 == 0) return CCD_EINVAL;
    if (s->window < 0 || (s->window > 0 && s->window < s->P)) return CCD_EINVAL;
    if (s->score_path < CCD_PATH_AUTO || s->score_path > CCD_PATH_MFMA_UNIT) return CCD_EINVAL;
    if (s->dtype != CCD_BF16 && s->score_path == CCD_PATH_MFMA_SLICES) return CCD_EUNSUPPORTED;
    // fp32 caches on the matrix cores: head dimension 64, no sliding window (and no CaP keys: checked with the call)
    if (s->dtype != CCD_BF16 && s->score_path == CCD_PATH_MFMA_UNIT && (s->d != 64 || s->window > 0)) return CCD_EUNSUPPORTED;
  }
  if (need & kNeedNov) {
    if (s->T < 0 || s->T > s->k) return CCD_EINVAL;
    if (s->nov_stride_b < 0 || s->nov_stride_l < 0 || s->nov_stride_h < 0) return CCD_EINVAL;
    const bool per_head = s->nov_stride_l != 0 || s->nov_stride_h != 0;
    if (per_head && s->nov_stride_h < s->n_cap) return CCD_EINVAL;
    if (!per_head && s->B > 1 && s->nov_stride_b < s->n_valid) return CCD_EINVAL;
  }
  return CCD_OK;
}

static Dims make_dims(const ccd_shape_t* s) {
  Dims D{};
  D.B = s->B; D.L = s->L; D.Hq = s->Hq; D.Hkv = s->Hkv; D.d = s->d;
  D.G = (s->Hq > 0 && s->Hkv > 0) ? s->Hq / s->Hkv : 0;
  D.n = s->n_valid; D.n_cap = s->n_cap; D.k = s->k; D.P = s->P; D.T = s->T;
  D.GP = D.G * s->P;
  D.pool_w = s->pool_w; D.pool_mode = s->pool_mode; D.dtype = s->dtype;
  D.units = s->B * s->L * s->Hkv;
  D.unit0 = 0;
  D.units_run = D.units;
  const double scale = s->scale > 0.f ? (double)s->scale : 1.0 / sqrt((double)(s->d > 0 ? s->d : 1));
  D.scale_log2 = (float)(scale * 1.4426950408889634074);
  D.score_path = s->score_path;
  D.window = s->window;
  D.win_off = s->window > 0 ? s->n_valid + 1 - s->window : 0;
  D.head = 0;
  D.head0 = 0;
  if (s->window > 0 && s->n_valid + s->P > s->window) {
    const int64_t hidden = (int64_t)s->n_valid + s->P - s->window;        // tokens hidden from the last CaP token
    D.head = (int)((hidden + 31) / 32 * 32 < s->n_valid ? (hidden + 31) / 32 * 32 : s->n_valid);
    const int64_t unseen = (int64_t)s->n_valid + 1 - s->window;           // tokens hidden from the first one, so from all
    D.head0 = unseen > 0 ? (int)(unseen / 32 * 32) : 0;
    if (D.head0 > D.head) D.head0 = D.head;
  }
  D.kv_sb = s->kv_stride_b; D.kv_sl = s->kv_stride_l; D.kv_sh = s->kv_stride_h;
  D.q_sb = s->q_stride_b; D.q_sl = s->q_stride_l; D.q_sh = s->q_stride_h;
  D.nov_sb = s->nov_stride_b; D.nov_sl = s->nov_stride_l; D.nov_sh = s->nov_stride_h;
  return D;
}

constexpr int kMinSlice = 256;   // smallest token slice any plan uses: sizes the per-slice statistics

// compute units of the current device (asked once; the answer of the first device serves all: one GPU model per node)
static int compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    int n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
    cus = n > 0 ? n : 256;
  }
  return cus;
}
// workgroup slots for the slice kernels of the score passes (two workgroups per compute unit)
static int score_slots() { return 2 * compute_units(); }

// Token slice per workgroup: the longest of 2048 / 1024 / 512 / 256 that still gives every slot a workgroup.  Long
// slices amortise the per-workgroup prologue, and a grid of exactly one round has no half-empty last round (the
// headline shape: 256 units x 2 slices of 2048 = 512 workgroups on 512 slots, 6 us per pass less than 4 slices of
// 1024 in two rounds).
static int pick_slice(const Dims& D) {
  const int64_t slots = score_slots();
  for (int slice = mfma_max_slice(); slice > kMinSlice; slice /= 2)
    if ((int64_t)D.units_run * ((D.n + slice - 1) / slice) >= slots) return slice;
  return kMinSlice;
}

static ScorePlan plan_mfma(const Dims& D) {
  ScorePlan pl{};
  pl.use_mfma = 1;
  pl.slice1 = pl.slice2 = pick_slice(D);   // multiples of 32, at most mfma_max_slice()
  pl.n_slices1 = (D.n + pl.slice1 - 1) / pl.slice1;
  pl.n_slices2 = (D.n + pl.slice2 - 1) / pl.slice2;
  pl.cap_block = 0;
  pl.head_block = 0;
  pl.lse_given = 0;
  // One workgroup per unit (both passes in one kernel) when the units fill at least three fifths of the chip round by
  // round; the slice kernels otherwise (few units: they cut a unit into token slices).  Measured on the headline shape
  // with 128 / 192 / 256 / 320 units: 180 / 223 / 220 / 393 us per call against 147 / 246 / 233 / 412 us, and with
  // 32 to 128 query rows per unit (the unit kernel then sweeps 64 or 128 rows at a time) it is 15 - 20 % ahead.
  if (D.score_path == CCD_PATH_MFMA_UNIT) {
    pl.unit_kernel = 1;
  } else if (D.score_path == CCD_PATH_AUTO && score_unit_supported(D)) {
    const int cus = compute_units();
    const int rounds = (D.units_run + cus - 1) / cus;
    pl.unit_kernel = (5 * (int64_t)D.units_run >= 3 * (int64_t)rounds * cus) ? 1 : 0;
  }
  return pl;
}

// cap_keys: the call puts the CaP tokens' own keys into the softmax
ScorePlan plan_score(const Dims& D, bool cap_keys) {
  ScorePlan pl{};
  pl.use_mfma = (D.dtype == CCD_BF16 && D.score_path != CCD_PATH_VALU) ? 1 : 0;
  // a windowed head longer than the head kernels of the matrix-core paths take (about 2000 CaP tokens under a window):
  // the vector-ALU kernels mask inside their loops and take any, so the automatic choice goes there
  if (pl.use_mfma && D.score_path == CCD_PATH_AUTO && D.head - D.head0 > mfma_max_slice()) pl.use_mfma = 0;
  if (pl.use_mfma) {
    return plan_mfma(D);
  } else {
    pl.slice1 = kMinSlice;
    pl.slice2 = 256;   // one token per thread
  }
  pl.n_slices1 = (D.n + pl.slice1 - 1) / pl.slice1;
  pl.n_slices2 = (D.n + pl.slice2 - 1) / pl.slice2;
  pl.cap_block = 0;
  pl.head_block = 0;
  pl.lse_given = 0;
  // fp32 caches: the unit kernel (fp32 values as sums of bf16 products on the matrix cores) where it exists - head
  // dimension 64, plain softmax over the cached tokens - when asked for, and by itself unless a few units with long
  // rows would leave most of the chip idle under it (a workgroup takes about 27 us per 1000 tokens and sweep of 256
  // query rows; measured faster than the vector-ALU kernels from 4 units of 512 tokens to 256 units of 4096)
  if (D.dtype == CCD_FP32 && score_unit_supported(D) && !cap_keys && D.window == 0) {
    if (D.score_path == CCD_PATH_MFMA_UNIT) {
      pl.unit_kernel = 1;
    } else if (D.score_path == CCD_PATH_AUTO) {
      const int cus = compute_units();
      const int64_t rounds = (D.units_run + cus - 1) / cus, sweeps = (D.GP + 255) / 256;
      pl.unit_kernel = (2 * D.units_run >= cus || rounds * sweeps * D.n <= 6000) ? 1 : 0;
    }
  }
  return pl;
}
// a path the caller named that this call cannot take
static bool path_refused(const Dims& D, const ScorePlan& pl) {
  return D.dtype == CCD_FP32 && D.score_path == CCD_PATH_MFMA_UNIT && !pl.unit_kernel;
}

struct Workspace {
  size_t off_part, off_lse, off_u, total;
};

// The layout does not depend on the kernel path, so a workspace sized once serves either.
static Workspace layout_workspace(const Dims& D) {
  Workspace w{};
  size_t off = 0;
  const size_t max_slices = (D.n + kMinSlice - 1) / kMinSlice + 1;   // + the block of the CaP keys (causal variant)
  w.off_part = off;   off = align_up(off + (size_t)D.units * max_slices * D.GP * sizeof(float2), 256);
  w.off_lse = off;    off = align_up(off + (size_t)D.units * D.GP * sizeof(float), 256);
  w.off_u = off;      off = align_up(off + (size_t)D.units * D.n * sizeof(float), 256);
  w.total = off;
  return w;
}

static int check_workspace(const Workspace& w, const void* ws, size_t ws_bytes) {
  if (ws == nullptr || ws_bytes < w.total) return CCD_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return CCD_EWORKSPACE;
  return CCD_OK;
}

// ---- optional per-kernel timing of ccd_compress -------------------------------------------------------
enum Stage { kStStats = 0, kStMerge, kStProb, kStSelect, kStCompact, kStSelCompact, kStCapBlock, kStHead, kStUnit, kNumStages };
static const char* const kStageNames[kNumStages] = {"score_stats", "score_merge",    "score_prob", "select",     "compact",
                                                    "select_compact", "cap_block",   "window_head", "score_unit"};

// A timed stage owns two events; the kernels launched while it is open take them along (ccd_launch.h): the first
// kernel's begin stamp and the last kernel's end stamp are what the stage reports.
StageTimer* g_stage_timer = nullptr;
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> pool;       // every event ever created
  size_t used = 0;                    // events handed out since the last collect
  std::vector<int> stage_of;          // stage of the span that starts at event 2*i
  int64_t calls = 0;
  StageTimer timer{nullptr, nullptr, false};
  hipEvent_t next() {
    if (used == pool.size()) {
      hipEvent_t e;
      // (no system-scope fence with these events: cache write-backs and invalidations at every kernel boundary would
      // change the very durations being measured)
      if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[used++];
  }
  void begin(int stage, hipStream_t) {
    if (!on) return;
    timer.start = next();
    timer.stop = next();
    timer.first = true;
    stage_of.push_back(stage);
    if (timer.start && timer.stop) g_stage_timer = &timer;
  }
  void end(hipStream_t) { g_stage_timer = nullptr; }
};
static Profiler g_prof;

static int launch_status() { return hipGetLastError() == hipSuccess ? CCD_OK : CCD_ELAUNCH; }

// Raw CaP score u[unit, t] (Eq. 2, before pooling).  With K_cap the CaP tokens' own keys join the softmax (causally): their
// statistics become one more entry per unit of `part` on the vector-ALU path (the matrix-core pass 2 computes them
// itself).  (The NuC slots, Sec. 3.3.3 step 1, are found by the selection kernels from the novelty row.)
// lse (nullable): the caller's natural-log-sum-exp of every CaP query row [units, G*P]: the statistics pass (and
// with it K_cap) is not needed, the probabilities follow from one pass over K.
static void run_cap_scores(const Dims& D, ScorePlan pl, const Workspace& w, const void* Q, const void* K,
                           const void* K_cap, const float* lse, char* ws, hipStream_t st) {
  float2* part = reinterpret_cast<float2*>(ws + w.off_part);
  float* lse2 = reinterpret_cast<float*>(ws + w.off_lse);
  float* u = reinterpret_cast<float*>(ws + w.off_u);
  if (pl.unit_kernel) {
    // statistics, merge and probabilities of every unit in one kernel; a windowed head keeps its two small kernels
    float* lse_io = lse2;
    if (lse != nullptr) {
      pl.lse_given = 1;
      lse_io = const_cast<float*>(lse);   // only read when pl.lse_given
    } else if (D.head > 0) {
      pl.head_block = 1;
      g_prof.begin(kStHead, st);
      launch_head_stats_mfma(D, pl, Q, K, part, st);
      g_prof.end(st);
    }
    g_prof.begin(kStUnit, st);
    launch_score_unit(D, pl, Q, K, K_cap, part, u, lse_io, st);
    g_prof.end(st);
    if (D.head > 0) {
      g_prof.begin(kStHead, st);
      launch_head_prob_mfma(D, pl, Q, K, lse_io, u, st);
      g_prof.end(st);
    }
    return;
  }
  if (lse != nullptr) {
    pl.lse_given = 1;
    float* lse_rw = const_cast<float*>(lse);   // only read when pl.lse_given
    g_prof.begin(kStProb, st);
    if (pl.use_mfma) launch_prob_mfma(D, pl, Q, K, nullptr, part, u, lse_rw, st);
    else             launch_prob_valu(D, pl, Q, K, lse, u, st);
    g_prof.end(st);
    if (pl.use_mfma && D.head > 0) {
      g_prof.begin(kStHead, st);
      launch_head_prob_mfma(D, pl, Q, K, lse, u, st);
      g_prof.end(st);
    }
    return;
  }
  if (K_cap != nullptr && !pl.use_mfma) {    // (the matrix-core pass 2 takes the CaP keys in its prologue)
    pl.cap_block = 1;
    g_prof.begin(kStCapBlock, st);
    launch_cap_block_stats_valu(D, pl, Q, K_cap, part, st);
    g_prof.end(st);
  }
  if (pl.use_mfma) {
    if (D.head > 0) {                        // sliding window: the tokens some CaP token does not see
      pl.head_block = 1;
      g_prof.begin(kStHead, st);
      launch_head_stats_mfma(D, pl, Q, K, part, st);
      g_prof.end(st);
    }
    g_prof.begin(kStStats, st);
    launch_stats_mfma(D, pl, Q, K, part, st);
    g_prof.end(st);
    g_prof.begin(kStProb, st);
    launch_prob_mfma(D, pl, Q, K, K_cap, part, u, lse2, st);
    g_prof.end(st);
    if (D.head > 0) {
      g_prof.begin(kStHead, st);
      launch_head_prob_mfma(D, pl, Q, K, lse2, u, st);
      g_prof.end(st);
    }
  } else {
    g_prof.begin(kStStats, st);
    launch_stats_valu(D, pl, Q, K, part, st);
    g_prof.end(st);
    g_prof.begin(kStMerge, st);
    launch_merge(D, pl, part, lse2, st);
    g_prof.end(st);
    g_prof.begin(kStProb, st);
    launch_prob_valu(D, pl, Q, K, lse2, u, st);
    g_prof.end(st);
  }
}

}  // namespace ccd

using namespace ccd;

extern "C" {

size_t ccd_workspace_bytes(const ccd_shape_t* shape) {
  if (check_shape(shape, kNeedFull) != CCD_OK) return 0;
  const Dims D = make_dims(shape);
  return layout_workspace(D).total;
}

static int score_impl(const ccd_shape_t* shape, const void* Q_cat, const void* K, const void* K_cap, const float* lse,
                      const float* novelty, float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape, kNeedFull);
  if (rc != CCD_OK) return rc;
  if (Q_cat == nullptr || K == nullptr || scores == nullptr) return CCD_EINVAL;
  if (novelty == nullptr && shape->T > 0) return CCD_EINVAL;
  if (!aligned16(Q_cat) || !aligned16(K) || !aligned16(K_cap) || !aligned16(lse)) return CCD_EALIGN;
  const Dims D = make_dims(shape);
  const ScorePlan pl = plan_score(D, K_cap != nullptr);
  if (path_refused(D, pl)) return CCD_EUNSUPPORTED;
  if (pl.use_mfma && D.head - D.head0 > mfma_max_slice()) return CCD_EUNSUPPORTED;   // (a matrix-core path was named)
  const Workspace w = layout_workspace(D);
  rc = check_workspace(w, workspace, workspace_bytes);
  if (rc != CCD_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  run_cap_scores(D, pl, w, Q_cat, K, K_cap, lse, ws, st);
  launch_finalize_select(D, reinterpret_cast<const float*>(ws + w.off_u), novelty, scores, nullptr, st);
  return launch_status();
}

int ccd_score(const ccd_shape_t* shape, const void* Q_cat, const void* K, const float* novelty, float* scores,
              void* workspace, size_t workspace_bytes, void* hip_stream) {
  return score_impl(shape, Q_cat, K, nullptr, nullptr, novelty, scores, workspace, workspace_bytes, hip_stream);
}

int ccd_score_kcat(const ccd_shape_t* shape, const void* Q_cat, const void* K, const void* K_cap, const float* novelty,
                   float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (K_cap == nullptr) return CCD_EINVAL;
  return score_impl(shape, Q_cat, K, K_cap, nullptr, novelty, scores, workspace, workspace_bytes, hip_stream);
}

int ccd_score_lse(const ccd_shape_t* shape, const void* Q_cat, const void* K, const float* lse, const float* novelty,
                  float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (lse == nullptr) return CCD_EINVAL;
  return score_impl(shape, Q_cat, K, nullptr, lse, novelty, scores, workspace, workspace_bytes, hip_stream);
}

int ccd_select(const ccd_shape_t* shape, const float* scores, int32_t* keep_idx, void* hip_stream) {
  int rc = check_shape(shape, 0);
  if (rc != CCD_OK) return rc;
  if (scores == nullptr || keep_idx == nullptr) return CCD_EINVAL;
  const Dims D = make_dims(shape);
  launch_finalize_select(D, nullptr, nullptr, const_cast<float*>(scores), keep_idx,
                         static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

int ccd_compact(const ccd_shape_t* shape, const void* K_src, const void* V_src, const int32_t* keep_idx, void* K_dst,
                void* V_dst, float* novelty_inout, void* hip_stream) {
  int rc = check_shape(shape, kNeedKV | (novelty_inout ? kNeedNov : 0));
  if (rc != CCD_OK) return rc;
  if (K_src == nullptr || V_src == nullptr || K_dst == nullptr || V_dst == nullptr || keep_idx == nullptr)
    return CCD_EINVAL;
  if (!aligned16(K_src) || !aligned16(V_src) || !aligned16(K_dst) || !aligned16(V_dst)) return CCD_EALIGN;
  const Dims D = make_dims(shape);
  const bool per_head = shape->nov_stride_l != 0 || shape->nov_stride_h != 0;
  launch_compact(D, K_src, V_src, keep_idx, K_dst, V_dst, per_head ? novelty_inout : nullptr,
                 static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

int ccd_append(const ccd_shape_t* shape, void* K, void* V, float* novelty, const void* K_new, const void* V_new,
               const float* novelty_new, int32_t count, void* hip_stream) {
  if (shape == nullptr) return CCD_EINVAL;
  if (shape->B < 1 || shape->L < 1 || shape->Hkv < 1) return CCD_EINVAL;
  if ((int64_t)shape->B * shape->L * shape->Hkv > (int64_t)1 << 24) return CCD_EINVAL;
  if (shape->n_valid < 0 || shape->n_cap < 1 || count < 0 || (int64_t)shape->n_valid + count > shape->n_cap) return CCD_EINVAL;
  if (shape->dtype != CCD_FP32 && shape->dtype != CCD_BF16) return CCD_EUNSUPPORTED;
  if (shape->d != 64 && shape->d != 128) return CCD_EUNSUPPORTED;
  const int64_t esz = shape->dtype == CCD_FP32 ? 4 : 2;
  if (shape->kv_stride_h < (int64_t)shape->n_cap * shape->d || shape->kv_stride_l < 0 || shape->kv_stride_b < 0) return CCD_EINVAL;
  if ((shape->kv_stride_b * esz) % 16 || (shape->kv_stride_l * esz) % 16 || (shape->kv_stride_h * esz) % 16) return CCD_EALIGN;
  if (K == nullptr || V == nullptr) return CCD_EINVAL;
  if (count == 0) return CCD_OK;                      // an empty chunk (its pointers may be null): nothing to do
  if (K_new == nullptr || V_new == nullptr) return CCD_EINVAL;
  if ((novelty == nullptr) != (novelty_new == nullptr)) return CCD_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(K_new) || !aligned16(V_new)) return CCD_EALIGN;
  const bool per_head = shape->nov_stride_l != 0 || shape->nov_stride_h != 0;
  if (novelty != nullptr) {
    if (shape->nov_stride_b < 0 || shape->nov_stride_l < 0 || shape->nov_stride_h < 0) return CCD_EINVAL;
    if (per_head && shape->nov_stride_h < shape->n_cap) return CCD_EINVAL;
    if (!per_head && shape->B > 1 && shape->nov_stride_b < (int64_t)shape->n_valid + count) return CCD_EINVAL;
  }
  const Dims D = make_dims(shape);
  launch_append(D, count, K, V, K_new, V_new, novelty, novelty_new, per_head, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

// ccd_compress, optionally with CR-RoPE of the kept keys on the side (K_rot != nullptr), other keys to attend to
// (K_score != nullptr) and the CaP tokens' own keys in the softmax (K_cap != nullptr)
static int compress_impl(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty, float* scores_opt,
                         int32_t* keep_idx, const void* K_score, const void* K_cap, const float* lse,
                         const float* rope_cos, const float* rope_sin, void* K_rot, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape, kNeedFull);
  if (rc != CCD_OK) return rc;
  if (Q_cat == nullptr || K == nullptr || V == nullptr || keep_idx == nullptr) return CCD_EINVAL;
  if (novelty == nullptr && shape->T > 0) return CCD_EINVAL;
  if (!aligned16(Q_cat) || !aligned16(K) || !aligned16(V)) return CCD_EALIGN;
  if (K_rot != nullptr) {
    if (rope_cos == nullptr || rope_sin == nullptr || K_rot == K || K_rot == V) return CCD_EINVAL;
    if (!aligned16(K_rot) || !aligned16(rope_cos) || !aligned16(rope_sin)) return CCD_EALIGN;
  }
  if (K_score != nullptr && (K_score == V || !aligned16(K_score))) return K_score == V ? CCD_EINVAL : CCD_EALIGN;
  if (K_cap != nullptr && (K_cap == K || K_cap == V || K_cap == K_rot)) return CCD_EINVAL;
  if (!aligned16(K_cap)) return CCD_EALIGN;
  if (lse != nullptr && K_cap != nullptr) return CCD_EINVAL;     // the normalisers already account for the CaP keys
  if (!aligned16(lse)) return CCD_EALIGN;
  const void* K_attn = K_score != nullptr ? K_score : K;     // the keys the CaP queries attend to
  const Dims D = make_dims(shape);
  const ScorePlan pl = plan_score(D, K_cap != nullptr);
  if (path_refused(D, pl)) return CCD_EUNSUPPORTED;
  if (pl.use_mfma && D.head - D.head0 > mfma_max_slice()) return CCD_EUNSUPPORTED;   // (a matrix-core path was named)
  const Workspace w = layout_workspace(D);
  rc = check_workspace(w, workspace, workspace_bytes);
  if (rc != CCD_OK) return rc;
  if (shape->n_valid < shape->n_cap || shape->n_valid <= shape->k) return CCD_NOOP;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  const float* u = reinterpret_cast<const float*>(ws + w.off_u);
  const bool per_head = shape->nov_stride_l != 0 || shape->nov_stride_h != 0;
  if (g_prof.on) ++g_prof.calls;
  run_cap_scores(D, pl, w, Q_cat, K_attn, K_cap, lse, ws, st);
  if (select_compact_supported(D)) {
    g_prof.begin(kStSelCompact, st);
    launch_select_compact(D, u, novelty, per_head, scores_opt, keep_idx, K, V, rope_cos, rope_sin, K_rot, st);
    g_prof.end(st);
    return launch_status();
  }
  g_prof.begin(kStSelect, st);
  launch_finalize_select(D, u, novelty, scores_opt, keep_idx, st);
  g_prof.end(st);
  g_prof.begin(kStCompact, st);
  launch_compact(D, K, V, keep_idx, K, V, per_head ? novelty : nullptr, st);
  if (K_rot != nullptr) launch_rope_rows(D, K, rope_cos, rope_sin, D.k, K_rot, st);
  g_prof.end(st);
  return launch_status();
}

int ccd_compress(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty, float* scores_opt,
                 int32_t* keep_idx, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return compress_impl(shape, Q_cat, K, V, novelty, scores_opt, keep_idx, nullptr, nullptr, nullptr, nullptr, nullptr,
                       nullptr, workspace, workspace_bytes, hip_stream);
}

// Device address of `scratch` on the current GPU, asked once per GPU (each GPU holds its own copy at its own address).
static int scratch_of_current_device(void** out) {
  constexpr int kMaxDevices = 64;
  static void* ptrs[kMaxDevices] = {};      // racing first calls on one GPU store the same value
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CCD_ELAUNCH;
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return CCD_ELAUNCH;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return CCD_OK;
}

int ccd_compress_noalloc(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty, float* scores_opt,
                         int32_t* keep_idx, void* hip_stream) {
  int rc = check_shape(shape, kNeedFull);
  if (rc != CCD_OK) return rc;
  if (layout_workspace(make_dims(shape)).total > (size_t)CCD_NOALLOC_WORKSPACE_BYTES) return CCD_EWORKSPACE;
  void* ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc != CCD_OK) return rc;
  return compress_impl(shape, Q_cat, K, V, novelty, scores_opt, keep_idx, nullptr, nullptr, nullptr, nullptr, nullptr,
                       nullptr, ws, (size_t)CCD_NOALLOC_WORKSPACE_BYTES, hip_stream);
}

int ccd_compress_lse(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, const float* lse, float* novelty,
                     float* scores_opt, int32_t* keep_idx, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (lse == nullptr) return CCD_EINVAL;
  return compress_impl(shape, Q_cat, K, V, novelty, scores_opt, keep_idx, nullptr, nullptr, lse, nullptr, nullptr, nullptr,
                       workspace, workspace_bytes, hip_stream);
}

int ccd_compress_kcat(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, const void* K_cap, float* novelty,
                      float* scores_opt, int32_t* keep_idx, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (K_cap == nullptr) return CCD_EINVAL;
  return compress_impl(shape, Q_cat, K, V, novelty, scores_opt, keep_idx, nullptr, K_cap, nullptr, nullptr, nullptr,
                       nullptr, workspace, workspace_bytes, hip_stream);
}

int ccd_compress_rope(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty, float* scores_opt,
                      int32_t* keep_idx, const void* K_score, const void* K_cap, const float* lse, const float* rope_cos,
                      const float* rope_sin, void* K_rot, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (K_rot == nullptr) return CCD_EINVAL;
  return compress_impl(shape, Q_cat, K, V, novelty, scores_opt, keep_idx, K_score, K_cap, lse, rope_cos, rope_sin, K_rot,
                       workspace, workspace_bytes, hip_stream);
}

int ccd_cr_rope(const ccd_shape_t* shape, const void* K, const float* rope_cos, const float* rope_sin, int32_t count,
                void* K_rot, void* hip_stream) {
  int rc = check_shape(shape, kNeedKV);
  if (rc != CCD_OK) return rc;
  if (K == nullptr || K_rot == nullptr || rope_cos == nullptr || rope_sin == nullptr || K_rot == K) return CCD_EINVAL;
  if (count < 0 || count > shape->n_cap) return CCD_EINVAL;
  if (!aligned16(K) || !aligned16(K_rot) || !aligned16(rope_cos) || !aligned16(rope_sin)) return CCD_EALIGN;
  if (count == 0) return CCD_OK;
  const Dims D = make_dims(shape);
  launch_rope_rows(D, K, rope_cos, rope_sin, count, K_rot, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

int ccd_nuc_from_logits(const void* logits, const int32_t* labels, float* novelty, int64_t rows, int32_t V,
                        int64_t row_stride, int32_t dtype, void* hip_stream) {
  if (logits == nullptr || labels == nullptr || novelty == nullptr) return CCD_EINVAL;
  if (rows < 0 || rows > 0x7FFFFFFF || V < 1 || row_stride < V) return CCD_EINVAL;
  if (dtype != CCD_FP32 && dtype != CCD_BF16) return CCD_EUNSUPPORTED;
  if (!aligned16(logits) || (row_stride * (dtype == CCD_FP32 ? 4 : 2)) % 16) return CCD_EALIGN;
  if (rows == 0) return CCD_OK;
  launch_nuc_from_logits(logits, labels, novelty, rows, V, row_stride, dtype, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

int ccd_profile_enable(int on) {
  g_prof.on = on != 0;
  return CCD_OK;
}

int ccd_profile_stages(void) { return kNumStages; }

const char* ccd_profile_stage_name(int stage) {
  return (stage >= 0 && stage < kNumStages) ? kStageNames[stage] : "";
}

int ccd_profile_collect(double* stage_ms, int64_t* calls) {
  if (stage_ms == nullptr || calls == nullptr) return CCD_EINVAL;
  for (int i = 0; i < kNumStages; ++i) stage_ms[i] = 0.0;
  *calls = g_prof.calls;
  int rc = CCD_OK;
  for (size_t i = 0; i + 1 < g_prof.used && i / 2 < g_prof.stage_of.size(); i += 2) {
    if (hipEventSynchronize(g_prof.pool[i + 1]) != hipSuccess) { rc = CCD_ELAUNCH; break; }
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.pool[i], g_prof.pool[i + 1]) == hipSuccess) stage_ms[g_prof.stage_of[i / 2]] += ms;
  }
  (void)hipGetLastError();    // a stage that launched nothing leaves two unused events and an error of the query
  g_prof.used = 0;
  g_prof.stage_of.clear();
  g_prof.calls = 0;
  return rc;
}

const char* ccd_strerror(int code) {
  switch (code) {
    case CCD_OK: return "ok";
    case CCD_NOOP: return "pot not full or nothing to drop: nothing done";
    case CCD_EINVAL: return "invalid argument (null pointer or shape field out of range)";
    case CCD_EUNSUPPORTED:
      return "unsupported: head dimension not 64 or 128, unknown dtype or pool mode, more than 65536 tokens, a matrix-core "
             "score path that an fp32 cache cannot take (token slices; units with a head dimension other than 64, a window "
             "or CaP keys), or a matrix-core score path named for a window with more than about 2000 CaP tokens";
    case CCD_EALIGN: return "pointer or stride not 16-byte aligned";
    case CCD_EWORKSPACE:
      return "workspace null, misaligned or too small (ccd_compress_noalloc: the shape needs more than the built-in "
             "CCD_NOALLOC_WORKSPACE_BYTES)";
    case CCD_ELAUNCH: return "HIP kernel launch failed";
    default: return "unknown code";
  }
}

}  // extern "C"
