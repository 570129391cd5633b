// Order-preserving gather-compaction of the cache rows (App. B: K' = K[keep_idx], V' = V[keep_idx]).
//
// In place, destination row j and source row keep_idx[j] live in the same buffer.  keep_idx is strictly
// ascending, so keep_idx[j] >= j: a row only ever moves towards the front.  One workgroup walks the destination
// rows of one (unit, tensor) in ascending chunks; inside a chunk every source row is first loaded into registers,
// then the workgroup synchronises, then the rows are stored.  A store of chunk c lands in rows
// [c*R, (c+1)*R), and every later chunk reads only rows >= (c+1)*R, so the only reads a store could overtake
// are those of its own chunk, which the barrier orders.  Out of place the same code runs without the barrier.
#include "ccd_common.h"
#include "ccd_rope.h"
#include "ccd_select_body.h"

namespace ccd {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Non-temporal 16-byte store: the compacted rows are not read again by this call, and marking them as streaming
// keeps them from lingering as dirty lines that the next kernel's reads would have to push out (measured: 9 us
// less for the compaction itself, 3 us less for the score pass that follows; streaming loads save another 3 us).
__device__ __forceinline__ void store_streaming(char* p, const uint4& v) {
  const u32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
// the source rows are read once as well
__device__ __forceinline__ uint4 load_streaming(const char* p) {
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

constexpr int kCpThreads = 1024;
constexpr int kCpUnroll = 4;

// Appending a chunk of new context behind the cached tokens (Sec. 3.2: the pot is filled until it is full): rows
// [n, n + count) of every unit of K and V take the chunk's rows, dense [units, count, d] on the source side.  A unit's
// share is one contiguous run on both sides; the grid is (unit, tensor, segment of 64 KiB), 16 bytes per lane and
// four of them in flight.  Carried novelty follows: entry n + j of every head takes the chunk's novelty of token j.
constexpr int kApThreads = 256;
constexpr int kApSegBytes = kApThreads * 16 * 16;     // bytes one workgroup moves: 64 KiB
__global__ __launch_bounds__(kApThreads) void append_rows_kernel(Dims D, int esz, int count, int segs, char* K, char* V,
                                                                 const char* Knew, const char* Vnew, float* novelty,
                                                                 const float* nov_new, int nov_per_head) {
  const int seg = blockIdx.x % segs;
  const int ut = blockIdx.x / segs;
  const int unit = ut >> 1;
  const bool isV = ut & 1;
  const UnitIdx ui = decode_unit(D, unit);
  const int64_t run = (int64_t)count * D.d * esz;                         // bytes of a unit's share
  char* dst = (isV ? V : K) + (kv_offset(D, ui) + (int64_t)D.n * D.d) * esz;
  const char* src = (isV ? Vnew : Knew) + (int64_t)unit * run;
  const int64_t b0 = (int64_t)seg * kApSegBytes + threadIdx.x * 16;
#pragma unroll
  for (int r = 0; r < 16; r += 4) {
    uint4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t b = b0 + (int64_t)(r + i) * (kApThreads * 16);
      if (b < run) v[i] = load_streaming(src + b);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t b = b0 + (int64_t)(r + i) * (kApThreads * 16);
      if (b < run) {          // the keys are read again by the next score pass, the values not before the compaction
        if (isV) store_streaming(dst + b, v[i]);
        else     *reinterpret_cast<uint4*>(dst + b) = v[i];
      }
    }
  }
  if (novelty != nullptr && !isV && seg == 0 && (nov_per_head || (ui.l == 0 && ui.h == 0))) {
    float* nd = novelty + nov_offset(D, ui) + D.n;
    const float* ns = nov_new + (int64_t)ui.b * count;
    for (int j = threadIdx.x; j < count; j += kApThreads) nd[j] = ns[j];
  }
}

template <int ROWB>
__global__ __launch_bounds__(kCpThreads) void compact_rows_kernel(Dims D, const char* Ksrc, const char* Vsrc,
                                                                  const int32_t* __restrict__ keep_idx, char* Kdst,
                                                                  char* Vdst) {
  constexpr int kLanesPerRow = ROWB / 16;
  constexpr int kRowsPerPass = kCpThreads / kLanesPerRow;
  const int unit = D.unit0 + (blockIdx.x >> 1);
  const bool isV = blockIdx.x & 1;
  const int64_t ubytes = kv_offset(D, decode_unit(D, unit)) * (int64_t)(ROWB / D.d);
  const char* src = (isV ? Vsrc : Ksrc) + ubytes;
  char* dst = (isV ? Vdst : Kdst) + ubytes;
  const bool inplace = (src == dst);
  const int32_t* keep = keep_idx + (int64_t)unit * D.k;
  const int lane_off = (threadIdx.x % kLanesPerRow) * 16;
  const int row_in_pass = threadIdx.x / kLanesPerRow;

  for (int base = 0; base < D.k; base += kRowsPerPass * kCpUnroll) {
    uint4 v[kCpUnroll];
    bool move[kCpUnroll];
#pragma unroll
    for (int i = 0; i < kCpUnroll; ++i) {
      const int j = base + i * kRowsPerPass + row_in_pass;
      move[i] = false;
      if (j < D.k) {
        int sidx = keep[j];
        sidx = min(max(sidx, 0), D.n_cap - 1);   // a corrupt index must not leave the pot
        move[i] = !(inplace && sidx == j);
        if (move[i]) v[i] = load_streaming(src + (int64_t)sidx * ROWB + lane_off);
      }
    }
    if (inplace) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < kCpUnroll; ++i) {
      const int j = base + i * kRowsPerPass + row_in_pass;
      if (move[i]) store_streaming(dst + (int64_t)j * ROWB + lane_off, v[i]);
    }
  }
}

// per-head novelty carried with the cache: nov[j] <- nov[keep_idx[j]], same chunk discipline
__global__ __launch_bounds__(kCpThreads) void compact_novelty_kernel(Dims D, const int32_t* __restrict__ keep_idx,
                                                                     float* novelty) {
  const int unit = D.unit0 + blockIdx.x;
  float* nov = novelty + nov_offset(D, decode_unit(D, unit));
  const int32_t* keep = keep_idx + (int64_t)unit * D.k;
  for (int base = 0; base < D.k; base += kCpThreads) {
    const int j = base + threadIdx.x;
    float v = 0.f;
    if (j < D.k) v = nov[min(max(keep[j], 0), D.n_cap - 1)];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (j < D.k) nov[j] = v;
  }
}

// Selection and compaction of one unit in ONE workgroup (ccd_compress, rows of up to 32768 tokens): the kept indices
// stay in LDS (in the space of the staged score row, which is dead by then) and K and V chunks move together, two
// 16-byte loads per tensor in flight per thread.  Against a selection kernel followed by a compaction kernel this
// saves a launch, the drain of a latency-bound grid, and the trip of keep_idx through memory; the compaction part
// runs as fast as with a workgroup per tensor (measured 88.5 against 89.3 us).
constexpr int kScUnroll = 2;
constexpr int kSplitFillWorkgroups = 256;   // one 1024-thread workgroup per compute unit

// ROPE (CR-RoPE, Sec. 3.5): the kernel also writes Krot[j] = rotary embedding at position j of the kept key j, for all
// j < k (rows that stay where they are included, so every kept K row is read); the pot itself keeps the plain keys.
//
// SPLIT (calls with few units, which leave most of the chip idle): `parts` workgroups per unit.  Each of them runs
// the whole selection for itself (same inputs, same kept list; only the first writes scores and keep_idx) and then
// moves its share of the bytes: one tensor (K for even parts, V for odd ones) and one column segment of
// ROWB / (parts / 2) bytes of every row (at least 128 bytes; the whole row with ROPE, which pairs columns d/2 apart).
// The shares are disjoint, so the workgroups of a unit need no ordering among themselves.  Carried novelty is not
// compacted here in this form (its entries are still being read by the other workgroups' selections).
constexpr int kScSplitUnroll = 4;

template <int KPT, int ROWB, bool ROPE, bool BF16, bool SPLIT>
__global__ __launch_bounds__(kCpThreads) void select_compact_kernel(Dims D, const float* __restrict__ u,
                                                                    float* novelty, int carry_novelty, float* scores,
                                                                    int32_t* __restrict__ keep_idx, char* Kbuf,
                                                                    char* Vbuf, const float* __restrict__ rope_cos,
                                                                    const float* __restrict__ rope_sin, char* Krot,
                                                                    int parts) {
  __shared__ TopkShared<kCpThreads> sh;
  __shared__ __attribute__((aligned(16))) float u_stage[KPT * kCpThreads + 2 * kStagePad];
  int32_t* keep_lds = reinterpret_cast<int32_t*>(u_stage);
  if constexpr (SPLIT) {
    const int part = blockIdx.x % parts, unit = D.unit0 + blockIdx.x / parts;
    finalize_select_body<kCpThreads, KPT, true>(D, unit, u, novelty, part == 0 ? scores : nullptr,
                                                part == 0 ? keep_idx : nullptr, sh, u_stage, keep_lds);
    __syncthreads();
    const bool is_v = part & 1;
    const int seg = part >> 1, lanes = (ROWB / 16) / (parts >> 1);     // 16-byte lanes per row segment: 8, 16 or 32
    const int lane_shift = __ffs(lanes) - 1;
    const int lane_in_row = seg * lanes + (threadIdx.x & (lanes - 1));
    const int row_in_pass = threadIdx.x >> lane_shift, rows_per_pass = kCpThreads >> lane_shift;
    const int lane_off = lane_in_row * 16;
    const int64_t ubytes = kv_offset(D, decode_unit(D, unit)) * (int64_t)(ROWB / D.d);
    char* tb = (is_v ? Vbuf : Kbuf) + ubytes;
    char* rb = ROPE ? Krot + ubytes : nullptr;
    const bool rot = ROPE && !is_v;
    const int half_d = D.d / 2;
    for (int base = 0; base < D.k; base += rows_per_pass * kScSplitUnroll) {
      uint4 a[kScSplitUnroll];
      bool move[kScSplitUnroll];
      RopeCoef<ROWB, BF16> coef[ROPE ? kScSplitUnroll : 1];
#pragma unroll
      for (int i = 0; i < kScSplitUnroll; ++i) {
        const int j = base + i * rows_per_pass + row_in_pass;
        move[i] = false;
        if (j < D.k) {
          const int sidx = keep_lds[j];
          move[i] = sidx != j;
          if (move[i] || rot) a[i] = load_streaming(tb + (int64_t)sidx * ROWB + lane_off);
          if (ROPE && rot) coef[i].load(lane_in_row, rope_cos + (int64_t)j * half_d, rope_sin + (int64_t)j * half_d);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kScSplitUnroll; ++i) {
        const int j = base + i * rows_per_pass + row_in_pass;
        if (move[i]) store_streaming(tb + (int64_t)j * ROWB + lane_off, a[i]);
        if (ROPE && rot && j < D.k)
          store_streaming(rb + (int64_t)j * ROWB + lane_off, rope_lane<ROWB, BF16>(a[i], lane_in_row, coef[ROPE ? i : 0]));
      }
    }
    return;
  }
  const int unit = D.unit0 + blockIdx.x;
  finalize_select_body<kCpThreads, KPT, true>(D, unit, u, novelty, scores, keep_idx, sh, u_stage, keep_lds);
  __syncthreads();

  if (carry_novelty) {
    // novelty carried per head: its kept entries move up like the rows (keep[j] >= j: a chunk's sources are read
    // before anything at or above them is written)
    float* nov = novelty + nov_offset(D, decode_unit(D, unit));
    for (int base = 0; base < D.k; base += kCpThreads) {
      const int j = base + threadIdx.x;
      float v = 0.f;
      if (j < D.k) v = nov[keep_lds[j]];
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (j < D.k) nov[j] = v;
    }
  }

  constexpr int kLanesPerRow = ROWB / 16;
  constexpr int kRowsPerPass = kCpThreads / kLanesPerRow;
  const int64_t ubytes = kv_offset(D, decode_unit(D, unit)) * (int64_t)(ROWB / D.d);
  char* kb = Kbuf + ubytes;
  char* vb = Vbuf + ubytes;
  char* rb = ROPE ? Krot + ubytes : nullptr;
  const int lane_in_row = threadIdx.x % kLanesPerRow;
  const int lane_off = lane_in_row * 16;
  const int row_in_pass = threadIdx.x / kLanesPerRow;
  const int half_d = D.d / 2;
  for (int base = 0; base < D.k; base += kRowsPerPass * kScUnroll) {
    uint4 a[kScUnroll], b[kScUnroll];
    bool move[kScUnroll];
    RopeCoef<ROWB, BF16> coef[ROPE ? kScUnroll : 1];
#pragma unroll
    for (int i = 0; i < kScUnroll; ++i) {
      const int j = base + i * kRowsPerPass + row_in_pass;
      move[i] = false;
      if (j < D.k) {
        const int sidx = keep_lds[j];             // written by this workgroup: ascending, in [j, n)
        move[i] = sidx != j;
        if (move[i] || ROPE) a[i] = load_streaming(kb + (int64_t)sidx * ROWB + lane_off);
        if (move[i]) b[i] = load_streaming(vb + (int64_t)sidx * ROWB + lane_off);
        if (ROPE) coef[i].load(lane_in_row, rope_cos + (int64_t)j * half_d, rope_sin + (int64_t)j * half_d);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kScUnroll; ++i) {
      const int j = base + i * kRowsPerPass + row_in_pass;
      if (move[i]) {
        store_streaming(kb + (int64_t)j * ROWB + lane_off, a[i]);
        store_streaming(vb + (int64_t)j * ROWB + lane_off, b[i]);
      }
      if (ROPE && j < D.k)
        store_streaming(rb + (int64_t)j * ROWB + lane_off, rope_lane<ROWB, BF16>(a[i], lane_in_row, coef[ROPE ? i : 0]));
    }
  }
}

// Stand-alone CR-RoPE: Krot[j] = rotary embedding at position j of K[j], j < count, for every unit of the launch.
// A thread handles kRopeUnroll rows (all their loads in flight together).
constexpr int kRopeUnroll = 4;

template <int ROWB, bool BF16>
__global__ __launch_bounds__(256) void rope_rows_kernel(Dims D, const char* __restrict__ Kbuf,
                                                        const float* __restrict__ rope_cos,
                                                        const float* __restrict__ rope_sin, int count, char* Krot) {
  constexpr int kLanesPerRow = ROWB / 16;
  constexpr int kRowsPerPass = 256 / kLanesPerRow;
  constexpr int kRowsPerBlock = kRowsPerPass * kRopeUnroll;
  const int blocks_per_unit = (count + kRowsPerBlock - 1) / kRowsPerBlock;
  const int unit = D.unit0 + blockIdx.x / blocks_per_unit;
  const int64_t ubytes = kv_offset(D, decode_unit(D, unit)) * (int64_t)(ROWB / D.d);
  const int lane_in_row = threadIdx.x % kLanesPerRow;
  const int j0 = (blockIdx.x % blocks_per_unit) * kRowsPerBlock + threadIdx.x / kLanesPerRow;
  const int half_d = D.d / 2;
  uint4 x[kRopeUnroll];
  RopeCoef<ROWB, BF16> coef[kRopeUnroll];
#pragma unroll
  for (int i = 0; i < kRopeUnroll; ++i) {
    const int j = j0 + i * kRowsPerPass;
    if (j < count) {                                           // whole rows: both lanes of a pair agree
      x[i] = load_streaming(Kbuf + ubytes + (int64_t)j * ROWB + lane_in_row * 16);
      coef[i].load(lane_in_row, rope_cos + (int64_t)j * half_d, rope_sin + (int64_t)j * half_d);
    }
  }
#pragma unroll
  for (int i = 0; i < kRopeUnroll; ++i) {
    const int j = j0 + i * kRowsPerPass;
    if (j < count)
      store_streaming(Krot + ubytes + (int64_t)j * ROWB + lane_in_row * 16, rope_lane<ROWB, BF16>(x[i], lane_in_row, coef[i]));
  }
}

}  // namespace

bool select_compact_supported(const Dims& D) { return D.n <= 32 * kCpThreads; }

// pooling + NuC lift + top-k + in-place compaction of K and V (and of carried per-head novelty).
// Krot != nullptr: CR-RoPE of the kept keys on the side (rope_cos / rope_sin: [>= k, d/2] fp32).
// A launch with so few units that most compute units would stay idle gives every unit 2, 4 or 8 workgroups (see the
// kernel); carried novelty then follows in a small kernel of its own.
void launch_select_compact(const Dims& D, const float* u, float* novelty, bool carry_novelty, float* scores,
                           int32_t* keep_idx, void* K, void* V, const float* rope_cos, const float* rope_sin, void* Krot,
                           hipStream_t s) {
  const int rowb = D.d * (D.dtype == 0 ? 4 : 2);
  const int max_parts = Krot != nullptr ? 2 : 2 * (rowb / 128);
  int parts = 1;
  while (parts * 2 <= max_parts && (int64_t)D.units_run * parts * 2 <= kSplitFillWorkgroups) parts *= 2;
  const bool split = parts > 1;
  const dim3 grid((unsigned)D.units_run * parts), block(kCpThreads);
#define CCD_LAUNCH(KPT, RB, ROPE, BF, SPLIT)                                                                           \
  launch((select_compact_kernel<KPT, RB, ROPE, BF, SPLIT>), grid, block, s, D, u, novelty,                \
                     (carry_novelty && !SPLIT) ? 1 : 0, scores, keep_idx, (char*)K, (char*)V, rope_cos, rope_sin,        \
                     (char*)Krot, parts)
#define CCD_LAUNCH_RB(KPT, ROPE, SPLIT)                                           \
  if (rowb == 128) CCD_LAUNCH(KPT, 128, ROPE, true, SPLIT);                        \
  else if (rowb == 256 && D.dtype == 1) CCD_LAUNCH(KPT, 256, ROPE, true, SPLIT);    \
  else if (rowb == 256) CCD_LAUNCH(KPT, 256, ROPE, false, SPLIT);                   \
  else CCD_LAUNCH(KPT, 512, ROPE, false, SPLIT)
#define CCD_LAUNCH_SPLIT(KPT, ROPE)                              \
  if (split) { CCD_LAUNCH_RB(KPT, ROPE, true); } else { CCD_LAUNCH_RB(KPT, ROPE, false); }
  const int kpt = (D.n + kCpThreads - 1) / kCpThreads;
  if (Krot == nullptr) {
    if (kpt <= 4) { CCD_LAUNCH_SPLIT(4, false); } else if (kpt <= 16) { CCD_LAUNCH_SPLIT(16, false); } else { CCD_LAUNCH_SPLIT(32, false); }
  } else {
    if (kpt <= 4) { CCD_LAUNCH_SPLIT(4, true); } else if (kpt <= 16) { CCD_LAUNCH_SPLIT(16, true); } else { CCD_LAUNCH_SPLIT(32, true); }
  }
#undef CCD_LAUNCH_SPLIT
#undef CCD_LAUNCH_RB
#undef CCD_LAUNCH
  if (split && carry_novelty)
    launch(compact_novelty_kernel, dim3(D.units_run), block, s, D, keep_idx, novelty);
}

void launch_rope_rows(const Dims& D, const void* K, const float* rope_cos, const float* rope_sin, int count, void* Krot,
                      hipStream_t s) {
  const int rowb = D.d * (D.dtype == 0 ? 4 : 2);
  const int rows_per_block = 256 / (rowb / 16) * kRopeUnroll;
  const dim3 grid((unsigned)((count + rows_per_block - 1) / rows_per_block) * (unsigned)D.units_run), block(256);
#define CCD_LAUNCH(RB, BF) \
  launch((rope_rows_kernel<RB, BF>), grid, block, s, D, (const char*)K, rope_cos, rope_sin, count, (char*)Krot)
  if (rowb == 128) CCD_LAUNCH(128, true);
  else if (rowb == 256 && D.dtype == 1) CCD_LAUNCH(256, true);
  else if (rowb == 256) CCD_LAUNCH(256, false);
  else CCD_LAUNCH(512, false);
#undef CCD_LAUNCH
}

void launch_append(const Dims& D, int count, void* K, void* V, const void* K_new, const void* V_new, float* novelty,
                   const float* novelty_new, bool nov_per_head, hipStream_t s) {
  const int esz = D.dtype == 0 ? 4 : 2;
  const int64_t run = (int64_t)count * D.d * esz;
  const int segs = (int)((run + kApSegBytes - 1) / kApSegBytes);
  dim3 grid((unsigned)(D.units * 2 * segs)), block(kApThreads);
  launch(append_rows_kernel, grid, block, s, D, esz, count, segs, (char*)K, (char*)V, (const char*)K_new,
         (const char*)V_new, novelty, novelty_new, nov_per_head ? 1 : 0);
}

void launch_compact(const Dims& D, const void* Ksrc, const void* Vsrc, const int32_t* keep_idx, void* Kdst, void* Vdst,
                    float* novelty, hipStream_t s) {
  const int rowb = D.d * (D.dtype == 0 ? 4 : 2);
  dim3 grid(2u * D.units_run), block(kCpThreads);
#define CCD_LAUNCH(RB)                                                                                             \
  launch((compact_rows_kernel<RB>), grid, block, s, D, (const char*)Ksrc, (const char*)Vsrc, keep_idx, \
                     (char*)Kdst, (char*)Vdst)
  if (rowb == 128) CCD_LAUNCH(128);
  else if (rowb == 256) CCD_LAUNCH(256);
  else CCD_LAUNCH(512);
#undef CCD_LAUNCH
  if (novelty != nullptr)
    launch(compact_novelty_kernel, dim3(D.units_run), block, s, D, keep_idx, novelty);
}

}  // namespace ccd
