// Device code of the bf16 MFMA score passes (Eq. 2); see ccd_score_mfma.hip for the design notes.
#pragma once
#include "ccd_common.h"

namespace ccd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMT = 256;            // threads per workgroup (4 waves)
constexpr int kStep = 32;           // tokens per tile
// K tiles arrive in batches; the LDS ring holds two: one is consumed while the other one lands.  Pass 1 takes K cold
// from HBM and uses batches of three tiles; pass 2 finds part of K in the memory-side cache, makes do with batches of
// two and spends the LDS on partial sums for slices twice as long.
template <int PASS> struct Ring {
  static constexpr int kBatch = PASS == 1 ? 3 : 2;
  static constexpr int kDepth = 2 * kBatch;
};
constexpr int kQB = 2;              // 32-query blocks per wave
constexpr int kQPerPass = 4 * kQB * 32;   // query rows a workgroup covers per sweep over its slice
constexpr int kMaxSlice = 2048;     // slice limit (per-wave partial sums of pass 2 live in LDS)
constexpr float kNegHuge = -1.0e30f;

// The two workgroups that share a CU do not progress alike: the instruction arbiter serves the older wave first, so
// one workgroup runs at full rate (A) and the other (B) at about half of it until A is done, and B then finishes
// alone on a half-used CU (measured: A ends after 74 us, B after 104 us in pass 1).  Wave priorities even this out.
// Workgroups draw alternating parities per CU (an atomic toggle indexed by the hardware CU id; its start value does
// not matter).  Parity 0 runs at priority 2 for the first kPrioSwitch of its tiles and at priority 0 afterwards,
// parity 1 stays at priority 1: first the one, then the other gets the issue slots, and with the switch at
// f/(f+s) ~ 0.65 of the work (f, s = the full and the starved rate) both finish together.
__device__ uint32_t g_cu_toggle[2048];
constexpr float kPrioSwitch = 0.65f;

__device__ __forceinline__ int cu_parity() {
  uint32_t xcc, hw;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
  const uint32_t cu = ((xcc & 7u) << 8) | ((hw >> 8) & 0xFFu);   // XCC, shader engine, shader array, CU
  return (int)(atomicXor(&g_cu_toggle[cu], 1u) & 1u);
}

// row of the 32x32 accumulator tile held in register r by a lane of half `half` (lane / 32)
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// block -> (unit, slice): consecutive blocks go to different XCDs, so the slices of one unit are placed on
// blocks with the same residue mod 8 and share that XCD's L2 for their query fragments.
__device__ __forceinline__ bool decode_block(const Dims& D, int blk, int n_slices, int& unit, int& slice) {
  const int xcd = blk & 7, j = blk >> 3;
  unit = (j / n_slices) * 8 + xcd;     // index inside the launch's range of units
  slice = j % n_slices;
  return unit < D.units_run;
}

// K tiles go from HBM straight into LDS (global_load_lds_dwordx4): one wave instruction moves 64 x 16 bytes to
// consecutive LDS addresses starting at M0, each lane choosing its own global address.  No padding is possible
// in that scheme, so bank conflicts of the fragment reads are avoided by an XOR swizzle instead: the 16-byte
// chunk c of row r is stored at chunk position c ^ swz(r) of that row.
template <int HD>
struct Tiles {
  static constexpr int kRowBytes = HD * 2;
  static constexpr int kChunksPerRow = HD / 8;                       // 16-byte chunks: 16 or 8
  static constexpr int kRowsPerInstr = 64 / kChunksPerRow;           // rows one wave instruction moves
  static constexpr int kInstrPerTile = kStep / kRowsPerInstr;        // 8 or 4
  static constexpr int kInstrPerWave = kInstrPerTile / 4;            // 2 or 1
  static constexpr int kSlotBytes = kStep * kRowBytes;
  __device__ static __forceinline__ int swz(int row) { return HD == 128 ? (row & 15) : ((row >> 1) & 7); }
};

__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds_addr) {
  // gbase and lds_addr are wave-uniform; lane L's 16 bytes land at lds_addr + 16 * L
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase)
               : "memory");
}

// DMA loads to LDS do not retire in issue order (measured: waiting for "all but the youngest n" let stale tiles
// through), so the only safe wait is for everything this wave has in flight.
__device__ __forceinline__ void wait_all_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// this wave's share of tile `tile` of the slice -> ring slot at LDS byte address slot_addr.  voff_full holds the
// lane offsets of the wave's kInstrPerWave instructions inside a full tile (computed once per workgroup).  Only the
// last tile of a pot can be partial: its rows past the end re-read the last valid row; they are masked (pass 1) or
// never stored (pass 2).
template <int HD>
__device__ __forceinline__ void tile_offsets(uint32_t (&voff_full)[Tiles<HD>::kInstrPerWave], int wave, int lane) {
#pragma unroll
  for (int i = 0; i < Tiles<HD>::kInstrPerWave; ++i) {
    const int row = (wave + 4 * i) * Tiles<HD>::kRowsPerInstr + lane / Tiles<HD>::kChunksPerRow;
    const int c = (lane % Tiles<HD>::kChunksPerRow) ^ Tiles<HD>::swz(row);
    voff_full[i] = (uint32_t)(row * Tiles<HD>::kRowBytes + c * 16);
  }
}

template <int HD>
__device__ __forceinline__ void issue_tile(const uint16_t* Ku, int t0, int t1, int tile, uint32_t slot_addr, int wave,
                                           int lane, const uint32_t (&voff_full)[Tiles<HD>::kInstrPerWave]) {
  const int tile_t0 = t0 + tile * kStep;
  const uint16_t* base = Ku + (int64_t)tile_t0 * HD;
  const int last = t1 - 1 - tile_t0;
  if (last >= kStep - 1) {
#pragma unroll
    for (int i = 0; i < Tiles<HD>::kInstrPerWave; ++i) dma16(base, voff_full[i], slot_addr + (wave + 4 * i) * 1024);
  } else {
#pragma unroll
    for (int i = 0; i < Tiles<HD>::kInstrPerWave; ++i) {
      const int j = wave + 4 * i;
      const int row = j * Tiles<HD>::kRowsPerInstr + lane / Tiles<HD>::kChunksPerRow;
      const int c = (lane % Tiles<HD>::kChunksPerRow) ^ Tiles<HD>::swz(row);
      dma16(base, (uint32_t)(min(row, last) * Tiles<HD>::kRowBytes + c * 16), slot_addr + j * 1024);
    }
  }
}

// fragment reads of tile slot SLOT: koff[ks] is the lane's swizzled byte offset inside a slot
template <int HD, int SLOT>
__device__ __forceinline__ void load_k_frags(bf16x8 (&a)[HD / 16], const uint8_t* lds, const int (&koff)[HD / 16]) {
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks)
    a[ks] = *reinterpret_cast<const bf16x8*>(lds + SLOT * Tiles<HD>::kSlotBytes + koff[ks]);
}

template <int HD>
__device__ __forceinline__ void load_q_frags(bf16x8 (&bq)[kQB][HD / 16], const Dims& D, UnitIdx ui, const uint16_t* Q,
                                             int qbase, int col, int half) {
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const int q = qbase + qb * 32 + col;
    if (q < D.GP) {
      const uint16_t* qp = Q + q_offset(D, ui, q) + half * 8;
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks) bq[qb][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    } else {
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks) bq[qb][ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }
}

// logits of one 32-token tile against the wave's 2 x 32 query rows; the two chains alternate so that
// dependent MFMAs are never adjacent.  PASS 1: D[token][query], PASS 2: D[query][token].
template <int HD, int PASS>
__device__ __forceinline__ void logits(floatx16 (&acc)[kQB], const bf16x8 (&a)[HD / 16], const bf16x8 (&bq)[kQB][HD / 16]) {
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[qb][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks)
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
      if (PASS == 1) acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bq[qb][ks], acc[qb], 0, 0, 0);
      else           acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[qb][ks], a[ks], acc[qb], 0, 0, 0);
    }
}

// pass 1: fold the 16 token rows a lane holds into its query's running (max, sum); nvalid < 32 masks the tail
template <bool MASKED>
__device__ __forceinline__ void fold_stats(floatx16 (&acc)[kQB], float (&m_raw)[kQB], float (&Z)[kQB], float c, int half,
                                           int nvalid) {
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    if (MASKED) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (acc_row(r, half) >= nvalid) acc[qb][r] = -INFINITY;
    }
    float t0 = fmaxf(fmaxf(acc[qb][0], acc[qb][1]), acc[qb][2]);
    float t1 = fmaxf(fmaxf(acc[qb][3], acc[qb][4]), acc[qb][5]);
    float t2 = fmaxf(fmaxf(acc[qb][6], acc[qb][7]), acc[qb][8]);
    float t3 = fmaxf(fmaxf(acc[qb][9], acc[qb][10]), acc[qb][11]);
    float t4 = fmaxf(fmaxf(acc[qb][12], acc[qb][13]), acc[qb][14]);
    t0 = fmaxf(fmaxf(t0, t1), t2);
    t3 = fmaxf(fmaxf(t3, t4), acc[qb][15]);
    const float m_new = fmaxf(fmaxf(t0, t3), m_raw[qb]);
    const float negm = -m_new * c;
    float z0 = Z[qb] * fast_exp2((m_raw[qb] - m_new) * c), z1 = 0.f;   // exact difference first: m may be huge
    m_raw[qb] = m_new;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      z0 += fast_exp2(fmaf(acc[qb][r], c, negm));
      z1 += fast_exp2(fmaf(acc[qb][r + 1], c, negm));
    }
    Z[qb] = z0 + z1;
  }
}

// pass 1, the common case: add the 16 token rows a lane holds to its query's sum of 2^((x - m_ref) c) WITHOUT moving
// the reference m_ref (no maximum, no rescaling: 5 instead of 5.5 ALU instructions per logit and no dependent
// chain through the maximum).  The reference is the lane's maximum over the slice's first tile; a sum that leaves
// the fp32 range (some later logit more than ~127 / c above the reference) is detected after the slice, and the
// slice is then redone with fold_stats.
__device__ __forceinline__ void fold_sum(const floatx16 (&acc)[kQB], const float (&m_ref)[kQB], float (&Z)[kQB], float c) {
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const float negm = -m_ref[qb] * c;
    // four independent chains at a time: an exp2 result is never the operand of the very next instruction (which
    // would cost a wait state each time)
    float e[16];
#pragma unroll
    for (int r = 0; r < 16; r += 4) {
#pragma unroll
      for (int i = 0; i < 4; ++i) e[r + i] = fmaf(acc[qb][r + i], c, negm);
#pragma unroll
      for (int i = 0; i < 4; ++i) e[r + i] = fast_exp2(e[r + i]);
    }
    float z0 = Z[qb] + e[0], z1 = e[1];
#pragma unroll
    for (int r = 2; r < 16; r += 2) {
      z0 += e[r];
      z1 += e[r + 1];
    }
    Z[qb] = z0 + z1;
  }
}

// pass 2: probability of the lane's token under its 2 x 16 query rows, summed
__device__ __forceinline__ float fold_prob(const floatx16 (&acc)[kQB], const float (&neg_lse)[kQB][16], float c) {
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      s0 += fast_exp2(fmaf(acc[qb][r], c, neg_lse[qb][r]));
      s1 += fast_exp2(fmaf(acc[qb][r + 1], c, neg_lse[qb][r + 1]));
    }
  return s0 + s1;
}

// The CaP tokens' own keys in the softmax (Eq. 2 read as the model's causal attention row): query row q = g * P + i
// also sees the CaP keys 0 .. i.  Computes, for the wave's 2 x 32 query rows whose fragments are in bq, the
// (max2, sum) statistics over the visible CaP keys and returns the pair of the lane's OWN query row
// qbase + lane (block lane / 32, column lane % 32).  Same operand roles as pass 1 (D[key][query]: a lane owns a
// query and folds key rows); the P key rows of the unit (Kc, [P, HD]) are too few to stage, so their fragments
// come straight from global memory like the queries'.
template <int HD>
__device__ __forceinline__ float2 cap_block_stats(const Dims& D, const uint16_t* __restrict__ Kc,
                                                  const bf16x8 (&bq)[kQB][HD / 16], int qbase, int col, int half, float c) {
  constexpr int KS = HD / 16;
  int cap_pos[kQB];                               // CaP position i of the lane's query in each block
  float m_raw[kQB], Z[kQB];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    cap_pos[qb] = (qbase + qb * 32 + col) % D.P;
    m_raw[qb] = kNegHuge;
    Z[qb] = 0.f;
  }
  for (int j0 = 0; j0 < D.P; j0 += kStep) {
    bf16x8 a[KS];
    const int j = j0 + col;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      a[ks] = j < D.P ? *reinterpret_cast<const bf16x8*>(Kc + (int64_t)j * HD + half * 8 + ks * 16)
                      : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    floatx16 acc[kQB];
    logits<HD, 1>(acc, a, bq);
    // key row j0 + row is visible to CaP position i iff it is not after it (rows past P are after every i)
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (j0 + acc_row(r, half) > cap_pos[qb]) acc[qb][r] = -INFINITY;
    fold_stats<false>(acc, m_raw, Z, c, half, kStep);
  }
  float2 own = make_float2(kNegHuge, 0.f);
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    // the two lane halves hold different key rows of the same query: merge (key 0 is visible to every query and
    // lies in half 0, so the merged maximum is finite)
    const float m_o = __shfl_xor(m_raw[qb], 32), z_o = __shfl_xor(Z[qb], 32);
    const float M = fmaxf(m_raw[qb], m_o);
    const float z = Z[qb] * fast_exp2((m_raw[qb] - M) * c) + z_o * fast_exp2((m_o - M) * c);
    if (qb == half) own = make_float2(M * c, z);
  }
  return own;
}

// scheduling shape of one pipelined step: the LDS fragment reads first, a run of ALU work on the current tile
// to cover their latency, then one MFMA of the next tile per group of ALU instructions
template <int KS, int VALU_LEAD, int VALU_PER_MFMA>
__device__ __forceinline__ void interleave_hint() {
  __builtin_amdgcn_sched_group_barrier(0x100, KS, 0);          // DS reads
  __builtin_amdgcn_sched_group_barrier(0x002, VALU_LEAD, 0);   // VALU
#pragma unroll
  for (int i = 0; i < 2 * KS; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);
  }
}

// Pass 1 over the tokens [t0, t1) of a unit the careful way (running maximum, rescaled sums), tile by tile without
// any overlap.  Called by all threads of the workgroup; uses ring slot 0 (`ring` points at it), which must be idle.
// q_row0 / q_row1: the lane's query rows of block 0 and 1, or null past the end.  WINDOWED: first0 / first1 are the
// first tokens those queries see (sliding attention window); a query that sees none gets (kNegHuge, 0).
struct MaxSum2 { float m[kQB], Z[kQB]; };
template <int HD, bool WINDOWED>
__device__ __forceinline__ MaxSum2 stats_sweep_body(const uint16_t* __restrict__ Ku, int t0, int t1,
                                                    const uint16_t* __restrict__ q_row0,
                                                    const uint16_t* __restrict__ q_row1,
                                                    __attribute__((address_space(3))) uint8_t* ring, float c,
                                                    int first0, int first1) {
  constexpr int KS = HD / 16;
  static_assert(kQB == 2, "two query rows per lane are passed in");
  // arguments of a callable function arrive in vector registers; the DMA wants its base addresses in scalar ones
  const uint64_t ku_bits = reinterpret_cast<uint64_t>(Ku);
  Ku = reinterpret_cast<const uint16_t*>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(ku_bits >> 32)) << 32) |
                                         (uint32_t)__builtin_amdgcn_readfirstlane((int)ku_bits));
  t0 = __builtin_amdgcn_readfirstlane(t0);
  t1 = __builtin_amdgcn_readfirstlane(t1);
  const uint32_t lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)ring);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const uint8_t* lds = (const uint8_t*)ring;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = col * Tiles<HD>::kRowBytes + (((2 * ks + half) ^ Tiles<HD>::swz(col)) << 4);
  uint32_t voff_full[Tiles<HD>::kInstrPerWave];
  tile_offsets<HD>(voff_full, wave, lane);
  bf16x8 bq[kQB][KS];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const uint16_t* qp = qb == 0 ? q_row0 : q_row1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      bq[qb][ks] = qp != nullptr ? *reinterpret_cast<const bf16x8*>(qp + half * 8 + ks * 16) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  MaxSum2 r;
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) { r.m[qb] = kNegHuge; r.Z[qb] = 0.f; }
  const int S = (t1 - t0 + kStep - 1) / kStep;
  for (int s = 0; s < S; ++s) {
    issue_tile<HD>(Ku, t0, t1, s, lds_addr, wave, lane, voff_full);
    wait_all_dma();
    __syncthreads();
    bf16x8 a[KS];
    load_k_frags<HD, 0>(a, lds, koff);
    floatx16 acc[kQB];
    logits<HD, 1>(acc, a, bq);
    const int nvalid = t1 - t0 - s * kStep;
    if (WINDOWED) {
      const int tile_t = t0 + s * kStep;
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        const int first = qb == 0 ? first0 : first1;
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (tile_t + acc_row(i, half) < first) acc[qb][i] = -INFINITY;
      }
    }
    if (nvalid < kStep) fold_stats<true>(acc, r.m, r.Z, c, half, nvalid);
    else                fold_stats<false>(acc, r.m, r.Z, c, half, kStep);
    __syncthreads();   // slot 0 is overwritten by the next tile
  }
  return r;
}

// The fallback of the pipelined pass 1 for sweeps whose fixed-reference sums overflowed.  Not inlined: it is rare,
// and as a function it leaves the registers of the main loop alone.
template <int HD>
__device__ __attribute__((noinline)) MaxSum2 stats_sweep_careful(const uint16_t* __restrict__ Ku, int t0, int t1,
                                                                 const uint16_t* __restrict__ q_row0,
                                                                 const uint16_t* __restrict__ q_row1,
                                                                 __attribute__((address_space(3))) uint8_t* ring,
                                                                 float c) {
  return stats_sweep_body<HD, false>(Ku, t0, t1, q_row0, q_row1, ring, c, 0, 0);
}

// Pass 2 for the tokens [t0, t1) that a sliding attention window hides from some queries: probabilities of each
// token under the workgroup's query rows that do see it, summed per wave into up_w[token - t0] (this wave's row of
// the partial sums in LDS).  Tile by tile without overlap; ring slot 0 must be idle; ends with a barrier.  qrow_base:
// index of the wave's first query row; lse_w: the wave's 64 log2-sum-exps (LDS); a query row g*P + i sees token t
// iff t >= win_off + i.
template <int HD>
__device__ __forceinline__ void prob_head_masked(const uint16_t* __restrict__ Ku, int t0, int t1,
                                                           const uint16_t* __restrict__ q_row0,
                                                           const uint16_t* __restrict__ q_row1,
                                                           __attribute__((address_space(3))) uint8_t* ring, float c,
                                                           const float* lse_w, float* up_w, int qrow_base, int P,
                                                           int win_off) {
  constexpr int KS = HD / 16;
  static_assert(kQB == 2, "two query rows per lane are passed in");
  const uint64_t ku_bits = reinterpret_cast<uint64_t>(Ku);
  Ku = reinterpret_cast<const uint16_t*>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(ku_bits >> 32)) << 32) |
                                         (uint32_t)__builtin_amdgcn_readfirstlane((int)ku_bits));
  t0 = __builtin_amdgcn_readfirstlane(t0);
  t1 = __builtin_amdgcn_readfirstlane(t1);
  const uint32_t lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)ring);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const uint8_t* lds = (const uint8_t*)ring;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = col * Tiles<HD>::kRowBytes + (((2 * ks + half) ^ Tiles<HD>::swz(col)) << 4);
  uint32_t voff_full[Tiles<HD>::kInstrPerWave];
  tile_offsets<HD>(voff_full, wave, lane);
  bf16x8 bq[kQB][KS];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const uint16_t* qp = qb == 0 ? q_row0 : q_row1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      bq[qb][ks] = qp != nullptr ? *reinterpret_cast<const bf16x8*>(qp + half * 8 + ks * 16) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  const int S = (t1 - t0 + kStep - 1) / kStep;
  for (int s = 0; s < S; ++s) {
    issue_tile<HD>(Ku, t0, t1, s, lds_addr, wave, lane, voff_full);
    wait_all_dma();
    __syncthreads();
    bf16x8 a[KS];
    load_k_frags<HD, 0>(a, lds, koff);
    floatx16 acc[kQB];
    logits<HD, 2>(acc, a, bq);                   // D[query][token]: the lane owns token s * 32 + col
    const int t = t0 + s * kStep + col;
    float us = 0.f;
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = qb * 32 + acc_row(r, half);
        const bool sees = t >= win_off + (qrow_base + row) % P;
        const float p = fast_exp2(fmaf(acc[qb][r], c, -lse_w[row]));
        us += sees ? p : 0.f;
      }
    us += __shfl_xor(us, 32);
    if (half == 0) up_w[s * kStep + col] = us;
    __syncthreads();   // slot 0 is overwritten by the next tile; after the last one the sums are visible
  }
}

// PASS 1 writes part[unit][slice][q] = (max2, sum); PASS 2 reads part (all slices of the unit), adds the block of
// the CaP keys in the causal variant (Kcap != nullptr), writes u[unit][t].
// LDS of one score pass.  The K ring must stay first (DMA destinations are addressed relative to it).
template <int HD, int PASS>
struct ScoreLds {
  __attribute__((aligned(1024))) uint8_t ring[Ring<PASS>::kDepth * Tiles<HD>::kSlotBytes];
  float up[PASS == 2 ? 4 : 1][PASS == 2 ? kMaxSlice : 1];   // per-wave partial sums (pass 2)
  float lse_s[PASS == 2 ? kQPerPass : 1];
  int parity;
  int redo[2];     // pass 1: some sum of the sweep left the fp32 range
};

// One (unit, token slice) of one pass, executed by a workgroup of kMT threads.  Ends with every thread past a
// barrier, so the LDS may be reused at once.
template <int HD, int PASS>
__device__ __forceinline__ void score_pass_body(const Dims& D, const ScorePlan& pl, int unit, int slice,
                                                const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                                                float2* __restrict__ part, float* __restrict__ u,
                                                const uint16_t* __restrict__ Kcap, float* __restrict__ lse_out,
                                                ScoreLds<HD, PASS>& sm) {
  constexpr int KS = HD / 16;
  constexpr int SLOTB = Tiles<HD>::kSlotBytes;
  constexpr int kBatch = Ring<PASS>::kBatch, kDepth = Ring<PASS>::kDepth;
  uint8_t* lds = sm.ring;
  auto& up = sm.up;
  auto& lse_s = sm.lse_s;
  const int slice_len = PASS == 1 ? pl.slice1 : pl.slice2;
  const UnitIdx ui = decode_unit(D, unit);
  const uint16_t* Ku = K + kv_offset(D, ui);
  // [t0s, t1): the slice.  [t0s, t0): its tokens that a sliding attention window hides from some query (none without
  // a window, and only in the first slice or two with one): they are left to the two small kernels of the windowed
  // head.  [t0, t1): tokens every query sees - the pipelined loop below.
  const int t0s = slice * slice_len, t1 = min(D.n, t0s + slice_len);
  const int t0 = max(t0s, min(D.head, t1));
  const int S = (t1 - t0 + kStep - 1) / kStep;       // tiles of the main part (the last one may be partial)
  const int S_full = (t1 - t0) / kStep;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const float c = D.scale_log2;
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = col * Tiles<HD>::kRowBytes + (((2 * ks + half) ^ Tiles<HD>::swz(col)) << 4);
  uint32_t voff_full[Tiles<HD>::kInstrPerWave];
  tile_offsets<HD>(voff_full, wave, lane);

  if (threadIdx.x == 0) sm.parity = cu_parity();     // read after the first barrier below
  const int s_switch = (int)(kPrioSwitch * (float)S);
  for (int qc = 0; qc < D.GP; qc += kQPerPass) {
    const int redo_slot = (qc / kQPerPass) & 1;     // alternating: the flag of the sweep before may still be read
    if (PASS == 1 && threadIdx.x == 0) sm.redo[redo_slot] = 0;
    // start the K stream first: batch 0 is in flight while the query fragments are fetched
#pragma unroll
    for (int i = 0; i < kBatch; ++i)
      if (i < S) issue_tile<HD>(Ku, t0, t1, i, lds_addr + i * SLOTB, wave, lane, voff_full);

    bf16x8 bq[kQB][KS];
    load_q_frags<HD>(bq, D, ui, Q, qc + wave * (kQB * 32), col, half);

    float m_raw[kQB], Z[kQB];
    float neg_lse[kQB][16];
    if (PASS == 1) {
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) { m_raw[qb] = kNegHuge; Z[qb] = 0.f; }
    } else {
      // merge the per-slice statistics of pass 1 into log2-sum-exp per query (thread = query of this sweep: the
      // thread's own query row is one of its wave's 2 x 32)
      const int q = qc + threadIdx.x;
      float lse = INFINITY;
      float2 cap = make_float2(kNegHuge, 0.f);         // the block of the CaP keys (causal variant), else nothing
      if (Kcap != nullptr)
        cap = cap_block_stats<HD>(D, Kcap + (int64_t)unit * D.P * HD, bq, qc + wave * (kQB * 32), col, half, c);
      if (pl.lse_given) {            // the caller's normalisers (natural log): nothing to merge
        if (q < D.GP) lse = lse_out[(int64_t)unit * D.GP + q] * 1.44269504088896340736f;
      } else if (q < D.GP) {
        const float2* p = part + (int64_t)unit * pl.n_slices1 * D.GP + q;
        if (pl.head_block) {         // statistics of the windowed head, left there by its own kernel
          const float2 hd = part[extra_block_index(D, pl, unit, q)];
          const float Mh = fmaxf(cap.x, hd.x);
          cap = make_float2(Mh, cap.y * fast_exp2(cap.x - Mh) + hd.y * fast_exp2(hd.x - Mh));
        }
        float M = cap.x;
        for (int j = 0; j < pl.n_slices1; ++j) M = fmaxf(M, p[(int64_t)j * D.GP].x);
        float z = cap.y * fast_exp2(cap.x - M);
        for (int j = 0; j < pl.n_slices1; ++j) {
          const float2 v = p[(int64_t)j * D.GP];
          z += v.y * fast_exp2(v.x - M);
        }
        lse = M + __log2f(z);
        if (pl.head_block && slice == 0) lse_out[(int64_t)unit * D.GP + q] = lse;   // for the head's probabilities
      }
      lse_s[threadIdx.x] = lse;
    }
    wait_all_dma();
    __syncthreads();
    const bool leads = sm.parity == 0;
    if (leads) __builtin_amdgcn_s_setprio(2);
    else       __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = kBatch; i < kDepth; ++i)      // batch 1 lands while batch 0 is consumed
      if (i < S) issue_tile<HD>(Ku, t0, t1, i, lds_addr + i * SLOTB, wave, lane, voff_full);
    if (PASS == 2) {
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_lse[qb][r] = -lse_s[wave * (kQB * 32) + qb * 32 + acc_row(r, half)];
    }
    bf16x8 a[KS];
    floatx16 accA[kQB], accB[kQB];
    load_k_frags<HD, 0>(a, lds, koff);
    logits<HD, PASS>(accA, a, bq);
    if (PASS == 1 && S_full > 0) {
      // reference of the sums of this sweep: the lane's maximum over tile 0 (see fold_sum)
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        float t = accA[qb][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) t = fmaxf(t, accA[qb][r]);
        m_raw[qb] = t;
      }
    }

    // Step s (ring slot I = s mod kDepth) folds tile s on the ALU while the MFMAs of tile s+1 run.  Tiles arrive in
    // batches of b = kBatch: the batch that holds tile s+2 must have landed by the end of every step with
    // s mod b == b-2 (wait + barrier there, nowhere else); right after that barrier the slots of the batch
    // consumed before are free, and the next batch (tiles s+b+1 .. s+2b seen from step s with s mod b == b-1) is
    // requested into them.
#define CCD_STEP(I, CUR, NXT)                                                                     \
    if constexpr ((I) < kDepth) {                                                                 \
      if (s >= S_full) break;                                                                     \
      if (leads && s == s_switch) __builtin_amdgcn_s_setprio(0);                                  \
      if ((I) % kBatch == kBatch - 1) {                                                           \
        _Pragma("unroll") for (int i = 0; i < kBatch; ++i)                                        \
          if (s + kBatch + 1 + i < S)                                                             \
            issue_tile<HD>(Ku, t0, t1, s + kBatch + 1 + i,                                        \
                           lds_addr + (((I) + kBatch + 1 + i) % kDepth) * SLOTB, wave, lane, voff_full); \
      }                                                                                           \
      load_k_frags<HD, ((I) + 1) % kDepth>(a, lds, koff);                                         \
      logits<HD, PASS>(NXT, a, bq);                                                               \
      if (PASS == 1) {                                                                            \
        fold_sum(CUR, m_raw, Z, c);                                                               \
        interleave_hint<KS, 14, 6>();                                                             \
      } else {                                                                                    \
        float us = fold_prob(CUR, neg_lse, c);                                                    \
        interleave_hint<KS, 14, 5>();                                                             \
        us += __shfl_xor(us, 32);                                                                 \
        if (half == 0) {                                                                          \
          float* dst = &up[wave][s * kStep + col];                                                \
          *dst = (qc == 0) ? us : *dst + us;                                                      \
        }                                                                                         \
      }                                                                                           \
      if ((I) % kBatch == kBatch - 2) {                                                           \
        wait_all_dma();                                                                           \
        __builtin_amdgcn_s_barrier();                                                             \
      }                                                                                           \
      ++s;                                                                                        \
    }
    int s = 0;
    while (true) {
      CCD_STEP(0, accA, accB)
      CCD_STEP(1, accB, accA)
      CCD_STEP(2, accA, accB)
      CCD_STEP(3, accB, accA)
      CCD_STEP(4, accA, accB)
      CCD_STEP(5, accB, accA)
    }
#undef CCD_STEP
    static_assert(kDepth <= 6 && kDepth % 2 == 0, "the step sequence above is written out for up to six slots");
    if (PASS == 1 && S_full > 0) {
      // Did a sum leave the fp32 range (or meet a NaN)?  Then the whole workgroup redoes the sweep the careful way
      // below.  Otherwise move each reference to where its sum is of order one (Z = mant * 2^e -> reference
      // + e / c), so that the tail fold and the merges see the magnitudes of a (maximum, sum) pair.
      bool bad = false;
      const float inv_c = 1.0f / c;
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        bad |= !(Z[qb] < INFINITY);
        // (2^-e by ldexp: exp2 would flush it to zero for e near 127; the residual factor makes the new sum
        // consistent with the ROUNDED new reference)
        const int e = __builtin_amdgcn_frexp_expf(Z[qb]);
        const float m_new = m_raw[qb] + (float)e * inv_c;
        Z[qb] = __builtin_amdgcn_ldexpf(Z[qb], -e) * fast_exp2(fmaf(m_raw[qb] - m_new, c, (float)e));
        m_raw[qb] = m_new;
      }
      if (__any(bad) && lane == 0) sm.redo[redo_slot] = 1;
    }
    // the logits of tile S_full - the partial tail tile, if there is one - are in accA or accB by parity
    if (S > S_full) {
      if (S_full & 1) {
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) accA[qb] = accB[qb];
      }
      if (PASS == 1) {
        fold_stats<true>(accA, m_raw, Z, c, half, (t1 - t0) - S_full * kStep);
      } else {
        float us = fold_prob(accA, neg_lse, c);
        us += __shfl_xor(us, 32);
        if (half == 0) {
          float* dst = &up[wave][S_full * kStep + col];
          *dst = (qc == 0) ? us : *dst + us;
        }
      }
    }
    __syncthreads();   // ring, lse_s and up are reused by the next sweep / read below

    if (PASS == 1) {
      if (sm.redo[redo_slot]) {     // uniform over the workgroup
        const int q0 = qc + wave * (kQB * 32) + col;
        const MaxSum2 r = stats_sweep_careful<HD>(Ku, t0, t1, q0 < D.GP ? Q + q_offset(D, ui, q0) : nullptr,
                                                  q0 + 32 < D.GP ? Q + q_offset(D, ui, q0 + 32) : nullptr,
                                                  (__attribute__((address_space(3))) uint8_t*)lds, c);
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) { m_raw[qb] = r.m[qb]; Z[qb] = r.Z[qb]; }
      }
      // the two lane halves hold different token rows of the same query: merge, lower half writes
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        const float m_o = __shfl_xor(m_raw[qb], 32), z_o = __shfl_xor(Z[qb], 32);
        const float M = fmaxf(m_raw[qb], m_o);
        const float z = Z[qb] * fast_exp2((m_raw[qb] - M) * c) + z_o * fast_exp2((m_o - M) * c);
        const int q = qc + wave * (kQB * 32) + qb * 32 + col;
        if (half == 0 && q < D.GP) part[((int64_t)unit * pl.n_slices1 + slice) * D.GP + q] = make_float2(M * c, z);
      }
    }
  }
  if (PASS == 2) {
    float* uu = u + (int64_t)unit * D.n + t0;
    for (int t = threadIdx.x; t < t1 - t0; t += kMT)
      uu[t] = (up[0][t] + up[1][t]) + (up[2][t] + up[3][t]);
    __syncthreads();
  }
}

}  // namespace ccd
