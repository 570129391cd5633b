// Representative score of Eq. 2 on the matrix cores, one workgroup per unit: both passes in one kernel.  bf16 caches
// (head dimension 64 or 128), and fp32 caches of head dimension 64 as sums of bf16 products (see "fp32 caches" below).
//
// The slice kernels of ccd_score_mfma.hip share every K tile among the four waves of a workgroup through LDS (each
// wave owns 64 query rows), and the traffic that goes with it - DMA into the ring, eight fragment reads per wave and
// tile, a barrier per batch - costs more than the arithmetic hides.  Here the roles are turned round: a wave owns a
// quarter of the unit's TOKENS and all 256 query rows of a sweep.  The fragments of the 256 query rows (256 registers
// per lane) stay in the accumulation registers for the whole unit - matrix instructions read their operands from
// there directly - and the wave's own K tiles come straight from global memory into vector registers, two tiles
// ahead of their use.  No LDS on the K path, no barrier, no wave ever waits for another one inside a pass.  One
// workgroup per compute unit (each lane holds 512 registers).
//
// Because one workgroup sees all tokens of its unit, the statistics of pass 1 change hands through LDS: pass 2
// follows in the same kernel, the per-slice statistics buffer and the second launch are not needed.
//
//   pass 1  D[token][query] = Kfrag x Qfrag: a lane owns one query row of each of the eight 32-row blocks and adds
//           2^((x - reference) c) of its 16 token rows to that row's sum (fixed reference per wave and row: the maximum
//           over the wave's first tile; a sum that leaves the fp32 range makes the wave redo its tokens with a
//           running maximum);
//   merge   the four waves' (reference, sum) pairs, the CaP keys' block (causal variant) and the windowed head become
//           one log2-sum-exp per query row;
//   pass 2  D[query][token] = Qfrag x Kfrag: a lane owns one token and adds 2^(x c - lse2[query]) over the 16 query
//           rows of each accumulator; the negated lse2 values of a block pair are re-read from LDS (two addresses per
//           wave: a broadcast) one step ahead.  Tiles are walked backwards: what pass 1 read last is still cached.
//
// Steps are software pipelined inside a wave: the 16 MFMAs of one (tile, block pair) are issued between the ALU
// instructions that consume the accumulators of the step before.  Compiled with the VGPR form of the matrix
// instructions (results land in vector registers, where the ALU reads them; the query fragments are pinned to the
// accumulation registers).
//
// fp32 caches: an fp32 value x is split into hi = bf16(x) and lo = bf16(x - hi) (x - hi is exact in fp32; what is left
// is below 2^-17 |x|), and a product q k is taken as qh kh + ql kh + qh kl on the bf16 matrix instructions - three of
// them per product, accumulated in fp32 in that order, the dropped ql kl term being 2^-18 of the product.  The logit
// then carries a relative error of about 2^-16 of sum |q k| instead of fp32's 2^-24: two orders below what the
// scores are asked to keep.  A row of d fp32 values becomes 2 d bf16 values [hi | lo], so d = 64 has the fragment
// counts of a bf16 row of 128 and fits the same registers; K tiles are split in registers as they arrive (no copy of
// the cache in memory), query rows once per sweep.
#include <type_traits>

#include "ccd_score_mfma.h"

namespace ccd {

namespace {

constexpr int kUPairs = 4;                    // pairs of 32-query blocks per sweep, at most (a kernel is built for 1, 2 and 4)
constexpr int kUQ = kUPairs * kQB * 32;       // query rows per sweep, at most: 256
constexpr int kUBlock = 128;                  // tiles of a wave between two write-outs of its token sums (pass 2)
static_assert(kQB == 2, "a step covers two query blocks");

template <int HD>
struct UnitLds {
  float2 stat[4][kUQ];     // per wave: (max2, sum) of every query row of the sweep over the wave's tokens
  float neg_lse[kUQ];      // -log2-sum-exp per query row of the sweep
  float ubuf[4][kUBlock * kStep];   // per wave: the token sums of the block of tiles it is working on (pass 2)
};

// Shape of the work per head dimension HD and cache type (F32: fp32 values as [hi | lo] bf16 pairs)
template <int HD, bool F32>
struct UnitShape {
  static constexpr int KQ = HD / 16;                    // 16-wide steps along the head dimension
  static constexpr int KF = F32 ? 2 * KQ : KQ;          // fragments of a K tile, and of a 32-row block of query rows
  static constexpr int NMQ = F32 ? 3 * KQ : KQ;         // matrix instructions per 32 x 32 block of logits
  static constexpr int NM = kQB * NMQ;                  // ... per step (a pair of blocks)
  static constexpr int NCH = NM < 16 ? NM : 16;         // chunks the ALU work of a step is cut into
  static constexpr int EPC = 32 / NCH;                  // accumulator elements per chunk
  static_assert(kUPairs * kQB * KF * 4 <= 256, "the query fragments of the widest sweep fill the accumulation registers");
  // matrix instruction j (0 .. NMQ - 1) of a block: which K fragment meets which query fragment
  static constexpr int kfrag(int j) { return !F32 ? j : (j < 2 * KQ ? j % KQ : KQ + j % KQ); }
  static constexpr int qfrag(int j) { return !F32 ? j : (j < KQ ? j : (j < 2 * KQ ? j : j - 2 * KQ)); }
  // chunks of ALU work done once matrix instruction i of a step is issued: none behind the first, all behind the last
  static constexpr int chunks_by(int i) { return i < 0 ? 0 : (i == NM - 1 ? NCH : (i * NCH) / NM); }
};

// fragments of one 32-token tile, straight from global memory: lane (col, half) holds elements 16 ks + 8 half .. + 7
// of token row t_tile + col (rows past t_last re-read row t_last: masked in pass 1, never stored in pass 2)
template <int HD>
__device__ __forceinline__ void load_k_tile(bf16x8 (&a)[HD / 16], const uint16_t* __restrict__ Ku, int t_tile, int t_last,
                                            int col, int half) {
  const uint16_t* p = Ku + (int64_t)min(t_tile + col, t_last) * HD + half * 8;
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(p + ks * 16);
}

// fp32 caches: the same elements as 8 floats per k-step (two 16-byte loads), split into hi and lo fragments later
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <int HD>
struct RawTile {
  f32x4 v[HD / 16][2];
};
template <int HD>
__device__ __forceinline__ void load_k_raw(RawTile<HD>& r, const float* __restrict__ Ku, int t_tile, int t_last, int col,
                                           int half) {
  const float* p = Ku + (int64_t)min(t_tile + col, t_last) * HD + half * 8;
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks) {
    r.v[ks][0] = *reinterpret_cast<const f32x4*>(p + ks * 16);
    r.v[ks][1] = *reinterpret_cast<const f32x4*>(p + ks * 16 + 4);
  }
}
// x0, x1 -> (bf16(x0), bf16(x1)) packed, and the same of what the rounding left over: 3 ALU instructions per value
__device__ __forceinline__ void split2(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  hi = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){x0, x1}, bf16x2));
  const float h0 = __uint_as_float(hi << 16), h1 = __uint_as_float(hi & 0xFFFF0000u);
  lo = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){x0 - h0, x1 - h1}, bf16x2));
}
__device__ __forceinline__ void split8(const f32x4 (&x)[2], bf16x8& hi, bf16x8& lo) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  uint32_t h[4], l[4];
  split2(x[0].x, x[0].y, h[0], l[0]);
  split2(x[0].z, x[0].w, h[1], l[1]);
  split2(x[1].x, x[1].y, h[2], l[2]);
  split2(x[1].z, x[1].w, h[3], l[3]);
  hi = __builtin_bit_cast(bf16x8, (u32x4){h[0], h[1], h[2], h[3]});
  lo = __builtin_bit_cast(bf16x8, (u32x4){l[0], l[1], l[2], l[3]});
}
// (A matrix instruction must not read a register that an ALU instruction wrote less than two issue slots before.  The
// compiler keeps that distance for instructions it knows; the matrix instructions here are assembly text to it, and it
// moves the conversions freely between them.  Every fragment therefore passes through two idle slots of its own,
// after its last conversion and before any matrix instruction that reads it.)
template <int HD>
__device__ __forceinline__ void split_k_tile(bf16x8 (&a)[HD / 8], const RawTile<HD>& r) {
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks) split8(r.v[ks], a[ks], a[HD / 16 + ks]);
#pragma unroll
  for (int f = 0; f < HD / 8; ++f) asm volatile("s_nop 1" : "+v"(a[f]));
}

// The matrix instructions are written out, with the query fragments at fixed places in the accumulation registers:
// fragment (pair p, block qb, k-step ks) of the sweep lives in a[4 f .. 4 f + 3], f = (p kQB + qb) KS + ks, for the
// whole sweep.  (Left to the compiler, these 256 registers per lane wander between the two register files and push
// the K fragments and accumulators into scratch memory.)  K fragments and results are ordinary values in vector
// registers, where the ALU reads the results.  PASS 1: D[token][query] = K x Q, PASS 2: D[query][token] = Q x K.
// The compiler does not know what these statements are and keeps no distance between them and the readers of their
// results.  The rule kept by hand: a result is read by an ALU instruction only after two more matrix instructions
// have been issued behind the one that produced it (pipelined steps: the order of every step is fixed by scheduling
// barriers), or after mma_results_ready().  The other way round - an ALU instruction writes a register that a matrix
// instruction then reads (fp32 caches: the split fragments) - two idle issue slots are put in between by hand as well.
#define CCD_ALL_ACC_REGISTERS "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127", "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143", "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159", "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191", "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207", "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", "a223", "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239", "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", "a253", "a254", "a255"

// every accumulation register belongs to the fragments from here on (the clobber list also makes the kernel claim them)
__device__ __forceinline__ void claim_acc_registers() { asm volatile("" ::: CCD_ALL_ACC_REGISTERS); }

// query fragment F (8 elements of the lane's query row, at `row` + byte_off) straight from global memory into its
// accumulation registers; the caller waits with q_frags_arrived() (the compiler does not see these loads)
template <int F, int BYTE_OFF>
__device__ __forceinline__ void load_q_frag_at(const uint16_t* row) {
  asm volatile("global_load_dwordx4 a[%1:%2], %0, off offset:%3"
               :: "v"(row), "n"(4 * F), "n"(4 * F + 3), "n"(BYTE_OFF)
               : "memory", CCD_ALL_ACC_REGISTERS);
}
template <int F>
__device__ __forceinline__ void zero_q_frag() {
  asm volatile("v_accvgpr_write_b32 a[%0], 0\n\tv_accvgpr_write_b32 a[%1], 0\n\t"
               "v_accvgpr_write_b32 a[%2], 0\n\tv_accvgpr_write_b32 a[%3], 0\n\ts_nop 3"
               :: "n"(4 * F), "n"(4 * F + 1), "n"(4 * F + 2), "n"(4 * F + 3)
               : CCD_ALL_ACC_REGISTERS);
}
// fragment F from four words in vector registers (fp32 caches: the split query rows)
template <int F>
__device__ __forceinline__ void put_q_frag(const bf16x8& f) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 w = __builtin_bit_cast(u32x4, f);
  // (four idle slots behind the writes: more than a matrix instruction needs before it may read these registers)
  asm volatile("v_accvgpr_write_b32 a[%0], %4\n\tv_accvgpr_write_b32 a[%1], %5\n\t"
               "v_accvgpr_write_b32 a[%2], %6\n\tv_accvgpr_write_b32 a[%3], %7\n\ts_nop 3"
               :: "n"(4 * F), "n"(4 * F + 1), "n"(4 * F + 2), "n"(4 * F + 3), "v"(w.x), "v"(w.y), "v"(w.z), "v"(w.w)
               : CCD_ALL_ACC_REGISTERS);
}
__device__ __forceinline__ void q_frags_arrived() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// F: index of the query fragment
template <int PASS, int F>
__device__ __forceinline__ void mma_first(floatx16& d, const bf16x8& k) {
  if (PASS == 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%2:%3], 0" : "=&v"(d) : "v"(k), "n"(4 * F), "n"(4 * F + 3) : CCD_ALL_ACC_REGISTERS);
  else           asm volatile("v_mfma_f32_32x32x16_bf16 %0, a[%2:%3], %1, 0" : "=&v"(d) : "v"(k), "n"(4 * F), "n"(4 * F + 3) : CCD_ALL_ACC_REGISTERS);
}
template <int PASS, int F>
__device__ __forceinline__ void mma_next(floatx16& d, const bf16x8& k) {
  if (PASS == 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%2:%3], %0" : "+v"(d) : "v"(k), "n"(4 * F), "n"(4 * F + 3) : CCD_ALL_ACC_REGISTERS);
  else           asm volatile("v_mfma_f32_32x32x16_bf16 %0, a[%2:%3], %1, %0" : "+v"(d) : "v"(k), "n"(4 * F), "n"(4 * F + 3) : CCD_ALL_ACC_REGISTERS);
}
// 24 idle issue cycles: more than the 8 passes of the last matrix instruction need to write their result
__device__ __forceinline__ void mma_results_ready(floatx16 (&acc)[kQB]) {
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc[0]), "+v"(acc[1]));
}

// compile-time loop: f(integral_constant<int, I>) for I = 0 .. N - 1
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// logits of one tile against block pair P, not overlapped with anything (first tile, ragged tile, careful redo)
template <class SH, int PASS, int P>
__device__ __forceinline__ void logits_now(floatx16 (&acc)[kQB], const bf16x8 (&ak)[SH::KF]) {
  static_for<0, SH::NM>([&](auto I) {
    constexpr int i = decltype(I)::value, j = i / 2, qb = i % 2, F = (P * kQB + qb) * SH::KF + SH::qfrag(j);
    if constexpr (j == 0) mma_first<PASS, F>(acc[qb], ak[SH::kfrag(0)]);
    else                  mma_next<PASS, F>(acc[qb], ak[SH::kfrag(j)]);
  });
  mma_results_ready(acc);
}

// One pipelined step: the NM matrix instructions of (tile, block pair P) into `nxt`, and between them the ALU work
// on the accumulators of the step before, cut into NCH chunks.  The first chunk runs behind the second matrix
// instruction at the earliest, the rest spread evenly, the last behind the last one: the results a chunk reads - block 0
// in the first half of the chunks, block 1 in the second - were produced at least three matrix instructions earlier.
template <class SH, int PASS, int P, class Chunk>
__device__ __forceinline__ void pipelined_step(floatx16 (&nxt)[kQB], const bf16x8 (&ak)[SH::KF], Chunk&& chunk) {
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, SH::NM>([&](auto I) {
    constexpr int i = decltype(I)::value, j = i / 2, qb = i % 2, F = (P * kQB + qb) * SH::KF + SH::qfrag(j);
    if constexpr (j == 0) mma_first<PASS, F>(nxt[qb], ak[SH::kfrag(0)]);
    else                  mma_next<PASS, F>(nxt[qb], ak[SH::kfrag(j)]);
    static_for<SH::chunks_by(i - 1), SH::chunks_by(i)>([&](auto C) { chunk(decltype(C)::value); });
    __builtin_amdgcn_sched_barrier(0);
  });
}

__device__ __forceinline__ float max16(const floatx16& v) {
  float t0 = fmaxf(fmaxf(v[0], v[1]), v[2]), t1 = fmaxf(fmaxf(v[3], v[4]), v[5]);
  float t2 = fmaxf(fmaxf(v[6], v[7]), v[8]), t3 = fmaxf(fmaxf(v[9], v[10]), v[11]);
  float t4 = fmaxf(fmaxf(v[12], v[13]), v[14]);
  return fmaxf(fmaxf(fmaxf(t0, t1), fmaxf(t2, t3)), fmaxf(t4, v[15]));
}

// negated log2-sum-exps of 32-row block `blk` of the sweep for the accumulator rows of this lane: rows
// 8 j + 4 half + 0..3 of a block are four consecutive floats.  `lane_base` = LDS byte address of neg_lse + 4 half, passed through an empty
// asm statement by the caller so that the reads are not hoisted out of the tile loop (the table does not change in
// there, and all 128 values of a lane would be kept in registers)
typedef __attribute__((address_space(3))) const float* LdsFloats;
__device__ __forceinline__ void load_neg_lse(float (&nl)[16], uint32_t lane_base, int blk) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) const f32x4* LdsQuad;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const f32x4 v = *reinterpret_cast<LdsQuad>((uintptr_t)(lane_base + (blk * 32 + 8 * j) * 4));
    nl[4 * j + 0] = v.x; nl[4 * j + 1] = v.y; nl[4 * j + 2] = v.z; nl[4 * j + 3] = v.w;
  }
}

// ET: element type of the caches in memory (uint16_t: bf16 bits; float: fp32, split on the fly)
// NP: pairs of 32-query blocks per sweep (1, 2 or 4: sweeps of 64, 128 or 256 query rows; units with few query rows
//     take the narrowest that holds them and spend one or two steps per tile instead of four)
template <int HD, class ET, int NP>
__global__ __launch_bounds__(kMT, 1) void score_unit_kernel(Dims D, ScorePlan pl, const ET* __restrict__ Q,
                                                            const ET* __restrict__ K,
                                                            const float2* __restrict__ part, float* __restrict__ u,
                                                            const ET* __restrict__ Kcap,
                                                            float* __restrict__ lse_io) {
  constexpr bool F32 = std::is_same<ET, float>::value;
  using SH = UnitShape<HD, F32>;
  constexpr int KF = SH::KF;           // fragments of a K tile / of a block of query rows
  constexpr int NCH = SH::NCH;         // ALU chunks per step
  constexpr int EPC = SH::EPC;         // accumulator elements per chunk
  constexpr int UQ = NP * kQB * 32;    // query rows per sweep
  static_assert(NP == 1 || NP == 2 || NP == 4, "steps per tile");
  __shared__ UnitLds<HD> sm;
  const int unit = D.unit0 + blockIdx.x;
  const UnitIdx ui = decode_unit(D, unit);
  const ET* Ku = K + kv_offset(D, ui);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const float c = D.scale_log2;
  // Tokens [D.head, n) are seen by every query row (all of them without a sliding window); the hidden head is left to
  // its own two small kernels.  Full 32-token tiles are dealt to the four waves in runs; a ragged last tile goes to the
  // last wave.
  const int tb = D.head;
  const int n_main = D.n - tb;
  const int full = n_main / kStep;
  const bool ragged = n_main > full * kStep;
  const int per = full / 4, rem = full % 4;
  const int s0 = wave * per + min(wave, rem);
  const int s1 = s0 + per + (wave < rem ? 1 : 0);            // full tiles [s0, s1) of pass 1
  const int s1p = s1 + ((ragged && wave == 3) ? 1 : 0);      // pass 2 takes the ragged tile like any other
  const int t_last = D.n - 1;
  float* uu = u + (int64_t)unit * D.n;
  claim_acc_registers();

  for (int qc = 0; qc < D.GP; qc += UQ) {
    // Fragments of the sweep's query rows into the accumulation registers: all 8 KS loads of a lane are in flight at
    // once, together with the first K tiles requested further down.  Rows past G * P (last sweep only) stay zero.
    if (qc + UQ > D.GP) {
      static_for<0, NP * kQB * KF>([&](auto Fc) { zero_q_frag<decltype(Fc)::value>(); });
    }
    static_for<0, NP * kQB>([&](auto Bc) {
      constexpr int blk = decltype(Bc)::value;
      const int q = qc + blk * 32 + col;
      if (q < D.GP) {
        const ET* row = Q + q_offset(D, ui, q) + half * 8;
        static_for<0, SH::KQ>([&](auto Kc) {
          constexpr int ks = decltype(Kc)::value;
          if constexpr (F32) {
            const f32x4 x[2] = {*reinterpret_cast<const f32x4*>(row + ks * 16),
                                *reinterpret_cast<const f32x4*>(row + ks * 16 + 4)};
            bf16x8 hi, lo;
            split8(x, hi, lo);
            put_q_frag<blk * KF + ks>(hi);
            put_q_frag<blk * KF + SH::KQ + ks>(lo);
          } else {
            load_q_frag_at<blk * KF + ks, ks * 32>(row);
          }
        });
      }
    });
    bf16x8 a[2][KF];
    floatx16 accA[kQB], accB[kQB];
    // fp32 caches: the tile requested last waits here, as it came from memory, until its turn to be split
    RawTile<F32 ? HD : 16> raw;
    // a[BUF] <- tile T of the wave, two tiles ahead of its use.  bf16: requested here.  fp32: tile T was requested one
    // tile earlier and is split into a[BUF] now; the request that goes out here is for tile T2, the one after it.
#define CCD_NEXT_TILE(BUF, T, T2)                                                        \
    if constexpr (F32) {                                                                 \
      split_k_tile<HD>(a[BUF], raw);                                                     \
      load_k_raw<HD>(raw, Ku, tb + (T2) * kStep, t_last, col, half);                     \
    } else {                                                                             \
      load_k_tile<HD>(a[BUF], Ku, tb + (T) * kStep, t_last, col, half);                  \
    }
    // a[BUF] <- tile T, needed at once (prologues, ragged tile, careful redo)
#define CCD_TILE_NOW(BUF, T)                                                             \
    if constexpr (F32) {                                                                 \
      load_k_raw<HD>(raw, Ku, tb + (T) * kStep, t_last, col, half);                      \
      split_k_tile<HD>(a[BUF], raw);                                                     \
    } else {                                                                             \
      load_k_tile<HD>(a[BUF], Ku, tb + (T) * kStep, t_last, col, half);                  \
    }

    if (!pl.lse_given) {
      // ---------------- pass 1 ----------------
      // per (pair, block): -reference * c and the sum in two partial chains
      float nm[NP][kQB], Z[NP][kQB][2];
#pragma unroll
      for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) { nm[p][qb] = -kNegHuge * c; Z[p][qb][0] = 0.f; Z[p][qb][1] = 0.f; }
      float m_ref[NP][kQB], Zs[NP][kQB];       // (reference, sum) pairs once the sweep is done
      // chunk j of the fold of pair P: elements j EPC .. + EPC - 1 of the 32 accumulator registers
#define CCD_FOLD1(CUR, P)                                                                 \
      [&](int j) {                                                                        \
        float t[EPC];                                                                     \
        _Pragma("unroll") for (int i = 0; i < EPC; ++i) {                                 \
          const int e = j * EPC + i;                                                      \
          t[i] = fmaf(CUR[e / 16][e % 16], c, nm[P][e / 16]);                             \
        }                                                                                 \
        _Pragma("unroll") for (int i = 0; i < EPC; ++i) t[i] = fast_exp2(t[i]);           \
        _Pragma("unroll") for (int i = 0; i < EPC; ++i) {                                 \
          const int e = j * EPC + i;                                                      \
          Z[P][e / 16][e & 1] += t[i];                                                    \
        }                                                                                 \
        /* the chunk ends here: its sums are demanded now, so its instructions are not  */  \
        /* sunk behind later matrix instructions (the sums are only read after the tile) */  \
        asm volatile("" : "+v"(Z[P][(j * EPC) / 16][0]), "+v"(Z[P][(j * EPC) / 16][1]));    \
      }
      if (s0 < s1) {
        if constexpr (F32) {
          load_k_raw<HD>(raw, Ku, tb + s0 * kStep, t_last, col, half);
          split_k_tile<HD>(a[0], raw);
          load_k_raw<HD>(raw, Ku, tb + min(s0 + 1, s1 - 1) * kStep, t_last, col, half);
        } else {
          load_k_tile<HD>(a[0], Ku, tb + s0 * kStep, t_last, col, half);
          load_k_tile<HD>(a[1], Ku, tb + min(s0 + 1, s1 - 1) * kStep, t_last, col, half);
        }
        q_frags_arrived();
        // the wave's first tile fixes the references and is folded without overlap
        static_for<0, NP>([&](auto Pc) {
          constexpr int p = decltype(Pc)::value;
          logits_now<SH, 1, p>(accA, a[0]);
#pragma unroll
          for (int qb = 0; qb < kQB; ++qb) nm[p][qb] = -max16(accA[qb]) * c;
          auto fold = CCD_FOLD1(accA, p);
#pragma unroll
          for (int j = 0; j < NCH; ++j) fold(j);
        });
        if constexpr (F32) {      // a[1] <- tile s0 + 1 (waiting in raw), a[0] <- tile s0 + 2, tile s0 + 3 requested
          split_k_tile<HD>(a[1], raw);
          load_k_raw<HD>(raw, Ku, tb + min(s0 + 2, s1 - 1) * kStep, t_last, col, half);
        }
        CCD_NEXT_TILE(0, min(s0 + 2, s1 - 1), min(s0 + 3, s1 - 1))
        int s = s0 + 1;
        logits_now<SH, 1, 0>(accA, a[1]);
        // Tile s: X holds the logits of (s, pair 0).  The steps take the other pairs of tile s from buffer CB and, last,
        // pair 0 of tile s + 1 from buffer NB; every step folds the pair computed by the step before.  The buffer of
        // tile s is free before the last step and takes tile s + 2.  With four or two pairs the logits of the next
        // tile end up in X again, with one pair in Y: there the two tiles of the loop body swap the accumulators.
#define CCD_P1_TILE(CB, NB, X, Y)                                                                 \
        if constexpr (NP == 4) {                                                                  \
          pipelined_step<SH, 1, 1>(Y, a[CB], CCD_FOLD1(X, 0));                                    \
          pipelined_step<SH, 1, 2>(X, a[CB], CCD_FOLD1(Y, 1));                                    \
          pipelined_step<SH, 1, 3>(Y, a[CB], CCD_FOLD1(X, 2));                                    \
        } else if constexpr (NP == 2) {                                                           \
          pipelined_step<SH, 1, 1>(Y, a[CB], CCD_FOLD1(X, 0));                                    \
        }                                                                                         \
        /* (always: a load under a condition would make every wait for K fragments a wait for all loads) */ \
        CCD_NEXT_TILE(CB, min(s + 2, s1 - 1), min(s + 3, s1 - 1))                                 \
        if constexpr (NP == 1) {                                                                  \
          pipelined_step<SH, 1, 0>(Y, a[NB], CCD_FOLD1(X, 0));                                    \
        } else {                                                                                  \
          pipelined_step<SH, 1, 0>(X, a[NB], CCD_FOLD1(Y, NP - 1));                               \
        }
        // (No branch inside a tile and none between the two tiles of the loop body: with straight-line code the
        // compiler can tell how many loads are in flight at every wait.  Behind the wave's last tile the last step
        // computes the logits of that tile's first pair once more; nobody reads them.)
        while (s + 1 < s1) {
          CCD_P1_TILE(1, 0, accA, accB)
          ++s;
          if constexpr (NP == 1) {
            CCD_P1_TILE(0, 1, accB, accA)
          } else {
            CCD_P1_TILE(0, 1, accA, accB)
          }
          ++s;
        }
        if (s < s1) {
          CCD_P1_TILE(1, 0, accA, accB)
        }
        mma_results_ready(accA);      // the surplus logits are in flight until here
        mma_results_ready(accB);
#undef CCD_P1_TILE
#undef CCD_FOLD1
        // Did a sum leave the fp32 range (or meet a NaN)?  Then this wave redoes its tokens with a running maximum.
        bool bad = false;
        const float inv_c = 1.0f / c;
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
          for (int qb = 0; qb < kQB; ++qb) {
            Zs[p][qb] = Z[p][qb][0] + Z[p][qb][1];
            m_ref[p][qb] = -nm[p][qb] * inv_c;
            bad |= !(Zs[p][qb] < INFINITY);
          }
        if (__any(bad)) {
#pragma unroll
          for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) { m_ref[p][qb] = kNegHuge; Zs[p][qb] = 0.f; }
          for (int t = s0; t < s1; ++t) {
            CCD_TILE_NOW(0, t)
            static_for<0, NP>([&](auto Pc) {
              constexpr int p = decltype(Pc)::value;
              logits_now<SH, 1, p>(accA, a[0]);
              fold_stats<false>(accA, m_ref[p], Zs[p], c, half, kStep);
            });
          }
        } else {
          // move each reference to where its sum is of order one (Z = mant * 2^e -> reference + e / c): the ragged
          // tile and the merges expect the magnitudes of a (maximum, sum) pair
#pragma unroll
          for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) {
              const int e = __builtin_amdgcn_frexp_expf(Zs[p][qb]);
              const float m_new = m_ref[p][qb] + (float)e * inv_c;
              Zs[p][qb] = __builtin_amdgcn_ldexpf(Zs[p][qb], -e) * fast_exp2(fmaf(m_ref[p][qb] - m_new, c, (float)e));
              m_ref[p][qb] = m_new;
            }
        }
      } else {
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
          for (int qb = 0; qb < kQB; ++qb) { m_ref[p][qb] = kNegHuge; Zs[p][qb] = 0.f; }
      }
      if (ragged && wave == 3) {
        CCD_TILE_NOW(0, full)
        q_frags_arrived();
        static_for<0, NP>([&](auto Pc) {
          constexpr int p = decltype(Pc)::value;
          logits_now<SH, 1, p>(accA, a[0]);
          fold_stats<true>(accA, m_ref[p], Zs[p], c, half, n_main - full * kStep);
        });
      }
      // the two lane halves hold different token rows of the same query row: merge, lower half writes
#pragma unroll
      for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
          const float m_o = __shfl_xor(m_ref[p][qb], 32), z_o = __shfl_xor(Zs[p][qb], 32);
          const float M = fmaxf(m_ref[p][qb], m_o);
          const float z = Zs[p][qb] * fast_exp2((m_ref[p][qb] - M) * c) + z_o * fast_exp2((m_o - M) * c);
          if (half == 0) sm.stat[wave][(p * kQB + qb) * 32 + col] = make_float2(M * c, z);
        }
    }

    // ---------------- merge: one log2-sum-exp per query row (thread = row of the sweep) ----------------
    {
      float2 cap = make_float2(kNegHuge, 0.f);     // the block of the CaP keys (causal variant), else nothing
      if constexpr (!F32) {          // (fp32 caches with CaP keys take the vector-ALU kernels: the host sees to that)
        if (Kcap != nullptr && wave < NP) {
          const uint16_t* Kc = Kcap + (int64_t)unit * D.P * HD;
          // the thread's own query row is one of the 2 x 32 rows of block pair `wave`: their fragments once more, in
          // vector registers this time (the registers of pass 1 are free here)
          bf16x8 bw[kQB][KF];
          load_q_frags<HD>(bw, D, ui, Q, qc + wave * (kQB * 32), col, half);
          cap = cap_block_stats<HD>(D, Kc, bw, qc + wave * (kQB * 32), col, half, c);
        }
      }
      __syncthreads();
      const int q = qc + threadIdx.x;
      const bool my_row = (int)threadIdx.x < UQ && q < D.GP;     // (threads past the sweep's rows have none)
      float lse = INFINITY;
      if (pl.lse_given) {            // the caller's normalisers (natural log): nothing to merge
        if (my_row) lse = lse_io[(int64_t)unit * D.GP + q] * 1.44269504088896340736f;
      } else if (my_row) {
        if (pl.head_block) {         // statistics of the windowed head, left there by its own kernel
          const float2 hd = part[extra_block_index(D, pl, unit, q)];
          const float Mh = fmaxf(cap.x, hd.x);
          cap = make_float2(Mh, cap.y * fast_exp2(cap.x - Mh) + hd.y * fast_exp2(hd.x - Mh));
        }
        float M = cap.x;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sm.stat[w][threadIdx.x].x);
        float z = cap.y * fast_exp2(cap.x - M);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float2 v = sm.stat[w][threadIdx.x];
          z += v.y * fast_exp2(v.x - M);
        }
        lse = M + __log2f(z);
        if (pl.head_block) lse_io[(int64_t)unit * D.GP + q] = lse;   // for the head's probabilities
      }
      sm.neg_lse[threadIdx.x] = -lse;
      __syncthreads();
    }

    // ---------------- pass 2: tiles s1p - 1 down to s0, in blocks of kUBlock ----------------
    // The sums of a block of tiles are collected in LDS and written out behind the block: a store (or, from the second
    // sweep on, a load and a store) inside the pipelined loop would sit among the K loads in the memory counter, and
    // every wait for K fragments would become a wait for everything.
    for (int sb = s1p; sb > s0; sb -= kUBlock) {
      const int sa = max(s0, sb - kUBlock);        // this block: tiles [sa, sb)
      float* ub = sm.ubuf[wave];
      float nl[kQB][16];      // normalisers of the pair being folded; each half is reloaded as soon as it is done with
      float us[2];
      uint32_t nl_base = (uint32_t)(uintptr_t)(LdsFloats)sm.neg_lse + 16 * half;
      // chunk j of the fold of a pair: 2^(x c - lse2) of EPC accumulator elements added to the token's sum; behind
      // the last chunk of a block of query rows, the normalisers of that block of pair NEXTP (the pair folded next) are
      // requested (with a single pair they never change)
#define CCD_FOLD2(CUR, NEXTP)                                                             \
      [&](int j) {                                                                        \
        float t[EPC];                                                                     \
        _Pragma("unroll") for (int i = 0; i < EPC; ++i) {                                 \
          const int e = j * EPC + i;                                                      \
          t[i] = fmaf(CUR[e / 16][e % 16], c, nl[e / 16][e % 16]);                        \
        }                                                                                 \
        _Pragma("unroll") for (int i = 0; i < EPC; ++i) t[i] = fast_exp2(t[i]);           \
        _Pragma("unroll") for (int i = 0; i < EPC; ++i) us[i & 1] += t[i];                \
        asm volatile("" : "+v"(us[0]), "+v"(us[1]));     /* as in pass 1 */               \
        if (NP > 1 && j == NCH / 2 - 1) load_neg_lse(nl[0], nl_base, (NEXTP) * kQB);      \
        if (NP > 1 && j == NCH - 1) load_neg_lse(nl[1], nl_base, (NEXTP) * kQB + 1);      \
      }
      int s = sb - 1;
      if constexpr (F32) {        // a[0] <- tile s, a[1] <- tile s - 1, tile s - 2 requested
        load_k_raw<HD>(raw, Ku, tb + s * kStep, t_last, col, half);
        split_k_tile<HD>(a[0], raw);
        load_k_raw<HD>(raw, Ku, tb + max(s - 1, sa) * kStep, t_last, col, half);
        split_k_tile<HD>(a[1], raw);
        load_k_raw<HD>(raw, Ku, tb + max(s - 2, sa) * kStep, t_last, col, half);
      } else {
        load_k_tile<HD>(a[0], Ku, tb + s * kStep, t_last, col, half);
        load_k_tile<HD>(a[1], Ku, tb + max(s - 1, sa) * kStep, t_last, col, half);
      }
      load_neg_lse(nl[0], nl_base, 0);
      load_neg_lse(nl[1], nl_base, 1);
      q_frags_arrived();
      logits_now<SH, 2, 0>(accA, a[0]);
      // Tile s: X holds the logits of (s, pair 0) and nl the normalisers of pair 0.  Same step structure as pass 1,
      // walking down; the token's sum is complete after the last step.
#define CCD_P2_TILE(CB, NB, X, Y)                                                                    \
      us[0] = 0.f; us[1] = 0.f;                                                                      \
      asm volatile("" : "+v"(nl_base));                                                              \
      if constexpr (NP == 4) {                                                                       \
        pipelined_step<SH, 2, 1>(Y, a[CB], CCD_FOLD2(X, 1));                                         \
        pipelined_step<SH, 2, 2>(X, a[CB], CCD_FOLD2(Y, 2));                                         \
        pipelined_step<SH, 2, 3>(Y, a[CB], CCD_FOLD2(X, 3));                                         \
      } else if constexpr (NP == 2) {                                                                \
        pipelined_step<SH, 2, 1>(Y, a[CB], CCD_FOLD2(X, 1));                                         \
      }                                                                                              \
      CCD_NEXT_TILE(CB, max(s - 2, sa), max(s - 3, sa))                                              \
      if constexpr (NP == 1) {                                                                       \
        pipelined_step<SH, 2, 0>(Y, a[NB], CCD_FOLD2(X, 0));                                         \
      } else {                                                                                       \
        pipelined_step<SH, 2, 0>(X, a[NB], CCD_FOLD2(Y, 0));                                         \
      }                                                                                              \
      {                                                                                              \
        float v = us[0] + us[1];                                                                     \
        v += __shfl_xor(v, 32);                                                                      \
        ub[(s - sa) * kStep + col] = v;      /* (both lane halves hold the same sum) */              \
      }
      while (s - 1 >= sa) {
        CCD_P2_TILE(0, 1, accA, accB)
        --s;
        if constexpr (NP == 1) {
          CCD_P2_TILE(1, 0, accB, accA)
        } else {
          CCD_P2_TILE(1, 0, accA, accB)
        }
        --s;
      }
      if (s >= sa) {
        CCD_P2_TILE(0, 1, accA, accB)
      }
      mma_results_ready(accA);        // the surplus logits are in flight until here
      mma_results_ready(accB);
#undef CCD_P2_TILE
#undef CCD_FOLD2
      // the block's sums (this wave wrote them, this wave reads them)
      const int t_blk = tb + sa * kStep, n_blk = min((sb - sa) * kStep, D.n - t_blk);
      for (int i = lane; i < n_blk; i += 64) uu[t_blk + i] = (qc == 0) ? ub[i] : uu[t_blk + i] + ub[i];
    }
    __syncthreads();   // the LDS tables are rewritten by the next sweep
#undef CCD_NEXT_TILE
#undef CCD_TILE_NOW
  }
}

}  // namespace

// One workgroup per unit pays when the units fill the chip round by round.
// (fp32 caches: head dimension 64 only - the split rows of 128 would need twice the fragment registers - and neither
// CaP keys in the softmax nor a sliding window, whose side kernels exist for bf16 only: the caller checks those)
bool score_unit_supported(const Dims& D) { return D.dtype == 1 ? (D.d == 64 || D.d == 128) : D.d == 64; }

// the kernel for (head dimension, cache type, pairs of query blocks per sweep)
template <int HD, class ET>
static void launch_score_unit_as(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const void* K_cap,
                                 const float2* part, float* u, float* lse_io, hipStream_t s) {
  dim3 grid((unsigned)D.units_run), block(kMT);
  const ET *q = (const ET*)Q, *k = (const ET*)K, *kc = (const ET*)K_cap;
  if (D.GP <= 64)       launch((score_unit_kernel<HD, ET, 1>), grid, block, s, D, pl, q, k, part, u, kc, lse_io);
  else if (D.GP <= 128) launch((score_unit_kernel<HD, ET, 2>), grid, block, s, D, pl, q, k, part, u, kc, lse_io);
  else                  launch((score_unit_kernel<HD, ET, 4>), grid, block, s, D, pl, q, k, part, u, kc, lse_io);
}

void launch_score_unit(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const void* K_cap,
                       const float2* part, float* u, float* lse_io, hipStream_t s) {
  if (D.dtype == 0)    launch_score_unit_as<64, float>(D, pl, Q, K, nullptr, part, u, lse_io, s);
  else if (D.d == 64)  launch_score_unit_as<64, uint16_t>(D, pl, Q, K, K_cap, part, u, lse_io, s);
  else                 launch_score_unit_as<128, uint16_t>(D, pl, Q, K, K_cap, part, u, lse_io, s);
}

}  // namespace ccd
