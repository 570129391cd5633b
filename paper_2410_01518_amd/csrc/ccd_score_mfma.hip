// Representative score of Eq. 2 for bf16 caches on the matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Same two-pass scheme as the vector-ALU kernels (the normaliser of every CaP query over ALL cached tokens is
// needed before probabilities can be summed over queries); the logits are recomputed in pass 2 rather than kept.
// A workgroup of 4 waves owns one token slice of one unit.  Each wave keeps the fragments of 64 query rows in
// registers for the whole slice; K streams HBM -> registers -> LDS (64-token tiles, double buffered, rows padded
// by 16 bytes so that fragment reads are bank-conflict free) and every wave reads each tile.
//
// The 32x32 accumulator tile puts its column index on the lane (lane % 32) and its row index on the register, so
// the operand order is chosen per pass to make the reduction run along registers, never across lanes:
//   pass 1  D[token][query] = Kfrag x Qfrag : each lane owns one query, folds its 16 token rows into a running
//           (max, sum of 2^(x - max)) pair;
//   pass 2  D[query][token] = Qfrag x Kfrag : each lane owns one token, adds 2^(x - lse2[query]) of its 16 query
//           rows into one partial sum.
// The fragment a lane holds is the same in both roles: the vector with index lane % 32, elements
// 8*(lane/32) .. +7 of each 16-element step of the head dimension.
#include "ccd_common.h"

namespace ccd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMT = 256;            // threads per workgroup (4 waves)
constexpr int kTile = 64;           // tokens per LDS buffer
constexpr int kQB = 2;              // 32-query blocks per wave
constexpr int kQPerPass = 4 * kQB * 32;   // query rows a workgroup covers per sweep over its slice
constexpr int kMaxSlice2 = 1024;    // pass-2 slice limit (per-wave partial sums live in LDS)
constexpr float kNegHuge = -1.0e30f;

// row of the 32x32 accumulator tile held in register r by a lane of half `half` (lane / 32)
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// block -> (unit, slice): consecutive blocks go to different XCDs, so the slices of one unit are placed on
// blocks with the same residue mod 8 and share that XCD's L2 for their query fragments.
__device__ __forceinline__ bool decode_block(const Dims& D, int n_slices, int& unit, int& slice) {
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  unit = (j / n_slices) * 8 + xcd;
  slice = j % n_slices;
  return unit < D.units;
}

template <int HD>
struct Tiles {
  static constexpr int kRowBytes = HD * 2 + 16;
  static constexpr int kChunksPerRow = HD / 8;                       // 16-byte chunks
  static constexpr int kChunksPerThread = kTile * kChunksPerRow / kMT;
};

template <int HD>
__device__ __forceinline__ void load_tile(uint4 (&g)[Tiles<HD>::kChunksPerThread], const uint16_t* Ku, int tile_t0, int t1) {
#pragma unroll
  for (int i = 0; i < Tiles<HD>::kChunksPerThread; ++i) {
    const int e = threadIdx.x + i * kMT;
    const int row = e / Tiles<HD>::kChunksPerRow, c = e % Tiles<HD>::kChunksPerRow;
    const int tok = tile_t0 + row;
    g[i] = tok < t1 ? *reinterpret_cast<const uint4*>(Ku + (int64_t)tok * HD + c * 8) : make_uint4(0, 0, 0, 0);
  }
}

template <int HD>
__device__ __forceinline__ void store_tile(const uint4 (&g)[Tiles<HD>::kChunksPerThread], uint8_t* buf) {
#pragma unroll
  for (int i = 0; i < Tiles<HD>::kChunksPerThread; ++i) {
    const int e = threadIdx.x + i * kMT;
    const int row = e / Tiles<HD>::kChunksPerRow, c = e % Tiles<HD>::kChunksPerRow;
    *reinterpret_cast<uint4*>(buf + row * Tiles<HD>::kRowBytes + c * 16) = g[i];
  }
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

template <int HD>
__global__ __launch_bounds__(kMT, 2) void stats_mfma_kernel(Dims D, ScorePlan pl, const uint16_t* __restrict__ Q,
                                                            const uint16_t* __restrict__ K, float2* __restrict__ part) {
  constexpr int KS = HD / 16;
  constexpr int ROWB = Tiles<HD>::kRowBytes;
  __shared__ __attribute__((aligned(16))) uint8_t lds[2][kTile * ROWB];
  int unit, slice;
  if (!decode_block(D, pl.n_slices1, unit, slice)) return;
  const UnitIdx ui = decode_unit(D, unit);
  const uint16_t* Ku = K + kv_offset(D, ui);
  const int t0 = slice * pl.slice1, t1 = min(D.n, t0 + pl.slice1);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const float c = D.scale_log2;

  for (int qc = 0; qc < D.GP; qc += kQPerPass) {
    bf16x8 bq[kQB][KS];
    load_q_frags<HD>(bq, D, ui, Q, qc + wave * (kQB * 32), col, half);
    float m_raw[kQB], Z[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) { m_raw[qb] = kNegHuge; Z[qb] = 0.f; }

    uint4 g[Tiles<HD>::kChunksPerThread];
    load_tile<HD>(g, Ku, t0, t1);
    for (int it = 0; it < ntiles; ++it) {
      uint8_t* buf = lds[it & 1];
      store_tile<HD>(g, buf);
      __syncthreads();
      if (it + 1 < ntiles) load_tile<HD>(g, Ku, t0 + (it + 1) * kTile, t1);
      const int tile_t0 = t0 + it * kTile;
#pragma unroll
      for (int sub = 0; sub < kTile / 32; ++sub) {
        const int nvalid = t1 - (tile_t0 + sub * 32);
        if (nvalid <= 0) break;
        bf16x8 a[KS];
        const uint8_t* rowp = buf + (sub * 32 + col) * ROWB + half * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(rowp + ks * 32);
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
          floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bq[qb][ks], acc, 0, 0, 0);
          if (nvalid < 32) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (acc_row(r, half) >= nvalid) acc[r] = -INFINITY;
          }
          float tmax = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, acc[r]);
          const float m_new = fmaxf(m_raw[qb], tmax);
          float z = Z[qb] * fast_exp2((m_raw[qb] - m_new) * c);
          m_raw[qb] = m_new;
          const float negm = -m_new * c;
#pragma unroll
          for (int r = 0; r < 16; ++r) z += fast_exp2(fmaf(acc[r], c, negm));
          Z[qb] = z;
        }
      }
    }
    __syncthreads();   // the LDS buffers are refilled by the next sweep

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

template <int HD>
__global__ __launch_bounds__(kMT, 2) void prob_mfma_kernel(Dims D, ScorePlan pl, const uint16_t* __restrict__ Q,
                                                           const uint16_t* __restrict__ K,
                                                           const float* __restrict__ lse2, float* __restrict__ u) {
  constexpr int KS = HD / 16;
  constexpr int ROWB = Tiles<HD>::kRowBytes;
  __shared__ __attribute__((aligned(16))) uint8_t lds[2][kTile * ROWB];
  __shared__ float up[4][kMaxSlice2];     // per-wave partial sums over the wave's query rows
  int unit, slice;
  if (!decode_block(D, pl.n_slices2, unit, slice)) return;
  const UnitIdx ui = decode_unit(D, unit);
  const uint16_t* Ku = K + kv_offset(D, ui);
  const int t0 = slice * pl.slice2, t1 = min(D.n, t0 + pl.slice2);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  const float c = D.scale_log2;

  for (int qc = 0; qc < D.GP; qc += kQPerPass) {
    bf16x8 bq[kQB][KS];
    load_q_frags<HD>(bq, D, ui, Q, qc + wave * (kQB * 32), col, half);
    float neg_lse[kQB][16];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int q = qc + wave * (kQB * 32) + qb * 32 + acc_row(r, half);
        neg_lse[qb][r] = q < D.GP ? -lse2[(int64_t)unit * D.GP + q] : -INFINITY;
      }

    uint4 g[Tiles<HD>::kChunksPerThread];
    load_tile<HD>(g, Ku, t0, t1);
    for (int it = 0; it < ntiles; ++it) {
      uint8_t* buf = lds[it & 1];
      store_tile<HD>(g, buf);
      __syncthreads();
      if (it + 1 < ntiles) load_tile<HD>(g, Ku, t0 + (it + 1) * kTile, t1);
#pragma unroll
      for (int sub = 0; sub < kTile / 32; ++sub) {
        if (t0 + it * kTile + sub * 32 >= t1) break;
        bf16x8 a[KS];
        const uint8_t* rowp = buf + (sub * 32 + col) * ROWB + half * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(rowp + ks * 32);
        float usum = 0.f;
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
          floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[qb][ks], a[ks], acc, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 16; ++r) usum += fast_exp2(fmaf(acc[r], c, neg_lse[qb][r]));
        }
        usum += __shfl_xor(usum, 32);
        if (half == 0) {
          float* dst = &up[wave][it * kTile + sub * 32 + col];
          *dst = (qc == 0) ? usum : *dst + usum;
        }
      }
    }
    __syncthreads();
  }
  float* uu = u + (int64_t)unit * D.n + t0;
  for (int t = threadIdx.x; t < t1 - t0; t += kMT) uu[t] = (up[0][t] + up[1][t]) + (up[2][t] + up[3][t]);
}

}  // namespace

int mfma_max_slice2() { return kMaxSlice2; }

void launch_stats_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, float2* part, hipStream_t s) {
  dim3 grid((unsigned)((D.units + 7) / 8 * 8) * pl.n_slices1), block(kMT);
  if (D.d == 64)
    hipLaunchKernelGGL((stats_mfma_kernel<64>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part);
  else
    hipLaunchKernelGGL((stats_mfma_kernel<128>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, part);
}

void launch_prob_mfma(const Dims& D, const ScorePlan& pl, const void* Q, const void* K, const float* lse2, float* u,
                      hipStream_t s) {
  dim3 grid((unsigned)((D.units + 7) / 8 * 8) * pl.n_slices2), block(kMT);
  if (D.d == 64)
    hipLaunchKernelGGL((prob_mfma_kernel<64>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, lse2, u);
  else
    hipLaunchKernelGGL((prob_mfma_kernel<128>), grid, block, 0, s, D, pl, (const uint16_t*)Q, (const uint16_t*)K, lse2, u);
}

}  // namespace ccd
