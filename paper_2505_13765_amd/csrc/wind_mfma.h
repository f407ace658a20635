// bf16 MFMA tile core for gfx950: C[M,N] += A[M,K] * B[N,K]^T, both operands K-contiguous.
//
// One workgroup owns a BM x BN tile, one wave a WM x WN sub-tile made of 32x32 blocks that
// v_mfma_f32_32x32x16_bf16 accumulates in fp32.  K is walked in steps of 64: the next step's
// operands are fetched from global memory into registers while the current step is multiplied out
// of LDS (two LDS stages, one barrier per step).  LDS rows are padded from 128 to 144 bytes so the
// 16-byte fragment reads of 32 consecutive rows fall on distinct banks.
//
// Fragment layout of the 32x32x16 instruction (lane l of 64):
//   A operand: row l%32 of the block, k = 8*(l/32) .. 8*(l/32)+7     (8 bf16 = 16 bytes)
//   B operand: column l%32 of the block, same k
//   accumulator register r (0..15): row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma once
#include "wind_util.h"

namespace wind {

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int BK = 64;
  static constexpr int LDS = BK + 8;  // row stride in bf16 elements
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
  static constexpr int NWAVES = WAVES_M * WAVES_N, NT = NWAVES * kWave;
  static constexpr int MI = WM / 32, NI = WN / 32;
  static constexpr int A_PER_T = BM * (BK / 8) / NT, B_PER_T = BN * (BK / 8) / NT;
  static constexpr int STAGE_ELEMS = (BM + BN) * LDS;
  static constexpr int SMEM_BYTES = 2 * STAGE_ELEMS * 2;
  static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
  static_assert((BM * (BK / 8)) % NT == 0 && (BN * (BK / 8)) % NT == 0, "loader shape");
  static_assert(WN <= 128, "a key carries 7 column bits");
};

// aload(i, row_in_tile, k) returns 8 consecutive bf16 of A's row as a u32x4; i is the index of the
// chunk among this thread's A_PER_T chunks (its row is the same at every K step).
// Bw points at row n0 of B ([N, K] bf16, at least BN rows readable).  K % 64 == 0.
template <class Cfg, class ALoad>
__device__ __forceinline__ void tile_gload(const ALoad &aload, const bf16_t *__restrict__ Bw, int K, int kt,
                                           int tid, u32x4 (&ra)[Cfg::A_PER_T], u32x4 (&rb)[Cfg::B_PER_T]) {
#pragma unroll
  for (int i = 0; i < Cfg::A_PER_T; ++i) {
    const int c = tid + i * Cfg::NT;
    ra[i] = aload(i, c >> 3, kt * 64 + (c & 7) * 8);
  }
#pragma unroll
  for (int i = 0; i < Cfg::B_PER_T; ++i) {
    const int c = tid + i * Cfg::NT;
    rb[i] = *reinterpret_cast<const u32x4 *>(Bw + (size_t)(c >> 3) * K + kt * 64 + (c & 7) * 8);
  }
}

template <class Cfg>
__device__ __forceinline__ void tile_sstore(bf16_t *stage, int tid, const u32x4 (&ra)[Cfg::A_PER_T],
                                            const u32x4 (&rb)[Cfg::B_PER_T]) {
  bf16_t *sA = stage, *sB = stage + Cfg::BM * Cfg::LDS;
#pragma unroll
  for (int i = 0; i < Cfg::A_PER_T; ++i) {
    const int c = tid + i * Cfg::NT;
    *reinterpret_cast<u32x4 *>(sA + (c >> 3) * Cfg::LDS + (c & 7) * 8) = ra[i];
  }
#pragma unroll
  for (int i = 0; i < Cfg::B_PER_T; ++i) {
    const int c = tid + i * Cfg::NT;
    *reinterpret_cast<u32x4 *>(sB + (c >> 3) * Cfg::LDS + (c & 7) * 8) = rb[i];
  }
}

template <class Cfg, class ALoad>
__device__ __forceinline__ void gemm_mainloop(const ALoad &aload, const bf16_t *__restrict__ Bw,
                                              int K, bf16_t *smem,
                                              f32x16 (&acc)[Cfg::MI][Cfg::NI]) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
  u32x4 ra[Cfg::A_PER_T], rb[Cfg::B_PER_T];

#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const int KT = K / 64;
  tile_gload<Cfg>(aload, Bw, K, 0, tid, ra, rb);
  tile_sstore<Cfg>(smem, tid, ra, rb);
  __syncthreads();
  const int a_off = wm * Cfg::WM * Cfg::LDS + (lane & 31) * Cfg::LDS + (lane >> 5) * 8;
  const int b_off = (Cfg::BM + wn * Cfg::WN) * Cfg::LDS + (lane & 31) * Cfg::LDS + (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    const bool more = kt + 1 < KT;
    if (more) tile_gload<Cfg>(aload, Bw, K, kt + 1, tid, ra, rb);
    const bf16_t *stage = smem + (kt & 1) * Cfg::STAGE_ELEMS;
    const bf16_t *a = stage + a_off;
    const bf16_t *b = stage + b_off;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[Cfg::MI], bfr[Cfg::NI];
#pragma unroll
      for (int mi = 0; mi < Cfg::MI; ++mi)
        af[mi] = *reinterpret_cast<const bf16x8 *>(a + mi * 32 * Cfg::LDS + ks * 16);
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
        bfr[ni] = *reinterpret_cast<const bf16x8 *>(b + ni * 32 * Cfg::LDS + ks * 16);
#pragma unroll
      for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < Cfg::NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
    }
    if (more) tile_sstore<Cfg>(smem + ((kt + 1) & 1) * Cfg::STAGE_ELEMS, tid, ra, rb);
    __syncthreads();
  }
}

// row (within the wave's WM rows) of accumulator block mi, register r, for this lane
__device__ __forceinline__ int acc_row(int mi, int r, int lane) {
  return mi * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

// ---------------------------------------------------------------------------------------------
// Row-wise top-2 across the 32 lanes that share lane/32 (they hold the 32 columns of a block).
// Every lane enters with N (logit, column) key pairs, one per accumulator row slot; each step
// hands half of the slots to a partner lane and merges the partner's half, so after the steps
// every lane owns N/32 slots (at least one), fully reduced.  The first four steps pair lanes inside
// a row of 16 with DPP permutations, which cost no more than a move (row mirror i <-> 15-i, half
// mirror i <-> 7-i, then i ^ 2 and i ^ 1: any sequence of perfect matchings works as long as the
// two partners own the same slots and disjoint columns); only the last step, which carries the
// fewest slots, crosses the two rows of 16 through the LDS crossbar.
template <int S>
__device__ __forceinline__ float rowtop2_partner(float x) {
  if constexpr (S == 0) return dpp_f32<0x140>(x);        // row_mirror
  else if constexpr (S == 1) return dpp_f32<0x141>(x);   // row_half_mirror
  else if constexpr (S == 2) return dpp_f32<0x4E>(x);    // quad_perm [2,3,0,1]
  else if constexpr (S == 3) return dpp_f32<0xB1>(x);    // quad_perm [1,0,3,2]
  else return __shfl_xor(x, 16, kWave);
}
// the lane bit that decides which half of the slots a lane keeps at step S
template <int S>
constexpr int rowtop2_bit() { return S == 0 ? 8 : S == 1 ? 4 : S == 2 ? 2 : S == 3 ? 1 : 16; }

template <int N, int S>
struct RowTop2 {
  template <int NO>
  static __device__ __forceinline__ void run(float (&k1)[N], float (&k2)[N], int lane, float (&o1)[NO], float (&o2)[NO]) {
    if constexpr (S == 5) {
      static_assert(N == NO, "slots per lane");
#pragma unroll
      for (int i = 0; i < N; ++i) { o1[i] = k1[i]; o2[i] = k2[i]; }
    } else if constexpr (N == 1) {
      float r1 = rowtop2_partner<S>(k1[0]), r2 = rowtop2_partner<S>(k2[0]);
      merge_top2(k1[0], k2[0], r1, r2);
      RowTop2<1, S + 1>::run(k1, k2, lane, o1, o2);
    } else {
      const bool up = (lane & rowtop2_bit<S>()) != 0;
      float n1[N / 2], n2[N / 2];
#pragma unroll
      for (int i = 0; i < N / 2; ++i) {
        float keep1 = up ? k1[i + N / 2] : k1[i], keep2 = up ? k2[i + N / 2] : k2[i];
        float send1 = up ? k1[i] : k1[i + N / 2], send2 = up ? k2[i] : k2[i + N / 2];
        float r1 = rowtop2_partner<S>(send1), r2 = rowtop2_partner<S>(send2);
        merge_top2(keep1, keep2, r1, r2);
        n1[i] = keep1;
        n2[i] = keep2;
      }
      RowTop2<N / 2, S + 1>::run(n1, n2, lane, o1, o2);
    }
  }
};
// First slot a lane owns after RowTop2<NS, 0>, and how many (consecutive) slots.
template <int NS>
__device__ __forceinline__ int rowtop2_first_slot(int lane) {
  constexpr int masks[5] = {8, 4, 2, 1, 16};   // rowtop2_bit<0..4>
  int base = 0, n = NS;
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    if (n > 1) {
      n >>= 1;
      if (lane & masks[i]) base += n;
    }
  }
  return base;
}
template <int NS>
constexpr int rowtop2_slots_per_lane() { return NS >= 32 ? NS / 32 : 1; }

}  // namespace wind
