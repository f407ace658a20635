// bf16 MFMA tile core with the work split by wave: four waves multiply, four waves only fetch.
//
// C[64 MI, 128] += A[64 MI, K] * B[128, K]^T for dense bf16 rows in memory, K in tiles of 64.
// A workgroup has eight waves (two per SIMD).  Waves 0..3 (the multipliers) own a (32 MI) x 64 block
// each, read their operand fragments from LDS and issue MFMAs, and never touch global memory inside
// the loop.  Waves 4..7 (the fetchers) issue the direct-to-LDS loads of the K tiles ahead and wait
// for them.  A wave issues its instructions in order, so a wave that does both stands at the vector
// memory pipeline's door whenever that pipeline is backed up, and its MFMA pipe runs dry meanwhile:
// with one 256 x 128 tile per CU the loads alone keep the pipeline 75 % busy.  Split by role, the
// fetchers absorb that waiting and the multipliers see only LDS.
//
// LDS: a ring of B stages (128 rows x 128 bytes each) at a fixed place, then a ring of A stages
// (64 MI rows x 128 bytes each).  The B ring does not depend on the tile height, so its first stages
// can be requested before the number of rows of this launch is known.  Chunk swizzle and the
// layout of a 1 KB load are those of wind_mfma_dma.h.
//
// Hand-over: one workgroup barrier per K tile.  Barrier j (j = 0 .. KT-1) is passed by a fetcher
// once its own loads of tile j have landed, and by a multiplier once its LDS reads of tile j-1 are
// complete; after it the multipliers work on tile j and the fetchers refill the stage of tile j-1
// with tile j-1+NS.  The multipliers sit at the barrier with the fragments of their last K step in
// registers, so their MFMA pipes keep running across it.
#pragma once
#include "wind_mfma_dma.h"

namespace wind {

template <int MI_>
struct WsCfg {
  static constexpr int MI = MI_, NI = 2;                    // a multiplier's block: 32 MI rows x 64 columns
  static constexpr int BM = 64 * MI_, BN = 128, BK = 64, ROWB = 128, CPR = 8, KSTEPS = 4;
  static constexpr int WM = 32 * MI_, WN = 64, WAVES_M = 2, WAVES_N = 2;
  static constexpr int NMUL = 4, NFETCH = 4, NT = (NMUL + NFETCH) * kWave;
  static constexpr int NS = MI_ == 4 ? 3 : 4;               // ring depth
  static constexpr int B_STAGE = BN * ROWB, A_STAGE = BM * ROWB;
  static constexpr int A_BASE = 4 * B_STAGE;                // room for the deepest B ring
  static constexpr int SMEM_BYTES = A_BASE + NS * A_STAGE;
  static constexpr int LB = BN / 8 / NFETCH, LA = BM / 8 / NFETCH;   // loads per fetcher and tile: B, A
  static constexpr int LPW = LA + LB;
  static_assert(SMEM_BYTES <= 160 * 1024, "LDS");
  static_assert((NS - 1) * LPW < 64, "vmcnt range");
};
constexpr int kWsSmemBytes = WsCfg<4>::SMEM_BYTES;
static_assert(WsCfg<1>::SMEM_BYTES <= kWsSmemBytes && WsCfg<2>::SMEM_BYTES <= kWsSmemBytes &&
                  WsCfg<3>::SMEM_BYTES <= kWsSmemBytes, "one launch size for every tile height");

// Fetcher side, first part: the B loads of the ring's first three stages (every tile height has at
// least three).  Needs nothing but the column tile.  With fewer than three K tiles the last one is
// fetched again into the stages nobody reads, so that the number of loads in flight stays the same.
__device__ __forceinline__ void ws_fetch_b_head(const bf16_t *__restrict__ Bw, int K, unsigned char *smem) {
  const int lane = threadIdx.x & 63, fw = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) - 4;
  const int KT = K / 64;
#pragma unroll
  for (int s = 0; s < 3; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (fw * 4 + i) * 8 + lane / 8, ch = (lane % 8) ^ lds_swizzle<8>(row);
      __builtin_amdgcn_global_load_lds((gmem_cptr *)(Bw + (size_t)row * K + (s < KT ? s : KT - 1) * 64 + ch * 8),
                                       (lds_ptr *)(smem + s * (128 * 128) + (fw * 4 + i) * 1024), 16, 0, 0);
    }
}

// Fetcher side, the rest.  A points at the tile's first row (rows K apart), Bw at the column tile's
// first row of B.  Every fetcher executes exactly KT barriers and leaves with loads possibly still
// in flight (redundant ones, when K has fewer tiles than the ring has stages): the caller waits for
// them before the LDS is reused or the wave ends.
template <class Cfg>
__device__ __forceinline__ void ws_fetch(const bf16_t *__restrict__ A, const bf16_t *__restrict__ Bw, int K,
                                         unsigned char *smem) {
  // the wave number as a scalar: LDS destinations (M0) are then computed on the scalar unit
  const int lane = threadIdx.x & 63, fw = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) - 4;
  const int KT = K / 64;
  uint32_t aoff[Cfg::LA], boff[Cfg::LB];   // byte offset of this lane's 16 bytes within a K tile's rows
#pragma unroll
  for (int i = 0; i < Cfg::LA; ++i) {
    const int row = (fw * Cfg::LA + i) * 8 + lane / 8;
    aoff[i] = (uint32_t)(row * K * 2 + ((lane % 8) ^ lds_swizzle<8>(row)) * 16);
  }
#pragma unroll
  for (int i = 0; i < Cfg::LB; ++i) {
    const int row = (fw * Cfg::LB + i) * 8 + lane / 8;
    boff[i] = (uint32_t)(row * K * 2 + ((lane % 8) ^ lds_swizzle<8>(row)) * 16);
  }
  auto issue_a = [&](int kt, int stage) {
    unsigned char *dst = smem + Cfg::A_BASE + stage * Cfg::A_STAGE + fw * Cfg::LA * 1024;
    const char *base = reinterpret_cast<const char *>(A) + kt * 128;
#pragma unroll
    for (int i = 0; i < Cfg::LA; ++i)
      __builtin_amdgcn_global_load_lds((gmem_cptr *)(base + aoff[i]), (lds_ptr *)(dst + i * 1024), 16, 0, 0);
  };
  auto issue_b = [&](int kt, int stage) {
    unsigned char *dst = smem + stage * Cfg::B_STAGE + fw * Cfg::LB * 1024;
    const char *base = reinterpret_cast<const char *>(Bw) + kt * 128;
#pragma unroll
    for (int i = 0; i < Cfg::LB; ++i)
      __builtin_amdgcn_global_load_lds((gmem_cptr *)(base + boff[i]), (lds_ptr *)(dst + i * 1024), 16, 0, 0);
  };
  // head: B0 B1 B2 are on their way (ws_fetch_b_head); A0 A1 A2, then the fourth stage whole
  // (past the end of K the last tile is fetched again, into a stage nobody reads)
  auto last = [&](int kt) { return kt < KT ? kt : KT - 1; };
  issue_a(0, 0); issue_a(last(1), 1); issue_a(last(2), 2);
  if (Cfg::NS == 4) { issue_b(last(3), 3); issue_a(last(3), 3); }
  constexpr int kTail = (Cfg::NS - 3) * Cfg::LPW;   // loads of the fourth stage
  wait_vmcnt<2 * Cfg::LA + kTail>();                // tile 0 has landed
  __builtin_amdgcn_s_barrier();
  if (KT == 1) return;
  wait_vmcnt<Cfg::LA + kTail>();                    // tile 1
  __builtin_amdgcn_s_barrier();
  // steady state: after barrier j the stage of tile j-1 is free
  int stage = 0;
  for (int j = 1; j + 1 < KT; ++j) {
    const int kn = j - 1 + Cfg::NS;
    if (kn < KT) {
      issue_b(kn, stage);
      issue_a(kn, stage);
    }
    stage = stage + 1 == Cfg::NS ? 0 : stage + 1;
    // tile j+1 must have landed; younger loads may stay in flight: tiles j+2 .. min(kn, KT-1)
    const int younger = (kn < KT ? kn : KT - 1) - (j + 1);
    if (younger >= 2) wait_vmcnt<2 * Cfg::LPW>();
    else if (younger == 1) wait_vmcnt<Cfg::LPW>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
  }
}

// Multiplier side.  The caller sets acc (bias or zero) before the call.  Every multiplier executes
// exactly KT barriers.  SWAP as in gemm_mainloop_dma_src: the transposed block is accumulated.
template <class Cfg, bool SWAP>
__device__ __forceinline__ void ws_multiply(int K, const unsigned char *smem, f32x16 (&acc)[Cfg::MI][Cfg::NI]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
  const int KT = K / 64;
  const int frow = lane & 31, kc = lane >> 5, sw = lds_swizzle<8>(frow);
  const int a_off = Cfg::A_BASE + (wm * Cfg::WM + frow) * Cfg::ROWB;
  const int b_off = (wn * Cfg::WN + frow) * Cfg::ROWB;
  bf16x8 af[2][Cfg::MI], bfr[2][Cfg::NI];
  auto load_frags = [&](int set, int stage, int ks) {
    const int chunk_off = ((2 * ks + kc) ^ sw) * 16;
    const unsigned char *pa = smem + a_off + stage * Cfg::A_STAGE + chunk_off;
    const unsigned char *pb = smem + b_off + stage * Cfg::B_STAGE + chunk_off;
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi) af[set][mi] = *reinterpret_cast<const bf16x8 *>(pa + mi * 32 * Cfg::ROWB);
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni) bfr[set][ni] = *reinterpret_cast<const bf16x8 *>(pb + ni * 32 * Cfg::ROWB);
  };
  auto mfma_step = [&](int set) {
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
        acc[mi][ni] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][ni], af[set][mi], acc[mi][ni], 0, 0, 0)
                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][mi], bfr[set][ni], acc[mi][ni], 0, 0, 0);
  };
  // The reads of the next K step are woven into the current step's MFMAs, one read behind each of
  // the first MI + NI MFMAs: a wave issues in order, and a burst of reads that has to queue at the
  // LDS would hold the MFMAs behind it back (measured: the multipliers' loop 12.4 -> 10.4 us for
  // a 256 x 128 x 1024 tile with nothing else running).
  auto weave = [] {
#pragma unroll
    for (int q = 0; q < Cfg::MI + Cfg::NI; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
    }
  };
  static_assert(Cfg::MI * Cfg::NI >= Cfg::MI + Cfg::NI || Cfg::MI == 1, "MFMAs to weave the reads into");
  __builtin_amdgcn_s_barrier();   // barrier 0: tile 0 has landed
  asm volatile("" ::: "memory");
  load_frags(0, 0, 0);
  int stage = 0;
  for (int kt = 0; kt + 1 < KT; ++kt) {
    const int next = stage + 1 == Cfg::NS ? 0 : stage + 1;
#pragma unroll
    for (int ks = 0; ks + 1 < Cfg::KSTEPS; ++ks) {
      load_frags((ks + 1) & 1, stage, ks + 1);
      mfma_step(ks & 1);
      weave();
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // my reads of tile kt are complete
    __builtin_amdgcn_s_barrier();                        // barrier kt+1
    asm volatile("" ::: "memory");
    load_frags(0, next, 0);
    mfma_step(1);
    weave();
    __builtin_amdgcn_sched_barrier(0);
    stage = next;
  }
#pragma unroll
  for (int ks = 0; ks < Cfg::KSTEPS; ++ks) {   // last tile
    if (ks + 1 < Cfg::KSTEPS) load_frags((ks + 1) & 1, stage, ks + 1);
    mfma_step(ks & 1);
  }
}

}  // namespace wind
