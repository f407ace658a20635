// bf16 MFMA tile core with direct global -> LDS loads (gfx950 global_load_lds_dwordx4) and a
// multi-stage LDS ring, for operands that already sit in memory as dense bf16 rows.
//
// C[BM,BN] += A[BM,K] * B[BN,K]^T.  K is walked in steps of BK; each step's A and B rows are
// fetched straight into one LDS stage by 16-byte-per-lane loads that bypass the register file, and
// NSTAGE-1 steps are kept in flight.  BK = 64 is the one to use: its 128-byte row segments are
// whole cache lines (64-byte segments of BK = 32 measured 77 instead of 118 GB/s per CU from L2).
//
// LDS layout of a stage: row r (A rows first, then B rows) occupies BK*2 dense bytes.  One load
// instruction of a wave fills 1024 contiguous bytes: lane l writes bytes [16 l, 16 l + 16) (checked
// on the hardware).  Bank conflicts of the 16-byte fragment reads are avoided by a swizzle instead
// of padding: the 16-byte chunk c of row r is stored at chunk position c ^ s(r).  The LDS has 64
// banks of 4 bytes (256 bytes per clock) and serves a 16-byte read 16 lanes at a time, so 16
// consecutive rows must land on 16 distinct 16-byte slots modulo 256 bytes: s(r) = (r >> 1) & 7 for
// 128-byte rows (BK = 64), (r >> 2) & 3 for 64-byte rows (BK = 32); measured 224-235 of 256 B/clk
// against 120 B/clk for the 32-bank swizzle r & 7.  The load side applies the
// swizzle by choosing which global chunk a lane fetches; it stays inside the row's 64/128 bytes,
// so global coalescing is unchanged.
//
// Synchronisation is by hand: completion of a stage is awaited with s_waitcnt vmcnt(n), n = loads
// of the younger stages still allowed in flight, followed by a bare s_barrier (a full
// __syncthreads() would make the compiler drain every outstanding load).
#pragma once
#include "wind_mfma.h"

namespace wind {

typedef __attribute__((address_space(1))) const void gmem_cptr;
typedef __attribute__((address_space(3))) void lds_ptr;

template <int BM_, int BN_, int WM_, int WN_, int BK_, int NSTAGE_>
struct DmaCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_, NSTAGE = NSTAGE_;
  static constexpr int ROWB = BK * 2;             // bytes per LDS row
  static constexpr int CPR = ROWB / 16;           // 16-byte chunks per row
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
  static constexpr int NWAVES = WAVES_M * WAVES_N, NT = NWAVES * kWave;
  static constexpr int MI = WM / 32, NI = WN / 32;
  static constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  static constexpr int SMEM_BYTES = NSTAGE * STAGE_BYTES;
  static constexpr int RPI = 64 / CPR;            // rows filled by one wave-wide load
  static constexpr int LOADS_PER_STAGE = (BM + BN) / RPI;
  static constexpr int LPW = LOADS_PER_STAGE / NWAVES;  // loads per wave per stage
  static constexpr int KSTEPS = BK / 16;
  static_assert(BK == 32 || BK == 64, "BK");
  static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
  static_assert(LOADS_PER_STAGE % NWAVES == 0 && BM % RPI == 0, "loader shape");
  static_assert(WN <= 128, "a key carries 7 column bits");
  static_assert(NSTAGE >= 2 && NSTAGE <= 5 && LPW * (NSTAGE - 1) < 64 && KSTEPS % 2 == 0, "ring depth, vmcnt range");
  static_assert(SMEM_BYTES <= 160 * 1024, "LDS");
};

template <int CPR>
__device__ __forceinline__ int lds_swizzle(int row) {
  return CPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// A points at the tile's first row ([>=BM rows, K] bf16 dense), Bw likewise for B (rows ldb apart,
// ldb = K unless given).  K % BK == 0.
// The caller initialises acc (zero, or a bias: the products are accumulated on top of it).
//
// Schedule.  Tile t lives in stage t % NSTAGE.  The operand fragments of K step ks+1 are read from
// LDS into a second register set before the MFMAs of step ks are issued, so a wave does not sit
// on an LDS wait with its MFMA pipe empty.  To carry this across tiles, the barrier that hands
// over tile kt+1 sits before the *last* K step of tile kt, whose fragments are in registers by
// then: the barrier certifies that tile kt+1 has landed (every wave waited for its own loads
// first) and that every wave has completed its LDS reads of tile kt (lgkmcnt(0) first), so the
// stage of tile kt is refilled with tile kt+NSTAGE.  NSTAGE-1 tiles stay in flight.  The refill is
// not issued in one burst: a wave that queues all its loads at once sits at the memory pipeline's
// door while its MFMA pipe runs dry, so a quarter goes out at the hand-over and the rest follows
// with the next three K steps (measured: 19 -> 16 us for a 256 x 128 x 1024 tile).
// Where a lane finds its 16 bytes of an A load: dense rows (the joint kernel) ...
struct DenseRows {
  const bf16_t *base;
  int ld;
  __device__ __forceinline__ const bf16_t *operator()(int, int row, int chunk, int kt, int BK) const {
    return base + (size_t)row * ld + kt * BK + chunk * 8;
  }
};

// asrc(i, row, chunk, kt, BK) returns the global address of the 8 bf16 at K offset kt*BK + chunk*8
// of A's row `row` (i = index of the load among the wave's LPW loads of a stage, for sources that
// cache per-load state); it is called once per load and K step, so gathered rows or rows stitched from two
// arrays cost a few integer operations per load, not a staging pass.
// SWAP = true issues the MFMAs with the operands exchanged: acc[mi][ni] then holds the transposed
// 32 x 32 block (B rows down the registers, A rows across the lanes), which lets an epilogue that
// reduces over B rows work inside a lane.
// `after_issue` runs once the first stages are on their way and before anything is awaited: the
// place for a caller to finish setting up acc from values it loaded earlier, behind the loads' latency,
// or to find out, in the same round trip as the first stages, whether the tile is wanted at all (`drop`).
struct NoInit {
  __device__ __forceinline__ void operator()() const {}
};
template <class Cfg, class ASrc, bool SWAP = false, class Init = NoInit>
__device__ __forceinline__ void gemm_mainloop_dma_src(const ASrc &asrc, const bf16_t *__restrict__ Bw,
                                                      int K, unsigned char *smem,
                                                      f32x16 (&acc)[Cfg::MI][Cfg::NI], Init after_issue = Init{},
                                                      int ldb = 0, const bool *drop = nullptr) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
  if (ldb == 0) ldb = K;   // B rows are K long unless the caller walks a K-slice of longer rows

  // the wave's loads of a stage: rows below BM are A rows, the rest B rows
  int lrow[Cfg::LPW], lchunk[Cfg::LPW];
  const bf16_t *bsrc[Cfg::LPW];
#pragma unroll
  for (int i = 0; i < Cfg::LPW; ++i) {
    const int q = wave * Cfg::LPW + i;
    lrow[i] = q * Cfg::RPI + lane / Cfg::CPR;
    lchunk[i] = (lane % Cfg::CPR) ^ lds_swizzle<Cfg::CPR>(lrow[i]);
    bsrc[i] = Bw + (size_t)(lrow[i] - Cfg::BM) * ldb + lchunk[i] * 8;
  }
  // the wave's loads of tile kt into `stage`: all of them (part < 0), or the part-th of KSTEPS shares
  auto issue = [&](int kt, int stage, int part) {
    unsigned char *dst = smem + stage * Cfg::STAGE_BYTES + wave * Cfg::LPW * 1024;
#pragma unroll
    for (int i = 0; i < Cfg::LPW; ++i) {
      if (part >= 0 && (i * Cfg::KSTEPS) / Cfg::LPW != part) continue;
      const bool is_a = (wave * Cfg::LPW + i) * Cfg::RPI < Cfg::BM;   // wave-uniform
      const bf16_t *p = is_a ? asrc(i, lrow[i], lchunk[i], kt, Cfg::BK) : bsrc[i] + kt * Cfg::BK;
      __builtin_amdgcn_global_load_lds((gmem_cptr *)p, (lds_ptr *)(dst + i * 1024), 16, 0, 0);
    }
  };

  const int KT = K / Cfg::BK;
#pragma unroll
  for (int s = 0; s < Cfg::NSTAGE; ++s) issue(s < KT ? s : KT - 1, s, -1);
  after_issue();
  // `drop` (the same for every thread of the workgroup): after_issue found that the tile is not wanted
  if (drop && *drop) {
    wait_vmcnt<0>();
    return;
  }

  // fragment addressing: lane l reads row l%32 of a 32-row block, k chunk 2*ks + l/32
  const int frow = lane & 31, kc = lane >> 5, sw = lds_swizzle<Cfg::CPR>(frow);
  const int a_row_off = (wm * Cfg::WM + frow) * Cfg::ROWB;
  const int b_row_off = (Cfg::BM + wn * Cfg::WN + frow) * Cfg::ROWB;
  bf16x8 af[2][Cfg::MI], bfr[2][Cfg::NI];
  auto load_frags = [&](int set, const unsigned char *st, int ks) {
    const int chunk_off = ((2 * ks + kc) ^ sw) * 16;
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
      af[set][mi] = *reinterpret_cast<const bf16x8 *>(st + a_row_off + mi * 32 * Cfg::ROWB + chunk_off);
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
      bfr[set][ni] = *reinterpret_cast<const bf16x8 *>(st + b_row_off + ni * 32 * Cfg::ROWB + chunk_off);
  };

  // Steady state is branch-free: past the end of K the refill simply re-fetches the last tile
  // into a stage nobody reads again, so every hand-over sees the same number of loads in flight.
  auto mfma_step = [&](int set) {
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
        acc[mi][ni] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][ni], af[set][mi], acc[mi][ni], 0, 0, 0)
                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][mi], bfr[set][ni], acc[mi][ni], 0, 0, 0);
  };
  wait_vmcnt<(Cfg::NSTAGE - 1) * Cfg::LPW>();                      // tile 0 has landed
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  load_frags(0, smem, 0);
  int stage = 0;
  // The refill in progress.  Before the first hand-over there is none; the youngest stage is
  // fetched again instead (same bytes to the same place), which keeps the loop free of branches
  // and only makes the first wait a little stricter.
  int pend_kt = Cfg::NSTAGE - 1 < KT ? Cfg::NSTAGE - 1 : KT - 1, pend_stage = Cfg::NSTAGE - 1;
  for (int kt = 0; kt + 1 < KT; ++kt) {
    const unsigned char *st = smem + stage * Cfg::STAGE_BYTES;
    const int next = stage + 1 == Cfg::NSTAGE ? 0 : stage + 1;
#pragma unroll
    for (int ks = 0; ks + 1 < Cfg::KSTEPS; ++ks) {
      load_frags((ks + 1) & 1, st, ks + 1);
      issue(pend_kt, pend_stage, ks + 1);
      __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs they overlap with
      mfma_step(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");              // my reads of tile kt are complete
    wait_vmcnt<(Cfg::NSTAGE - 2) * Cfg::LPW>();                    // tile kt+1 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int kn = kt + Cfg::NSTAGE;
    pend_kt = kn < KT ? kn : KT - 1;
    pend_stage = stage;
    issue(pend_kt, pend_stage, 0);
    load_frags(Cfg::KSTEPS & 1, smem + next * Cfg::STAGE_BYTES, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_step((Cfg::KSTEPS - 1) & 1);
    __builtin_amdgcn_sched_barrier(0);
    stage = next;
  }
  {  // last tile
    const unsigned char *st = smem + stage * Cfg::STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < Cfg::KSTEPS; ++ks) {
      if (ks + 1 < Cfg::KSTEPS) load_frags((ks + 1) & 1, st, ks + 1);
      mfma_step(ks & 1);
    }
  }
  wait_vmcnt<0>();   // the redundant refills must not outlive the kernel's use of LDS
}

template <class Cfg, bool SWAP = false, class Init = NoInit>
__device__ __forceinline__ void gemm_mainloop_dma(const bf16_t *__restrict__ A, const bf16_t *__restrict__ Bw,
                                                  int K, unsigned char *smem,
                                                  f32x16 (&acc)[Cfg::MI][Cfg::NI], Init after_issue = Init{}) {
  gemm_mainloop_dma_src<Cfg, DenseRows, SWAP, Init>(DenseRows{A, K}, Bw, K, smem, acc, after_issue);
}

// ---------------------------------------------------------------------------------------------
// The same core for square 256 x 256 (BT x BT) tiles with BK = 64, where two full stages already
// take 128 of the 160 KB of LDS.  The ring is cut into five 32 KB slots, one operand (BT rows x 128
// bytes) each; units are issued in the order A0 B0 A1 B1 A2 B2 ...; unit u lives in slot u % 5.
// When tile kt is handed back, its two slots take B(kt+2) and A(kt+3): every A load has two tile
// times to land, every B load one.  That split fits this workload: the B operand is the slice of
// W_out that the XCD-aware tile mapping keeps in the XCD's L2 (short latency), the A operand is the
// freshly written window rows that come from further away.
template <int BT_, int WM_, int WN_>
struct Ring5Cfg {
  static constexpr int BM = BT_, BN = BT_, WM = WM_, WN = WN_, BK = 64;
  static constexpr int ROWB = 128, CPR = 8, RPI = 8, KSTEPS = 4, NSLOT = 5;
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
  static constexpr int NWAVES = WAVES_M * WAVES_N, NT = NWAVES * kWave;
  static constexpr int MI = WM / 32, NI = WN / 32;
  static constexpr int UNIT_BYTES = BT_ * ROWB;
  static constexpr int SMEM_BYTES = NSLOT * UNIT_BYTES;
  static constexpr int LPU = (BT_ / RPI) / NWAVES;   // loads per wave per unit
  static_assert((BT_ / RPI) % NWAVES == 0 && BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "shape");
  static_assert(WN <= 128 && SMEM_BYTES <= 160 * 1024, "limits");
};

template <class Cfg, bool SWAP = false, class Init = NoInit>
__device__ __forceinline__ void gemm_mainloop_ring5(const bf16_t *__restrict__ A, const bf16_t *__restrict__ Bw,
                                                    int K, unsigned char *smem,
                                                    f32x16 (&acc)[Cfg::MI][Cfg::NI], Init after_issue = Init{}) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
  const bf16_t *src_a[Cfg::LPU], *src_b[Cfg::LPU];
#pragma unroll
  for (int i = 0; i < Cfg::LPU; ++i) {
    const int row = (wave * Cfg::LPU + i) * Cfg::RPI + lane / Cfg::CPR;
    const int c = (lane % Cfg::CPR) ^ lds_swizzle<Cfg::CPR>(row);
    src_a[i] = A + (size_t)row * K + c * 8;
    src_b[i] = Bw + (size_t)row * K + c * 8;
  }
  const int KT = K / Cfg::BK;
  // one load of an A unit / a whole B unit
  auto issue_a1 = [&](int i, int kt, int slot) {
    kt = kt < KT ? kt : KT - 1;
    unsigned char *dst = smem + slot * Cfg::UNIT_BYTES + wave * Cfg::LPU * 1024;
    __builtin_amdgcn_global_load_lds((gmem_cptr *)(src_a[i] + kt * Cfg::BK), (lds_ptr *)(dst + i * 1024), 16, 0, 0);
  };
  auto issue_a = [&](int kt, int slot) {
#pragma unroll
    for (int i = 0; i < Cfg::LPU; ++i) issue_a1(i, kt, slot);
  };
  auto issue_b = [&](int kt, int slot) {
    kt = kt < KT ? kt : KT - 1;
    unsigned char *dst = smem + slot * Cfg::UNIT_BYTES + wave * Cfg::LPU * 1024;
#pragma unroll
    for (int i = 0; i < Cfg::LPU; ++i)
      __builtin_amdgcn_global_load_lds((gmem_cptr *)(src_b[i] + kt * Cfg::BK), (lds_ptr *)(dst + i * 1024), 16, 0, 0);
  };
  // All waves refilling at once right after a barrier would queue 64 KB of loads behind the
  // address unit and hold every wave at issue; so only the B unit and the first load of the A unit
  // go out at the hand-over, the rest of the A unit follows one load per K step.
  issue_a(0, 0); issue_b(0, 1); issue_a(1, 2); issue_b(1, 3); issue_a1(0, 2, 4);
  after_issue();

  const int frow = lane & 31, kc = lane >> 5, sw = lds_swizzle<Cfg::CPR>(frow);
  const int a_row_off = (wm * Cfg::WM + frow) * Cfg::ROWB;
  const int b_row_off = (wn * Cfg::WN + frow) * Cfg::ROWB;
  bf16x8 af[2][Cfg::MI], bfr[2][Cfg::NI];
  auto load_frags = [&](int set, int slot_a, int slot_b, int ks) {
    const int chunk_off = ((2 * ks + kc) ^ sw) * 16;
    const unsigned char *pa = smem + slot_a * Cfg::UNIT_BYTES + a_row_off + chunk_off;
    const unsigned char *pb = smem + slot_b * Cfg::UNIT_BYTES + b_row_off + chunk_off;
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
  auto plus2 = [](int s) { return s + 2 >= Cfg::NSLOT ? s + 2 - Cfg::NSLOT : s + 2; };
  static_assert(Cfg::LPU == Cfg::KSTEPS, "one A load per K step");
  wait_vmcnt<2 * Cfg::LPU + 1>();   // A0, B0 have landed
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  load_frags(0, 0, 1, 0);
  int sa = 0, sb = 1;
  for (int kt = 0; kt + 1 < KT; ++kt) {
    const int sprev = sa == 0 ? Cfg::NSLOT - 1 : sa - 1;   // slot of B(kt-1), now taking A(kt+2)
#pragma unroll
    for (int ks = 0; ks + 1 < Cfg::KSTEPS; ++ks) {
      load_frags((ks + 1) & 1, sa, sb, ks + 1);
      issue_a1(ks + 1, kt + 2, sprev);
      __builtin_amdgcn_sched_barrier(0);
      mfma_step(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // my reads of tile kt are complete
    wait_vmcnt<Cfg::LPU>();                               // A(kt+1), B(kt+1) have landed; A(kt+2) may fly
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue_b(kt + 2, sa);
    issue_a1(0, kt + 3, sb);
    const int na = plus2(sa), nb = plus2(sb);
    load_frags(0, na, nb, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_step(1);
    __builtin_amdgcn_sched_barrier(0);
    sa = na;
    sb = nb;
  }
#pragma unroll
  for (int ks = 0; ks < Cfg::KSTEPS; ++ks) {   // last tile
    if (ks + 1 < Cfg::KSTEPS) load_frags((ks + 1) & 1, sa, sb, ks + 1);
    mfma_step(ks & 1);
  }
  wait_vmcnt<0>();   // the redundant refills must not outlive the kernel's use of LDS
}

}  // namespace wind
