// bf16 MFMA tile core for wide tiles: C[64 MI, 256] += A[64 MI, K] * B[256, K]^T, one wave per SIMD.
//
// Why another core.  A CU takes operands in through one 64 B/clk vector-memory path and multiplies
// 4096 flops/clk, so a tile of m x n outputs keeps the path busy mn / (64 (m + n)) of the time the
// MFMAs need: 75 % for 256 x 128, 50 % for 256 x 256, and the chip's L2s deliver about 21 TB/s to
// all CUs together, which 256 x 128 tiles of a 2048 x 8192 x 1024 product need for 18 of the 20 us
// the MFMAs take.  The 256-column tile needs a third less.  Its accumulators are 256 registers per
// lane (MI = 4), which leaves no room for a second wave on the SIMD: the workgroup is four waves of
// up to 512 registers, each multiplying a (32 MI) x 128 block AND fetching its share of the operands.
//
// Operands sit in memory in slabs of 32 K values: X[k / 32][row][k % 32] (a row of a slab is 64
// contiguous bytes, consecutive rows follow each other), so that a K stage of 32 is a dense range
// of memory and one wave-wide direct-to-LDS load (1 KB) covers 16 whole rows = 8 whole cache lines.
// With 32 KB per stage the 160 KB of LDS hold a ring of five stages, four of them in flight beyond
// the one being multiplied: twice the look-ahead, in time, of 64-wide K tiles.
//
// LDS: B ring (5 x 256 rows x 64 B), then A ring (5 x 256 rows x 64 B, of which 64 MI are used).
// The B ring's first stages are requested before the number of rows is known.  (Requesting the A
// rows as well at that point, for the tallest tile, was tried: no gain, the first stage's arrival is
// not what the row count waits for.)  The 16-byte chunk c of row r is stored at chunk position c ^ ((r >> 2) & 3): the
// fragment reads of 16 consecutive rows then fall on 16 distinct 16-byte slots modulo 256 bytes.
//
// Rows of a tile: the tile `mt` of `tiles` owns the 32-row blocks mt + tiles * q, q = 0 .. 2 MI - 1
// (block q sits at rows 32 q of the LDS stage); wave (wm, wn) multiplies blocks q = 2 mi + wm with
// columns 128 wn .. 128 wn + 127.
// Loads: a group of 16 rows per wave-wide load; wave w fetches A groups 4 i + w (i < MI) and B groups
// 4 w + i (i < 4) of every stage.  The loads are buffer loads: descriptor and slab offset in scalar
// registers, lane offsets that never change, so a refill costs the wave two instructions (measured
// against global loads with per-lane 64-bit addresses: 9 instead of 21 idle MFMA cycles per load).
//
// Schedule of a wave, per stage j (two K steps of 16): the MFMAs of the first step run with the
// fragment reads of the second woven in one behind each MFMA; then the wave waits for its own loads
// of stage j + 1 and for its own LDS reads, and meets the others at ONE workgroup barrier; the MFMAs
// of the second step follow with the reads of stage j + 1's first step woven in.  The refill of the
// ring (A of tile j + 4, B of tile j + 5) is spread over both steps, one load every few MFMAs.
// A wave issues one instruction every four cycles at best and an MFMA occupies its pipe for 32:
// whatever stands between two MFMAs beyond seven instructions shows as an idle MFMA pipe, there
// being no second wave on the SIMD to fill it, so the steady state is straight-line code (the
// ring's start-up and tail are separate copies of the stage with their own wait counts).
#pragma once
#include <type_traits>
#include "wind_mfma_dma.h"

namespace wind {

typedef __attribute__((ext_vector_type(4))) int i32x4;

template <int MI_>
struct WideCfg {
  static constexpr int MI = MI_, NI = 4;
  static constexpr int BM = 64 * MI_, BN = 256, BK = 32, ROWB = 64;
  static constexpr int WM = 32 * MI_, WN = 128, WAVES_M = 2, WAVES_N = 2, NWAVES = 4, NT = 256;
  static constexpr int LB = 4, LA = MI_;             // loads per wave and stage
  static constexpr int LPW = LA + LB;
  static_assert(4 * LPW < 64, "vmcnt range");
};
constexpr int kWideStages = 5, kWideStage = 256 * 64;
constexpr int kWideABase = kWideStages * kWideStage;
constexpr int kWideSmemBytes = 2 * kWideStages * kWideStage;
constexpr int kWideMinK = 320;     // ten stages: the ring's start-up and its tail do not overlap
static_assert(kWideSmemBytes <= 160 * 1024, "LDS");

// Buffer descriptor of a dense byte range (raw buffer, offsets beyond `bytes` read as zero).
__device__ __forceinline__ i32x4 wide_rsrc(const void *base, uint32_t bytes) {
  const uint64_t a = (uint64_t)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xFFFFu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}
// 16 bytes per lane from rsrc[soff + voff] to LDS: lane l's bytes land at dst + 16 l.  The compiler has no
// builtin for the 16-byte form, hence the assembly; it writes M0 (the LDS address), which the compiler sets
// itself before each of its own uses, and its completion is counted in vmcnt like any load's, which the
// code that calls this waits for by hand (the compiler's own counts do not know of these loads: any wait it
// inserts for a load of its own is then only stricter than needed, loads returning in order).
__device__ __forceinline__ void wide_load(i32x4 rsrc, unsigned char *dst, uint32_t voff, uint32_t soff) {
  const uint32_t m = (uint32_t)(uintptr_t)(lds_ptr *)dst;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(m), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
// lane offsets within a slab: B group gb of the column tile at row n0; A group g of tile mt
__device__ __forceinline__ uint32_t wide_boff(int n0, int gb) {
  const int lane = threadIdx.x & 63, brow = 16 * gb + (lane >> 2);
  return (uint32_t)((n0 + brow) * 64 + (((lane & 3) ^ ((brow >> 2) & 3)) * 16));
}
// (row0: where the tiles' row numbering starts in A; with tiles = 1 and mt = 0 a tile is the 64 MI rows from row0 on)
__device__ __forceinline__ uint32_t wide_aoff(int mt, int tiles, int g, int a_rows, int row0 = 0) {
  const int lane = threadIdx.x & 63, trow = 16 * g + (lane >> 2);
  int grow = row0 + (mt + tiles * (trow >> 5)) * 32 + (trow & 31);
  grow = grow < a_rows ? grow : a_rows - 1;   // blocks past the end of A: any row, its keys are not stored
  return (uint32_t)(grow * 64 + (((lane & 3) ^ ((trow >> 2) & 3)) * 16));
}

// B loads of the ring's five stages.  Needs nothing but the column tile.
__device__ __forceinline__ void wide_head_b(i32x4 rs_b, uint32_t slab_b, int n0, int KS, unsigned char *smem) {
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
#pragma unroll
  for (int s = 0; s < kWideStages; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i)
      wide_load(rs_b, smem + s * kWideStage + (wave * 4 + i) * 1024, wide_boff(n0, wave * 4 + i), (uint32_t)(s < KS ? s : KS - 1) * slab_b);
}
// The wave's first NA A loads of every stage, for the ring's five stages.
template <int NA>
__device__ __forceinline__ void wide_head_a(i32x4 rs_a, uint32_t slab_a, int mt, int tiles, int a_rows, int KS, unsigned char *smem,
                                            int row0 = 0) {
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
#pragma unroll
  for (int s = 0; s < kWideStages; ++s)
#pragma unroll
    for (int i = 0; i < NA; ++i)
      wide_load(rs_a, smem + kWideABase + s * kWideStage + (4 * i + wave) * 1024, wide_aoff(mt, tiles, 4 * i + wave, a_rows, row0),
                (uint32_t)(s < KS ? s : KS - 1) * slab_a);
}
// The K loop up to, but not including, the last K step, whose operand fragments are left in af[1],
// bfr[1] (wide_last_step).  rs_a / rs_b: descriptors of the slab layouts of A and B.  The B loads of
// stages 0..4 are on their way (wide_head_b); the A loads follow here.  K = 32 KS, KS >= 10.  acc is set
// by `after_issue`, which runs behind the first loads.  The transposed block is accumulated (MFMA operands
// exchanged): acc[mi][ni] holds B rows down the registers and A rows across the lanes, so that an epilogue
// which reduces over B rows works inside a lane.
template <class Cfg, class Init>
__device__ __forceinline__ void wide_mainloop(i32x4 rs_a, uint32_t slab_a, i32x4 rs_b, uint32_t slab_b, int KS, int mt, int tiles,
                                              int n0, int a_rows, unsigned char *smem,
                                              f32x16 (&acc)[Cfg::MI][Cfg::NI], bf16x8 (&af)[2][Cfg::MI], bf16x8 (&bfr)[2][Cfg::NI],
                                              Init after_issue, int row0 = 0) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int wm = wave >> 1, wn = wave & 1;
  wide_head_a<Cfg::LA>(rs_a, slab_a, mt, tiles, a_rows, KS, smem, row0);
  uint32_t aoff[Cfg::LA], boff[Cfg::LB];
#pragma unroll
  for (int i = 0; i < Cfg::LA; ++i) aoff[i] = wide_aoff(mt, tiles, 4 * i + wave, a_rows, row0);
#pragma unroll
  for (int i = 0; i < Cfg::LB; ++i) boff[i] = wide_boff(n0, wave * 4 + i);
  unsigned char *const lds_a = smem + kWideABase + wave * 1024, *const lds_b = smem + wave * 4 * 1024;
  uint32_t so_a = 5 * slab_a, so_b = 5 * slab_b;   // slab offsets of the next tiles to fetch
  auto issue_a1 = [&](int i, int stage_off) {
    wide_load(rs_a, lds_a + stage_off + i * 4096, aoff[i], so_a);
    if (i == Cfg::LA - 1) so_a += slab_a;
  };
  auto issue_b1 = [&](int i, int stage_off) {
    wide_load(rs_b, lds_b + stage_off + i * 1024, boff[i], so_b);
    if (i == Cfg::LB - 1) so_b += slab_b;
  };
  after_issue();

  // fragment addressing: lane l reads row l % 32 of a 32-row block, chunk 2 ks + l / 32 of the stage
  // (K step 1 is K step 0's address with bit 5 flipped)
  const int frow = lane & 31, kc = lane >> 5;
  const int c0 = (kc ^ ((frow >> 2) & 3)) * 16;
  const unsigned char *rd_a[2], *rd_b[2];   // block q = 2 mi + wm: + mi * 4096; column block ni: + ni * 2048
  rd_a[0] = smem + kWideABase + wm * 2048 + frow * 64 + c0;
  rd_b[0] = smem + wn * (128 * 64) + frow * 64 + c0;
  rd_a[1] = smem + kWideABase + wm * 2048 + frow * 64 + (c0 ^ 32);
  rd_b[1] = smem + wn * (128 * 64) + frow * 64 + (c0 ^ 32);
  // the q-th fragment read of K step ks of the stage at `off` into register set `set`, in the order the MFMAs want them
  auto read_frag = [&](int q, int set, int off, int ks) {
    if (q == 0) af[set][0] = *reinterpret_cast<const bf16x8 *>(rd_a[ks] + off);
    else if (q <= Cfg::NI) bfr[set][q - 1] = *reinterpret_cast<const bf16x8 *>(rd_b[ks] + off + (q - 1) * 2048);
    else af[set][q - Cfg::NI] = *reinterpret_cast<const bf16x8 *>(rd_a[ks] + off + (q - Cfg::NI) * 4096);
  };
  constexpr int NREAD = Cfg::MI + Cfg::NI, NMFMA = Cfg::MI * Cfg::NI;
  // One K step: the MFMAs on register set `set`; behind the first of them the NREAD fragment reads of
  // K step rks of the stage at `off` into the other set; `load(x)` issues what goes behind MFMA x.
  auto kstep = [&](int set, int off, int rks, auto &&load) {
    constexpr int PER = (NREAD + NMFMA - 1) / NMFMA;   // reads behind one MFMA (1, or 2 when MI = 1)
#pragma unroll
    for (int x = 0; x < NMFMA; ++x) {
      const int mi = x / Cfg::NI, ni = x % Cfg::NI;
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][ni], af[set][mi], acc[mi][ni], 0, 0, 0);
#pragma unroll
      for (int y = 0; y < PER; ++y)
        if (x * PER + y < NREAD) read_frag(x * PER + y, set ^ 1, off, rks);
      load(x);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto no_load = [](int) {};

  // the head's loads that follow those of a stage (B first, then A): the later stages' A loads
  constexpr int H = Cfg::LA;
  wait_vmcnt<4 * H>();   // stage 0 has landed
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int q = 0; q < NREAD; ++q) read_frag(q, 0, 0, 0);
  // Byte offsets of the stages within their rings: cur = the stage being multiplied, prv = the one before.
  int cur = 0, prv = 4 * kWideStage;
  // Stage j.  WAITN: loads that may still be in flight once tile j + 1 has landed; RA: A of tile j + 4 goes
  // into the stage tile j - 1 left; RB: B of tile j + 5 goes into stage j.
  auto body = [&](auto WAITN, auto RA, auto RB) {
    const int nxt = cur == 4 * kWideStage ? 0 : cur + kWideStage;
    kstep(0, cur, 1, [&](int x) {
      if constexpr (decltype(RA)::value) {
        if (x % Cfg::NI == Cfg::NI - 1) issue_a1(x / Cfg::NI, prv);   // one load every NI MFMAs
      }
    });
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // my reads of stage j are complete
    wait_vmcnt<decltype(WAITN)::value>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    kstep(1, nxt, 0, [&](int x) {
      if constexpr (decltype(RB)::value) {
        if (x % Cfg::MI == Cfg::MI - 1) issue_b1(x / Cfg::MI, cur);   // one load every MI MFMAs
      }
    });
    prv = cur; cur = nxt;
  };
  using std::integral_constant;
  using T = integral_constant<bool, true>;
  using F = integral_constant<bool, false>;
  // start-up: behind the last head load of tile j + 1 sit the head's loads of later tiles and the refills so far
  body(integral_constant<int, 3 * H>{}, F{}, T{});
  body(integral_constant<int, 2 * H + Cfg::LPW>{}, T{}, T{});
  body(integral_constant<int, H + 2 * Cfg::LPW>{}, T{}, T{});
  for (int j = 3; j + 5 < KS; ++j) body(integral_constant<int, 3 * Cfg::LPW>{}, T{}, T{});
  body(integral_constant<int, 3 * Cfg::LPW>{}, T{}, F{});   // j = KS - 5: the last refill
  body(integral_constant<int, 2 * Cfg::LPW>{}, F{}, F{});
  body(integral_constant<int, Cfg::LPW>{}, F{}, F{});
  body(integral_constant<int, 0>{}, F{}, F{});             // j = KS - 2
  kstep(0, cur, 1, no_load);                               // last stage, first K step
}

// The last K step.  Every accumulator's final MFMA writes a fresh value that the VALU can read, and
// fin(mi, p, lo, hi) gets the finished transposed blocks of columns 64 p .. 64 p + 31 and 64 p + 32 ..
// 64 p + 63 (p = 0, 1 within the wave's 128 columns) of row block mi while the next pair's MFMAs run.
template <class Cfg, class Fin>
__device__ __forceinline__ void wide_last_step(f32x16 (&acc)[Cfg::MI][Cfg::NI], const bf16x8 (&af)[Cfg::MI],
                                               const bf16x8 (&bfr)[Cfg::NI], Fin fin) {
  f32x16 r[2][2];
  auto last = [&](int k) {
    const int mi = k >> 1, p = k & 1;
    r[k & 1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[2 * p], af[mi], acc[mi][2 * p], 0, 0, 0);
    r[k & 1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[2 * p + 1], af[mi], acc[mi][2 * p + 1], 0, 0, 0);
  };
  last(0);
#pragma unroll
  for (int k = 0; k < 2 * Cfg::MI; ++k) {
    if (k + 1 < 2 * Cfg::MI) last(k + 1);
    __builtin_amdgcn_sched_barrier(0);
    fin(k >> 1, k & 1, r[k & 1][0], r[k & 1][1]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace wind
