// The joint kernel (output contraction with the row argmax in its epilogue), the same tile core with
// logits stored (debug, beam search), and the fp32 joiner of fp32 models.
#pragma once
#include "wind_types.h"

namespace wind {

// ---------------------------------------------------------------------------------------------
// Which (row tile, column tile) of an MT x NT tile grid the workgroup with linear id `lin` owns (lin
// must be congruent to the workgroup's launch id modulo 8).  Workgroups are handed to the 8 XCDs
// round-robin by launch id, and each XCD has its own 4 MB L2.  Column tiles are therefore
// dealt by (linear id mod 8): an XCD always works on the same slice of W_out, which then stays in
// its L2 across row tiles and across loop iterations, and only the window rows stream in.
__device__ __forceinline__ void joint_tile_of_block(int lin, int MT, int NT, int &mt, int &nt) {
  if (NT % 8 != 0) { mt = lin % MT; nt = lin / MT; return; }
  const int xcd = lin & 7, idx = lin >> 3, npx = NT >> 3;
  nt = xcd + 8 * (idx % npx);
  mt = idx / npx;
}

// The joint kernels accumulate the transposed tile (MFMA operands exchanged): a lane then holds ONE
// window row (lane % 32 of the 32-row block mi) and, per 32-column block ni, the 16 columns
// 8 * (r / 4) + 4 * (lane / 32) + r % 4.  The row argmax over the wave's WN columns is therefore a
// running top-2 inside the lane, plus one exchange between the two lanes that share a row.
//
// Accumulator start value: the output bias of each register's column, or a large negative number
// for columns past the vocabulary, so that the epilogue needs neither an add nor a mask.  The bias
// is requested before the tile core starts its loads and copied into the accumulators behind them.
template <class Cfg>
__device__ __forceinline__ void joint_load_bias(const ModelDev &m, float (&bias)[Cfg::NI][16], int n0) {
  const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) % Cfg::WAVES_N;
#pragma unroll
  for (int ni = 0; ni < Cfg::NI; ++ni) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int col = n0 + wn * Cfg::WN + ni * 32 + 8 * g + 4 * (lane >> 5);
      if (col + 3 < m.V) {
        const float4 b4 = *reinterpret_cast<const float4 *>(m.b_out + col);
        bias[ni][4 * g] = b4.x; bias[ni][4 * g + 1] = b4.y; bias[ni][4 * g + 2] = b4.z; bias[ni][4 * g + 3] = b4.w;
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) bias[ni][4 * g + q] = col + q < m.V ? m.b_out[col + q < m.V ? col + q : 0] : kKeyNone;
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the tile core's
}
template <class Cfg>
struct JointInitAcc {
  f32x16 (&acc)[Cfg::MI][Cfg::NI];
  const float (&bias)[Cfg::NI][16];
  __device__ __forceinline__ void operator()() const {
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][ni][r] = bias[ni][r];
  }
};

// The keys of entry idx of a key array with KW words per entry (2: two keys; 4: three keys and a pad).
template <int KW>
__device__ __forceinline__ float4 load_keys(const float *parts, size_t idx) {
  if constexpr (KW == 4) {
    return reinterpret_cast<const float4 *>(parts)[idx];
  } else {
    const float2 k = reinterpret_cast<const float2 *>(parts)[idx];
    return make_float4(k.x, k.y, kKeyNone, kKeyNone);
  }
}
__device__ __forceinline__ float4 no_keys() { return make_float4(kKeyNone, kKeyNone, kKeyNone, kKeyNone); }

// The column codes of a lower-half lane's 32 values of one 64-column part (two accumulator blocks), held in
// registers: as literals they cost a second instruction per key.  inf: key_inf().
struct KeyConsts {
  uint32_t code[32];
  float inf;
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      code[r] = kKeyColMask - (uint32_t)((r >> 4) * 32 + 8 * ((r & 15) >> 2) + (r & 3));
      asm volatile("" : "+v"(code[r]));
    }
    inf = key_inf();
  }
};

// Epilogue of the joint kernel: (logit, column) keys, per-row top-3 over the wave's WN columns,
// one float4 per (row, part) to memory.  The logits never leave registers.
template <class Cfg>
__device__ __forceinline__ void joint_keys_epilogue(const CallDev &c, f32x16 (&acc)[Cfg::MI][Cfg::NI],
                                                    int row0, int nt, int stride) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
  const int part = nt * Cfg::WAVES_N + wn, row_base = row0 + wm * Cfg::WM;
  // Keys are built with the column codes of the lower lane half; the upper half's columns are 4
  // higher, i.e. code bit 2 cleared (it is always set in the lower half's codes).  All keys of a
  // lane shift alike, so the correction waits until the lane's three winners are known.
  const unsigned fix = ~(unsigned)(4 * (lane >> 5));
  static_assert(Cfg::NI == 2, "one 64-column part per wave");
  KeyConsts kc;
  kc.init();
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi) {
    float k1 = kKeyNone, k2 = kKeyNone, k3 = kKeyNone;
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        push_top3(k1, k2, k3, __uint_as_float((__float_as_uint(acc[mi][ni][r]) & ~kKeyColMask) | kc.code[16 * ni + r]), kc.inf);
    k1 = __uint_as_float(__float_as_uint(k1) & fix);
    k2 = __uint_as_float(__float_as_uint(k2) & fix);
    k3 = __uint_as_float(__float_as_uint(k3) & fix);
    const float r1 = __shfl_xor(k1, 32, kWave), r2 = __shfl_xor(k2, 32, kWave), r3 = __shfl_xor(k3, 32, kWave);
    push_top3(k1, k2, k3, r1);
    push_top3(k1, k2, k3, r2);
    push_top3(k1, k2, k3, r3);
    if (lane < 32)
      reinterpret_cast<float4 *>(c.parts)[(size_t)(row_base + mi * 32 + lane) * stride + part] = make_float4(k1, k2, k3, kKeyNone);
  }
}

// ---------------------------------------------------------------------------------------------
// The joint kernel on the tile core whose waves are split into multipliers and fetchers
// (wind_mfma_ws.h).  The launch has `fill` x NT workgroups, fill = row tiles that fill the chip for
// NT column tiles.  Workgroup `lin` owns column tile nt(lin) whatever the row count, so a fetcher
// requests the first stages of its W_out slice before it knows how many window rows the iteration
// has; the row count then fixes the row tiles and their height:
//   R <= 64 fill:  ceil(R / 64) row tiles of 64 rows (workgroups beyond them leave)
//   else:          rounds = ceil(R / (256 fill)) row tiles per workgroup (mt, mt + fill, ...), each
//                  64 MI rows high, MI = ceil(R / (64 fill rounds)) in 1..4
// so every workgroup has the same work at any row count.  Between two tiles of a workgroup one
// more barrier hands the LDS back to the fetchers, who request the next tile's first stages while
// the multipliers reduce the finished tile to keys.
template <int MI>
__device__ __forceinline__ void joint_ws_tiles(const ModelDev &m, const CallDev &c, int n_rows, int mt0, int mt_step,
                                               int mt_end, int nt, bool head_done, unsigned char *smem_raw) {
  using Cfg = WsCfg<MI>;
  const int n0 = nt * Cfg::BN, Hj = m.Hj;
  const bf16_t *bw = reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)n0 * Hj;
  if (threadIdx.x >= Cfg::NMUL * kWave) {
    for (int mt = mt0; mt < mt_end && mt * Cfg::BM < n_rows; mt += mt_step) {
      if (mt != mt0) __builtin_amdgcn_s_barrier();   // the multipliers are done with the LDS
      if (mt != mt0 || !head_done) ws_fetch_b_head(bw, Hj, smem_raw);
      ws_fetch<Cfg>(c.z + (size_t)mt * Cfg::BM * Hj, bw, Hj, smem_raw);
    }
    wait_vmcnt<0>();
    return;
  }
  f32x16 acc[Cfg::MI][Cfg::NI];
  float bias[Cfg::NI][16];
  joint_load_bias<Cfg>(m, bias, n0);
  for (int mt = mt0; mt < mt_end && mt * Cfg::BM < n_rows; mt += mt_step) {
    JointInitAcc<Cfg>{acc, bias}();
    ws_multiply<Cfg, true>(Hj, smem_raw, acc);
    const int mn = mt + mt_step;
    if (mn < mt_end && mn * Cfg::BM < n_rows) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
    }
    joint_keys_epilogue<Cfg>(c, acc, mt * Cfg::BM, nt, c.nparts);
  }
}

__global__ __launch_bounds__(512) void joint_ws_kernel(ModelDev m, CallDev c, int parity, int fill, int NT) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int lin = (int)blockIdx.x;
  const bool fetcher = threadIdx.x >= 4 * kWave;
  const bool early = NT % 8 == 0;   // the column tile does not depend on the number of row tiles
  int mt = 0, nt = 0;
  if (early) {
    joint_tile_of_block(lin, fill, NT, mt, nt);
    if (fetcher) ws_fetch_b_head(reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)nt * 128 * m.Hj, m.Hj, smem_raw);
  }
  const int n_rows = c.n_active[parity] * c.W;
  const int fine = (n_rows + 63) / 64;
  int tiles, mi;   // row tiles in use, their height in units of 64 rows
  if (fine <= fill) {
    tiles = fine; mi = 1;
  } else {
    const int rounds = (n_rows + 256 * fill - 1) / (256 * fill);
    tiles = fill * rounds;
    mi = (n_rows + 64 * tiles - 1) / (64 * tiles);
  }
  const int mt_step = tiles < fill ? tiles : fill;
  if (!early && mt_step > 0) joint_tile_of_block(lin, mt_step, NT, mt, nt);
  if (n_rows == 0 || mt >= mt_step || nt >= NT) {
    if (fetcher) wait_vmcnt<0>();
    return;
  }
  switch (mi) {
    case 1: joint_ws_tiles<1>(m, c, n_rows, mt, mt_step, tiles, nt, early, smem_raw); break;
    case 2: joint_ws_tiles<2>(m, c, n_rows, mt, mt_step, tiles, nt, early, smem_raw); break;
    case 3: joint_ws_tiles<3>(m, c, n_rows, mt, mt_step, tiles, nt, early, smem_raw); break;
    default: joint_ws_tiles<4>(m, c, n_rows, mt, mt_step, tiles, nt, early, smem_raw); break;
  }
}

// ---------------------------------------------------------------------------------------------
// The joint kernel on 256-column tiles (wind_mfma_wide.h), for iterations with many window rows:
// W_out and the window rows are read in their slab layouts (ModelDev::w_out_slab; CallDev::z as
// the gather kernel writes it in slab mode).  The launch has `fill` x NT workgroups of four waves,
// fill = row tiles that fill the chip for NT column tiles of 256; tile heights and rounds follow the
// row count as in joint_ws_kernel, and the result (keys per row and 64-column part) is the same,
// bit for bit: every logit is the same chain of MFMAs over K in the same order.
// Keys of one row block and one 64-column part from its two finished accumulator blocks (lo: columns 0..31 of
// the part, hi: 32..63), see joint_keys_epilogue.
__device__ __forceinline__ void joint_wide_keys(const CallDev &c, const KeyConsts &kc, const f32x16 &lo, const f32x16 &hi,
                                                int row, int part) {
  const int lane = threadIdx.x & 63;
  const unsigned fix = ~(unsigned)(4 * (lane >> 5));
  float k1 = kKeyNone, k2 = kKeyNone, k3 = kKeyNone;
#pragma unroll
  for (int r = 0; r < 16; ++r) push_top3(k1, k2, k3, __uint_as_float((__float_as_uint(lo[r]) & ~kKeyColMask) | kc.code[r]), kc.inf);
#pragma unroll
  for (int r = 0; r < 16; ++r) push_top3(k1, k2, k3, __uint_as_float((__float_as_uint(hi[r]) & ~kKeyColMask) | kc.code[16 + r]), kc.inf);
  k1 = __uint_as_float(__float_as_uint(k1) & fix);
  k2 = __uint_as_float(__float_as_uint(k2) & fix);
  k3 = __uint_as_float(__float_as_uint(k3) & fix);
  const float r1 = __shfl_xor(k1, 32, kWave), r2 = __shfl_xor(k2, 32, kWave), r3 = __shfl_xor(k3, 32, kWave);
  push_top3(k1, k2, k3, r1);
  push_top3(k1, k2, k3, r2);
  push_top3(k1, k2, k3, r3);
  if (lane < 32 && row < c.Mpad && part < c.nparts)   // 256-column tiles may reach past the last 128-column tile's parts
    reinterpret_cast<float4 *>(c.parts)[(size_t)row * c.nparts + part] = make_float4(k1, k2, k3, kKeyNone);
}

template <int MI>
__device__ __forceinline__ void joint_wide_tiles(const ModelDev &m, const CallDev &c, i32x4 rs_a, i32x4 rs_b, int mt0, int mt_step,
                                                 int tiles, int nt, bool b_head_done, unsigned char *smem_raw) {
  using Cfg = WideCfg<MI>;
  const int n0 = nt * Cfg::BN, KS = m.Hj / 32;
  const uint32_t slab_b = (uint32_t)m.Vpad * 64u, slab_a = (uint32_t)c.Mpad * 64u;
  const int wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1, lane = threadIdx.x & 63;
  f32x16 acc[Cfg::MI][Cfg::NI];
  bf16x8 af[2][Cfg::MI], bfr[2][Cfg::NI];
  float bias[Cfg::NI][16];
  joint_load_bias<Cfg>(m, bias, n0);
  for (int mt = mt0; mt < tiles; mt += mt_step) {
    if (!b_head_done) wide_head_b(rs_b, slab_b, n0, KS, smem_raw);
    wide_mainloop<Cfg>(rs_a, slab_a, rs_b, slab_b, KS, mt, tiles, n0, c.Mpad, smem_raw, acc, af, bfr, JointInitAcc<Cfg>{acc, bias});
    b_head_done = false;
    if (mt + mt_step < tiles) {   // the next tile's first loads go out before this tile's keys are formed
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      wide_head_b(rs_b, slab_b, n0, KS, smem_raw);
      b_head_done = true;
    }
    KeyConsts kc;
    kc.init();
    wide_last_step<Cfg>(acc, af[1], bfr[1], [&](int mi, int p, const f32x16 &lo, const f32x16 &hi) {
      joint_wide_keys(c, kc, lo, hi, (mt + tiles * (2 * mi + wm)) * 32 + (lane & 31), nt * 4 + wn * 2 + p);
    });
  }
}

__global__ __launch_bounds__(256) void joint_wide_kernel(ModelDev m, CallDev c, int parity, int fill, int NT) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int lin = (int)blockIdx.x, KS = m.Hj / 32;
  const bool early = NT % 8 == 0;   // the column tile does not depend on the number of row tiles
  const uint32_t slab_b = (uint32_t)m.Vpad * 64u, slab_a = (uint32_t)c.Mpad * 64u;
  const i32x4 rs_b = wide_rsrc(m.w_out_slab, slab_b * (uint32_t)KS), rs_a = wide_rsrc(c.z, slab_a * (uint32_t)KS);
  int mt = 0, nt = 0;
  if (early) {
    joint_tile_of_block(lin, fill, NT, mt, nt);
    wide_head_b(rs_b, slab_b, nt * 256, KS, smem_raw);
  }
  const int n_rows = c.n_active[parity] * c.W;
  const int fine = (n_rows + 63) / 64;
  int tiles, mi;   // row tiles in use, their height in units of 64 rows
  if (fine <= fill) {
    tiles = fine; mi = 1;
  } else {
    const int rounds = (n_rows + 256 * fill - 1) / (256 * fill);
    tiles = fill * rounds;
    mi = (n_rows + 64 * tiles - 1) / (64 * tiles);
  }
  const int mt_step = tiles < fill ? tiles : fill;
  if (!early && mt_step > 0) joint_tile_of_block(lin, mt_step, NT, mt, nt);
  if (n_rows == 0 || mt >= mt_step || nt >= NT) {
    wait_vmcnt<0>();
    return;
  }
  switch (mi) {
    case 1: joint_wide_tiles<1>(m, c, rs_a, rs_b, mt, mt_step, tiles, nt, early, smem_raw); break;
    case 2: joint_wide_tiles<2>(m, c, rs_a, rs_b, mt, mt_step, tiles, nt, early, smem_raw); break;
    case 3: joint_wide_tiles<3>(m, c, rs_a, rs_b, mt, mt_step, tiles, nt, early, smem_raw); break;
    default: joint_wide_tiles<4>(m, c, rs_a, rs_b, mt, mt_step, tiles, nt, early, smem_raw); break;
  }
}

// The same tile core with the logits stored, bias added (columns 0..V, blank included): the debug entry
// point and beam search.  With z_lo, every row is the sum of two bf16 vectors, z + z_lo (the fp32 hidden
// vector split into a rounded value and the rounded remainder, about 16 mantissa bits together), and the
// products with both are accumulated: logits at close to fp32 accuracy at MFMA speed.
template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) void joint_mfma_store_kernel(ModelDev m, const bf16_t *z, const bf16_t *z_lo,
                                                                  int n_rows, float *logits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);
  const int row0 = blockIdx.x * Cfg::BM, n0 = blockIdx.y * Cfg::BN, Hj = m.Hj;
  const bf16_t *w = reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)n0 * Hj;
  f32x16 acc[Cfg::MI][Cfg::NI];
  {
    const bf16_t *zt = z + (size_t)row0 * Hj;
    auto aload = [&](int, int row, int k) -> u32x4 { return *reinterpret_cast<const u32x4 *>(zt + (size_t)row * Hj + k); };
    gemm_mainloop<Cfg>(aload, w, Hj, smem, acc);
  }
  if (z_lo) {
    f32x16 acc_lo[Cfg::MI][Cfg::NI];
    const bf16_t *zt = z_lo + (size_t)row0 * Hj;
    auto aload = [&](int, int row, int k) -> u32x4 { return *reinterpret_cast<const u32x4 *>(zt + (size_t)row * Hj + k); };
    __syncthreads();   // the first pass may still be reading its last stage
    gemm_mainloop<Cfg>(aload, w, Hj, smem, acc_lo);
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][ni][r] += acc_lo[mi][ni][r];
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
  for (int ni = 0; ni < Cfg::NI; ++ni) {
    const int col = n0 + wn * Cfg::WN + ni * 32 + (lane & 31);
    if (col > m.V) continue;
    const float bias = m.b_out[col];
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row0 + wm * Cfg::WM + acc_row(mi, r, lane);
        if (row < n_rows) logits[(size_t)row * (m.V + 1) + col] = acc[mi][ni][r] + bias;
      }
  }
}

// ---------------------------------------------------------------------------------------------
// Joiner rows in fp32 FMA with the argmax taken directly (ties to the lowest id).  One workgroup
// per window row.  Used by fp32 models in the loop, and by the debug entry point for any model.
//   rows_from_state = 1: row r = (active utterance r / W, window offset r % W)
//   rows_from_state = 0: row r = frame t0 + r of utterance b0 (debug), p taken from p_dbg
template <class WT>
__global__ __launch_bounds__(256) void joint_exact_kernel(ModelDev m, CallDev c, int parity, int rows_from_state,
                                                          int b0, int t0, int n_dbg, const float *p_dbg,
                                                          int round_z, float *logits_out, bf16_t *z_out) {
  extern __shared__ float zs[];
  __shared__ float s_val[4];
  __shared__ int s_idx[4];
  const int row = blockIdx.x;
  int b, tt;
  bool valid;
  const float *pr;
  if (rows_from_state) {
    const int a = row / c.W, j = row - a * c.W;
    const int na = c.n_active[parity];
    const int4 st = c.slot_state[parity * c.slot_stride + a];
    if (a >= na) return;
    b = st.x;
    tt = st.y + j;
    valid = tt < st.z;
    pr = c.p + (size_t)b * m.Hj;
  } else {
    if (row >= n_dbg) return;
    b = b0; tt = t0 + row; valid = true; pr = p_dbg;
  }
  const float *er = c.e + ((size_t)b * c.T + (valid ? tt : 0)) * m.Hj;
  for (int k = threadIdx.x; k < m.Hj; k += 256) {
    float x = valid ? fmaxf(er[k] + pr[k], 0.f) : 0.f;
    if (round_z) x = bf16_bits_to_f32(f32_to_bf16_bits(x));
    zs[k] = x;
    if (z_out) z_out[(size_t)row * m.Hj + k] = (bf16_t)f32_to_bf16_bits(x);
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const WT *w = reinterpret_cast<const WT *>(m.w_out);
  float best = -INFINITY;
  int best_i = 0x7FFFFFFF;
  for (int v = wave; v <= m.V; v += 4) {
    float a = 0.f;
    for (int k = lane; k < m.Hj; k += 64) a = fmaf(ldw(w, (size_t)v * m.Hj + k), zs[k], a);
    a = wave_sum(a) + m.b_out[v];
    if (logits_out && lane == 0) logits_out[(size_t)row * (m.V + 1) + v] = a;
    if (a > best) { best = a; best_i = v; }   // v ascends within a wave: first maximum kept
  }
  if (lane == 0) { s_val[wave] = best; s_idx[wave] = best_i; }
  __syncthreads();
  if (threadIdx.x == 0 && rows_from_state) {
    float bv = s_val[0];
    int bi = s_idx[0];
    for (int w2 = 1; w2 < 4; ++w2)
      if (s_val[w2] > bv || (s_val[w2] == bv && s_idx[w2] < bi)) { bv = s_val[w2]; bi = s_idx[w2]; }
    c.row_label[row] = valid ? bi : m.V;
  }
}

}  // namespace wind
