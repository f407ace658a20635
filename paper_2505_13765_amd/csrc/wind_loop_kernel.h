// The whole decode loop of one or two utterances as one resident kernel.
#pragma once
#include "wind_types.h"
#include "wind_decide_kernels.h"
#include "wind_pred_kernels.h"

namespace wind {

// ---------------------------------------------------------------------------------------------
// Small decodes as ONE resident kernel.  With one or two utterances and at most 32 window rows the
// loop of Algorithm 2 is a chain of short dependent steps, and between kernels every hand-over costs
// a launch gap plus cold caches.  Here G workgroups stay on the chip for the whole decode; each
// keeps its slice of the weights next to its ALUs for all iterations: 32 columns of W_out as MFMA
// fragments in registers, the recurrent weights of `upw` LSTM units and `ppw` rows of W_pred in LDS.
// What an iteration needs from the other workgroups goes through three exchanges in memory, each
// behind a grid barrier: the rows' keys (every workgroup then takes the same decisions and keeps
// the same pointers, so no state travels), the new hidden vector, the new projection.  An
// iteration without a label has one barrier.
//
// The barrier is one arrival word per workgroup that only grows; a workgroup that waits longer than
// spin_limit polls, or sees the abort word set, sets it and leaves the kernel, so every wave
// reaches the end whatever happens to the others.  The host treats a set abort word as an error.  All G workgroups must be
// resident at once; the host launches at most one per CU.
//
// Placement.  Workgroups are dealt to the chip's eight XCDs in turn by their launch index, and each XCD
// has an L2 of its own.  With at most 32 workgroups (one per CU of an XCD) the host launches eight
// times as many and only every eighth takes part (step = 8), which puts all of them behind ONE L2:
// an exchanged value is then stored through to that L2 and read from it, instead of travelling to
// the memory side and back (a barrier takes 0.6 us instead of 1.5 us).  The kernel checks the
// placement itself: the workgroups publish their XCD number in a first barrier that uses the
// everywhere-valid device-wide stores, and keep those stores unless all numbers are equal.
struct LoopDev {
  unsigned *bar;       // word 0: abort; word 1: 2 if the workgroups shared one L2, 1 if not; word (1 + g) * 32: barriers workgroup g has reached, the next word its XCD number + 1; all zero at launch
  float *h_x;          // [B][Hp] new hidden vectors
  float *p_x;          // [B][Hj] new projections
  float2 *parts_x;     // [2][32][nparts_tiny] keys, by iteration parity
  int G, upw, ppw;     // workgroups; LSTM units and W_pred rows per workgroup (multiples of 4)
  int step;            // launch index of workgroup g is g * step (8: all on one XCD, 1: spread over the chip)
  int zrows;           // rows of the window-row region of LDS (16 or 32; 0: none, the rows go straight into matrix-core operands)
  int max_iters;       // more iterations than any decode of this call can take
  unsigned spin_limit;
};
constexpr int kLoopMaxB = 2;
constexpr int kLoopNearG = 32;                 // CUs of one XCD
constexpr size_t kLoopMaxSmem = 154 * 1024;    // dynamic LDS the kernel may be launched with
constexpr int kLoopRows = 32;
constexpr int kLoopProdRows = 128;   // most weight rows (gate rows + projection rows) of one workgroup

struct LoopShared {
  int4 nslot[kLoopMaxB];
  int ncnt[kLoopMaxB];
  int emit_ub[kLoopMaxB], emit_tok[kLoopMaxB];
  int n_act, n_emit, ok, near;
  int rechecked[4];   // near-tie rows each wave re-decided in this window; -1: the wave did not get this iteration's keys (the kernel ends)
};

// LDS: [wl: upw*4 rows of Hp+8 bf16][wp: ppw rows of Hp+8 bf16][zs: zrows rows of Hj+8 bf16, at least 16 KB]
//      [hhi, hlo: B*Hp bf16 each][pfull: B*Hj f32][cst: B*upw f32][recs: B*upw*4 f32][wbl: Hj f32, fused form only]
// (rows padded by 16 bytes: 32 lanes that read the same k of 32 consecutive rows then hit different banks)
// bf16 elements of the window-row region zs.  The region also takes the K-split partial sums of the MFMA
// phase (4 waves x 16 registers x 64 lanes of fp32 = 16 KB), which is the larger of the two for Hj < 248.
__host__ __device__ inline size_t loop_z_elems(int Hj, int zrows) {
  const size_t z = (size_t)zrows * (Hj + 8);
  return z > 8192 ? z : 8192;
}
// the fused form of the window phase (zrows == 0) keeps the blank column of W_out in LDS as fp32
__host__ __device__ inline size_t loop_wblank_elems(int Hj, int zrows) { return zrows == 0 ? (size_t)Hj : 0; }
constexpr int kFusedRedFloats = 4 * 2 * 4 * 80 + 4 * 2 * 16;   // partial sums of the fused window phase, see there
constexpr int kFusedSteps = 5;   // K steps of 32 per wave in that form: Hj <= 4 * 32 * 5
__host__ __device__ inline size_t loop_smem_bytes(int Hp, int Hj, int B, int upw, int ppw, int zrows) {
  return (size_t)(upw * 4 + ppw) * (Hp + 8) * 2 + (size_t)B * upw * 16 + loop_z_elems(Hj, zrows) * 2 + loop_wblank_elems(Hj, zrows) * 4 + (size_t)B * Hp * 4 +
         (size_t)B * Hj * 4 + (size_t)B * upw * 4;
}

// Values that another workgroup of the running kernel wrote are read with agent-scope atomic loads
// (they skip the CU's own cache) and written with atomic stores, so that the barrier needs no cache
// invalidation and the read-only operands stay in L2 from iteration to iteration.  `near`: all
// workgroups share one L2, a store need only reach that (workgroup scope: written through the CU's
// cache); otherwise it goes to the memory side (agent scope).
__device__ __forceinline__ void st_shared_u32(unsigned *p, unsigned v, bool near) {
  if (near) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_shared_f32(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_shared_f32(float *p, float v, bool near) {
  st_shared_u32(reinterpret_cast<unsigned *>(p), __float_as_uint(v), near);
}
__device__ __forceinline__ float2 ld_shared_f32x2(const float2 *p) {
  const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}
__device__ __forceinline__ void st_shared_f32x2(float2 *p, float2 v, bool near) {
  const unsigned long long u = (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32);
  if (near) __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kLoopFlagStride = 32;   // one 128-byte line per workgroup's arrival word
// The barrier in two halves, so that work that needs nothing from the other workgroups can fill the
// time the arrivals take to travel: loop_arrive publishes this workgroup's arrival, loop_wait waits
// for everybody's.  Between the two a workgroup must not write anything the others read before
// the barrier, nor read what they write.
__device__ __forceinline__ void loop_arrive(const LoopDev &lp, int g, bool near, unsigned passed) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // every lane's own stores of the phase have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    if (!near) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // ... and are visible to the agent before the arrival is
    st_shared_u32(&lp.bar[(1 + g) * kLoopFlagStride], passed + 1, near);
  }
}
// Wave 0's part of the wait: every workgroup publishes the number of barriers it has reached; wave 0 watches
// all of them, one lane per workgroup (no read-modify-write on a shared word: the arrivals do not queue
// up).  Leaves the verdict in ls.ok (read by the others behind the next workgroup barrier) and returns it.
__device__ __forceinline__ bool loop_poll(const LoopDev &lp, unsigned epoch, LoopShared &ls) {
  unsigned spins = 0;
  int good = 1;
  for (;;) {
    bool here = true;
    for (int w0 = 0; w0 < lp.G; w0 += 64) {
      const int w = w0 + (int)threadIdx.x;
      unsigned v = epoch;
      if (w < lp.G) v = __hip_atomic_load(&lp.bar[(1 + w) * kLoopFlagStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      here = here && (int)(v - epoch) >= 0;
    }
    if (__all(here)) break;
    // the word that says another workgroup gave up is looked at every sixteenth time only: asking for it
    // takes as long as asking for the arrivals again
    if (++spins > lp.spin_limit) { good = 0; break; }
    if ((spins & 15u) == 0 && __hip_atomic_load(lp.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) { good = 0; break; }
  }
  if (threadIdx.x == 0) {
    if (!good) __hip_atomic_store(lp.bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ls.ok = good;
  }
  return good != 0;
}
__device__ __forceinline__ bool loop_wait(const LoopDev &lp, unsigned &passed, LoopShared &ls) {
  const unsigned epoch = ++passed;
  if (threadIdx.x < 64) loop_poll(lp, epoch, ls);
  __syncthreads();
  asm volatile("" ::: "memory");   // the exchange reads that follow stay behind the wait
  return ls.ok != 0;
}
__device__ __forceinline__ bool loop_barrier(const LoopDev &lp, int g, bool near, unsigned &passed, LoopShared &ls) {
  loop_arrive(lp, g, near, passed);
  return loop_wait(lp, passed, ls);
}

// Sums of 8 per-lane values over the wave with a halving exchange: each step a lane keeps half of
// its values and adds the partner's copies of them, until one value is left, which the last steps
// sum over the lanes that still hold parts of it.  The steps that carry the most values pair lanes
// inside a row of 16 with DPP permutations (row mirror, half mirror); the lane bit that decides
// which half is kept gives the value's index one bit per step: index = b3 b2 b4 (lane bits), i.e.
// value v ends up, complete, in lanes 16*(v&1) + 4*(v>>1) + 0..3 and the same + 32.
__device__ __forceinline__ float wave_sum8_scatter(const float (&v)[8], int lane) {
  float a[4], b[2];
  const bool u3 = (lane & 8) != 0, u2 = (lane & 4) != 0, u4 = (lane & 16) != 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = (u3 ? v[i + 4] : v[i]) + dpp_f32<kDppRowMirror>(u3 ? v[i] : v[i + 4]);
#pragma unroll
  for (int i = 0; i < 2; ++i) b[i] = (u2 ? a[i + 2] : a[i]) + dpp_f32<kDppRowHalfMirror>(u2 ? a[i] : a[i + 2]);
  float d = (u4 ? b[1] : b[0]) + __shfl_xor(u4 ? b[0] : b[1], 16, kWave);
  d += __shfl_xor(d, 32, kWave);
  d += dpp_f32<kDppQuadXor2>(d);
  d += dpp_f32<kDppQuadXor1>(d);
  return d;
}

// One wave's share of (32 * NBLK weight rows) x (hidden vectors) on the matrix cores: nks steps of 16 along
// K from hsrc (first operand: this lane's row of hi / lo vectors) and wsrc[blk] (second operand: this
// lane's weight row of block blk).  Lane n < 32 then holds row n's sums against first-operand rows
// 0..3 in registers 0..3; hi + lo per utterance go to red_w[row][b].
template <int NBLK>
__device__ __forceinline__ void loop_rows_times_h(const bf16_t *hsrc, const bf16_t *const (&wsrc)[4], int nks, float *red_w,
                                                  int lane, int n_wrows, int B) {
  f32x16 acc[NBLK];
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[blk][r] = 0.f;
  }
  // Two sets of operand registers take turns: while the products of one step run, the reads of the next
  // step land in the other set, and nothing has to be moved between them (a move would wait for its read).
  bf16x8 hv[2], wv[2][NBLK];
  auto read_step = [&](int set, int i) {
    const int ofs = min(i, nks - 1) * 16;   // past the end: the last step again, never used
    hv[set] = *reinterpret_cast<const bf16x8 *>(hsrc + ofs);
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) wv[set][blk] = *reinterpret_cast<const bf16x8 *>(wsrc[blk] + ofs);
  };
  auto products = [&](int set) {
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hv[set], wv[set][blk], acc[blk], 0, 0, 0);
  };
  read_step(0, 0);
  for (int i = 0; i < nks; i += 2) {
    read_step(1, i + 1);
    products(0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1 + NBLK, 0);   // the reads of the next step ...
    __builtin_amdgcn_sched_group_barrier(0x008, NBLK, 0);       // ... then this step's products
    if (i + 1 < nks) {
      read_step(0, i + 2);
      products(1);
      __builtin_amdgcn_sched_group_barrier(0x100, 1 + NBLK, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, NBLK, 0);
    }
  }
  if (lane < 32) {
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
      const int row = blk * 32 + lane;
      if (row < n_wrows) {
#pragma unroll
        for (int b = 0; b < kLoopMaxB; ++b)
          if (b < B) red_w[(size_t)row * kLoopMaxB + b] = acc[blk][2 * b] + acc[blk][2 * b + 1];
      }
    }
  }
}

// What the resident loop kernel expects to find before its launch, in one launch: the arrival words and the
// abort word at zero, the exchanged keys all ones ("two iterations old": the first iterations' tag is 0).
__global__ __launch_bounds__(256) void loop_prepare_kernel(int *bar, int bar_ints, int *keys, int key_ints) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < bar_ints + key_ints; i += gridDim.x * 256) {
    if (i < bar_ints) bar[i] = 0;
    else keys[i - bar_ints] = -1;
  }
}

// What the host reads after a decode by the resident loop kernel, in one launch instead of three copies:
// the active count, the loop's abort and placement words, and the call's counters, written straight
// into pinned host memory (h_flag, h_stats: device-visible addresses of it).
__global__ __launch_bounds__(128) void loop_collect_kernel(const int *n_active, const unsigned *bar, const unsigned long long *stats,
                                                          int n_stats, int *h_flag, unsigned long long *h_stats) {
  const int i = threadIdx.x;
  if (i == 0) h_flag[0] = n_active[0];
  if (i == 1 || i == 2) h_flag[i] = (int)bar[i - 1];
  if (i < n_stats) h_stats[i] = stats[i];
}

// NS: 0 = the window rows go through LDS; 1 .. kFusedSteps = the fused form for Hj = 128 NS (the number of
// K steps of 32 in a wave's quarter of K; a constant, because matrix-core products under a condition
// make the compiler move the accumulators in and out of their registers around every step).
template <int NS>
__global__ __launch_bounds__(256) void wind_loop_kernel(ModelDev m, CallDev c, LoopDev lp) {
  constexpr bool FUSED = NS > 0;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  __shared__ DecideShared sh;
  __shared__ LoopShared ls;
  __shared__ unsigned long long lstats[kNumStats];   // workgroup 0: the call's counters, written out at the end
  if (blockIdx.x % lp.step) return;   // launched only so that the workgroups that take part land on one XCD
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = blockIdx.x / lp.step;
  const int Hj = m.Hj, Hp = m.Hp, W = c.W, B = c.B;
  const int zstride = Hj + 8;
  const int wstride = Hp + 8, nr = lp.upw * 4;   // row stride of the weights in LDS; (unit, gate) rows of this workgroup
  bf16_t *wl = reinterpret_cast<bf16_t *>(smem_raw);
  bf16_t *wp = wl + (size_t)nr * wstride;
  bf16_t *zs = wp + (size_t)lp.ppw * wstride;
  // the hidden vectors as bf16 hi + lo (hi = RNE(h), lo = RNE(h - hi), 16 mantissa bits together): the dot
  // products with the bf16 weights then take one packed instruction per pair and part, with nothing to unpack
  bf16_t *hhi = zs + loop_z_elems(Hj, lp.zrows), *hlo = hhi + (size_t)B * Hp;
  float *pfull = reinterpret_cast<float *>(hlo + (size_t)B * Hp);
  auto put_h2 = [&](int i, float2 v) {   // elements i (even) and i + 1
    const uint32_t hb = pack_bf16x2(v.x, v.y);
    *reinterpret_cast<uint32_t *>(hhi + i) = hb;
    *reinterpret_cast<uint32_t *>(hlo + i) = pack_bf16x2(v.x - __uint_as_float(hb << 16), v.y - __uint_as_float(hb & 0xFFFF0000u));
  };
  float *cst = pfull + (size_t)B * Hj;
  float *recs = cst + (size_t)B * lp.upw;   // [B][nr] recurrent halves of the gate sums, see below
  float *wbl = recs + (size_t)B * nr;       // [Hj] blank column of W_out (fused form)

  // ---- once: this workgroup's weights, the state after the start-token step, the slot table
  const int unit0 = g * lp.upw, prow0 = g * lp.ppw;
  for (int i = tid * 8; i < nr * Hp; i += 256 * 8) {
    const int row = i / Hp, k = i - row * Hp;           // row = 4 * local unit + gate
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (unit0 + (row >> 2) < Hp)
      v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const bf16_t *>(m.w_cat[0]) + ((size_t)unit0 * 4 + row) * Hp + k);
    *reinterpret_cast<u32x4 *>(wl + (size_t)row * wstride + k) = v;
  }
  for (int i = tid * 8; i < lp.ppw * Hp; i += 256 * 8) {
    const int row = i / Hp, k = i - row * Hp;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (prow0 + row < Hj) v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const bf16_t *>(m.w_pred) + (size_t)(prow0 + row) * Hp + k);
    *reinterpret_cast<u32x4 *>(wp + (size_t)row * wstride + k) = v;
  }
  for (int i = tid * 2; i < B * Hp; i += 512) put_h2(i, *reinterpret_cast<const float2 *>(c.h + i));
  for (int i = tid; i < B * Hj; i += 256) pfull[i] = c.p[i];
  for (int i = tid; i < B * lp.upw; i += 256) {
    const int b = i / lp.upw, u = i - b * lp.upw;
    cst[i] = unit0 + u < Hp ? c.c[(size_t)b * Hp + unit0 + u] : 0.f;
  }
  if (tid < kLoopMaxB) {
    sh.slot[tid] = c.slot_state[tid];
    sh.cnt[tid] = c.slot_count[tid];
  }
  for (int i = tid; i < kNumStats; i += 256) lstats[i] = 0ull;
  // Read-only operands are fetched ahead into this XCD's L2, which nothing invalidates while the
  // kernel runs: here this workgroup's columns of every row of emb_gates, below the encoder
  // projections of the window after the current one.
  constexpr int kTouchSteps = FUSED ? 2 : 4;   // rows of the next window a thread touches: 8 * kTouchSteps >= W
  float warm = 0.f, pend[kLoopMaxB * kTouchSteps] = {};
  {
    const int lines = (lp.upw * 16 + 127) / 128;   // 128-byte lines per table row slice
    for (int i = tid; i < (m.V + 1) * lines; i += 256) {
      const int v = i / lines, l = i - v * lines;
      const size_t off = (size_t)v * 4 * Hp + (size_t)unit0 * 4 + l * 32;
      if (unit0 * 4 + l * 32 < 4 * Hp) warm += m.emb_gates[off];
    }
  }
  int na = c.n_active[0];
  // W_out fragments of this workgroup's 32 columns, this wave's quarter of K
  const bool has_cols = g < c.nparts_tiny;
  const int n0 = (has_cols ? g : 0) * kTinyCols;
  const int kq = Hj >> 2, k0 = wave * kq, nk = kq >> 4;
  // separate form: 32 x 32 x 16 products, lane = (column lane & 31, K half lane >> 5)
  const bf16_t *wrow = reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)(n0 + (lane & 31)) * Hj + k0 + (lane >> 5) * 8;
  bf16x8 bfrag[FUSED ? 1 : kTinyPrefetch];
  if constexpr (!FUSED) {
#pragma unroll
    for (int i = 0; i < kTinyPrefetch; ++i)
      if (i < nk) bfrag[i] = *reinterpret_cast<const bf16x8 *>(wrow + i * 16);
  }
  const int cip = lane & 31, col = n0 + cip;
  const bool col_ok = has_cols && col < m.V;
  const float col_bias = col_ok ? m.b_out[col_ok ? col : 0] : kKeyNone;
  // fused form: 16 x 16 x 32 products, two tiles of 16 columns, lane = (column lane & 15, K group lane >> 4)
  constexpr int ns32 = FUSED ? NS : 1;   // = (Hj / 4) / 32 in the fused form
  bf16x8 bfrag16[FUSED ? 2 : 1][ns32];
  float bias16[2] = {kKeyNone, kKeyNone};
  bool ok16[2] = {false, false};
  if constexpr (FUSED) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int cc = n0 + 16 * t + (lane & 15);
      ok16[t] = has_cols && cc < m.V;
      if (ok16[t]) bias16[t] = m.b_out[cc];
      const bf16_t *wr = reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)cc * Hj + k0 + (lane >> 4) * 8;   // rows up to Vpad exist
#pragma unroll
      for (int i = 0; i < ns32; ++i) bfrag16[t][i] = *reinterpret_cast<const bf16x8 *>(wr + i * 32);
    }
    for (int k = tid; k < Hj; k += 256) wbl[k] = m.w_blank[k];
  }
  const float b_blank = m.b_out[m.V];
  CallDev cl = c;   // the decision code reads the keys through parts and, for near-ties, the current projections through p
  cl.p = pfull;
  cl.parts = reinterpret_cast<float *>(zs);   // the iteration's keys are copied over the window rows once those are used up
  constexpr int KI = FUSED ? 1 : kTinyMaxHj / 256;
  float4 wblank[KI];
  if constexpr (!FUSED) {
#pragma unroll
    for (int i = 0; i < KI; ++i) {
      const int k = lane * 4 + 256 * i;
      wblank[i] = k < Hj ? *reinterpret_cast<const float4 *>(m.w_blank + k) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  unsigned passed = 0;
  __syncthreads();
  // Products of this workgroup's weight rows with the hidden vectors, on the matrix cores: sum over k of
  // w[row][k] * (hi[b][k] + lo[b][k]) for n_wrows rows of bf16 weights in LDS and every utterance b.  The
  // utterances' hi and lo vectors are rows 2b and 2b + 1 of the first operand (its other rows are zero),
  // 32 weight rows the second, so lane n < 32 ends up with its weight row's sums in its first registers;
  // K is split over the four waves, whose partial sums go to red[wave][row][b] (the window-row region,
  // which is free whenever this runs).  Up to 128 rows: four independent accumulator blocks in flight.
  // The projection rows follow the gate rows in LDS with the same stride, so one pass can cover both.
  float *red = reinterpret_cast<float *>(zs) + (FUSED ? kFusedRedFloats : 0);   // fused form: behind the window phase's own sums
  auto red_sum = [&](int row, int b) {
    float v = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) v += red[((size_t)w2 * kLoopProdRows + row) * kLoopMaxB + b];
    return v;
  };
  auto weight_rows_times_h = [&](const bf16_t *wbase, int n_wrows) {
    const int kq4 = Hp >> 2, kbeg = wave * kq4, nks = kq4 >> 4;
    const int mrow = lane & 31, kh = (lane >> 5) * 8;
    // rows of the first operand past the utterances' repeat the first: their sums are never looked at
    const bf16_t *hsrc = ((mrow & 1) ? hlo : hhi) + (size_t)(mrow < 2 * B ? (mrow >> 1) : 0) * Hp + kbeg + kh;
    const bf16_t *wsrc[4];
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)   // weight rows past the last repeat it, likewise
      wsrc[blk] = wbase + (size_t)min(blk * 32 + mrow, n_wrows - 1) * wstride + kbeg + kh;
    float *red_w = red + (size_t)wave * kLoopProdRows * kLoopMaxB;
    if (n_wrows <= 32) loop_rows_times_h<1>(hsrc, wsrc, nks, red_w, lane, n_wrows, B);
    else if (n_wrows <= 64) loop_rows_times_h<2>(hsrc, wsrc, nks, red_w, lane, n_wrows, B);
    else if (n_wrows <= 96) loop_rows_times_h<3>(hsrc, wsrc, nks, red_w, lane, n_wrows, B);
    else loop_rows_times_h<4>(hsrc, wsrc, nks, red_w, lane, n_wrows, B);
  };
  // One wave's block of 32 gate rows (blk = 0 .. 2) against the hidden vectors, K unsplit, for the utterances on
  // the emit list: lane n < 32 ends with gate row 32 blk + n's sums and puts them into recs itself.  Four sets
  // of operand registers and two accumulators take turns, so that neither a read nor a product waits for
  // the one before it.
  auto recurrent_block = [&](int blk, int n_em) {
    if (blk * 32 >= nr) return;
    const int mrow = lane & 31, kh = (lane >> 5) * 8, nks = Hp >> 4;   // Hp is a multiple of 64: nks of 4
    const bf16_t *hsrc = ((mrow & 1) ? hlo : hhi) + (size_t)(mrow < 2 * B ? (mrow >> 1) : 0) * Hp + kh;
    const bf16_t *wsrc = wl + (size_t)min(blk * 32 + mrow, nr - 1) * wstride + kh;
    f32x16 acc2[2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc2[q][r] = 0.f;
    bf16x8 hv[4], wv[4];   // four steps of operands in flight: an LDS read takes about as long as three products
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      hv[q] = *reinterpret_cast<const bf16x8 *>(hsrc + q * 16);
      wv[q] = *reinterpret_cast<const bf16x8 *>(wsrc + q * 16);
    }
    for (int i = 0; i < nks; i += 4) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc2[q & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hv[q], wv[q], acc2[q & 1], 0, 0, 0);
        const int ofs = min(i + 4 + q, nks - 1) * 16;   // past the end: the last step again, never used
        hv[q] = *reinterpret_cast<const bf16x8 *>(hsrc + ofs);
        wv[q] = *reinterpret_cast<const bf16x8 *>(wsrc + ofs);
      }
    }
    const int row = blk * 32 + lane;
    if (lane < 32 && row < nr)
      for (int r = 0; r < n_em; ++r) {
        const int ub = ls.emit_ub[r];
        float v = 0.f;
#pragma unroll
        for (int b = 0; b < kLoopMaxB; ++b)
          if (b == ub) v = (acc2[0][2 * b] + acc2[1][2 * b]) + (acc2[0][2 * b + 1] + acc2[1][2 * b + 1]);
        recs[ub * nr + row] = v;
      }
  };
  // The recurrent half of the gate sums, W_hh h, depends on the hidden vector only, which changes
  // when its utterance emits: it is formed as soon as the new vector is here (while the arrivals of
  // the projection exchange travel), so that a step, once the label is known, only adds the
  // label's row of input sums.  recs[b][4 * local unit + gate].
  weight_rows_times_h(wl, nr);
  __syncthreads();
  if (tid < nr)
    for (int b = 0; b < B; ++b) recs[b * nr + tid] = red_sum(tid, b);
  __syncthreads();
  // ---- where the workgroups sit: XCD numbers through a first barrier with device-wide stores
  bool near = false;
  {
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    xcc &= 15u;
    if (tid == 0) st_shared_u32(&lp.bar[(1 + g) * kLoopFlagStride + 1], xcc + 1u, false);
    if (!loop_barrier(lp, g, false, passed, ls)) return;
    if (tid < 64) {
      bool same = true;
      for (int w0 = 0; w0 < lp.G; w0 += 64) {
        const int w = w0 + tid;
        if (w < lp.G) same = same && __hip_atomic_load(&lp.bar[(1 + w) * kLoopFlagStride + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == xcc + 1u;
      }
      same = __all(same);
      if (tid == 0) ls.near = same && lp.step > 1;
    }
    __syncthreads();
    near = ls.near != 0;
    if (g == 0 && tid == 0) lp.bar[1] = near ? 2u : 1u;   // for the host: which stores this launch used
  }

  const bool dbg = c.dbg != nullptr && g == 0 && tid == 0;
  // With at most 64 parts per row and 4 rows per wave the decision only looks at the keys its caller hands it,
  // read straight from the exchange buffer; with at most 32 parts a wave decides four rows at once.  In the
  // fused form those keys carry the iteration's parity (key_with_tag), and the first exchange has no barrier:
  // a reader asks for the keys until all it needs are this iteration's.
  const bool direct = c.nparts_tiny <= 64 && W <= 4 * kRowsAhead;
  const bool quad = direct && c.nparts_tiny <= 32;
  const bool tagged = FUSED && quad;
  // The two key pairs (parts s and s + 16) of window row `row` for the four-rows-at-once decision.  Tagged keys are
  // asked for again until every lane of the wave has this iteration's (bounded like a barrier's wait: false when
  // the limit is reached or another workgroup gave up); the tag is taken out again.
  auto read_quad_keys = [&](const float2 *parts, int row, bool in_window, int s, int tag, float2 &kA, float2 &kB) {
    const float2 none = make_float2(kKeyNone, kKeyNone);
    const bool hasA = in_window && s < c.nparts_tiny, hasB = in_window && s + 16 < c.nparts_tiny;
    unsigned spins = 0;
    for (;;) {
      kA = hasA ? ld_shared_f32x2(parts + (size_t)row * c.nparts_tiny + s) : none;
      kB = hasB ? ld_shared_f32x2(parts + (size_t)row * c.nparts_tiny + s + 16) : none;
      if (!tagged) return true;
      const bool fresh = (!hasA || key_tag(kA.y) == tag) && (!hasB || key_tag(kB.y) == tag);
      if (__all(fresh)) break;
      if (++spins > lp.spin_limit || ((spins & 15u) == 0 && __hip_atomic_load(lp.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
        if (lane == 0) __hip_atomic_store(lp.bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
      }
    }
    kA.y = key_with_tag(kA.y, 0);
    kB.y = key_with_tag(kB.y, 0);
    return true;
  };
  unsigned rs[kStatJump0] = {};   // thread 64 of workgroup 0: counters of the single-utterance windows (fewer than 2^32 each)
  long long tsum[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, n_it = 0, n_em_it = 0;
  for (int it = 0; it < lp.max_iters && na > 0; ++it) {
    const int par = it & 1;
    const long long t0 = dbg ? wall_clock64() : 0;
    const int n_rows = na * W;
    float2 *parts = lp.parts_x + (size_t)par * kLoopRows * c.nparts_tiny;
    for (int j = tid; j <= kMaxWindow; j += 256) sh.hist[j] = 0u;
    // last iteration's touches of this window's lines (see below) are consumed here, before this iteration's
    // loads are issued: by now they have long arrived
#pragma unroll
    for (int i = 0; i < kLoopMaxB * kTouchSteps; ++i) { warm += pend[i]; pend[i] = 0.f; }
    f32x4 facc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    if constexpr (FUSED) {
      // ---- window rows straight into matrix-core operands: lane = (row lane & 15, K group lane >> 4) reads 8
      // consecutive projections per step of 32 of this wave's quarter of K, adds the prediction
      // projection, applies the ReLU and rounds: that is its part of the first operand of a 16 x 16 x 32
      // product against the W_out fragments in registers.  The fp32 blank logit and norm of the row
      // are summed over the K groups by lane exchanges and over the waves through LDS, like the products.
      const int row = lane & 15, kofs = k0 + (lane >> 4) * 8;
      // A row past the utterance's end (or past the last window) reads the utterance's first frame instead:
      // nothing looks at what such a row yields, and loads under a lane's condition would have to wait
      // for and merge with the registers' old values.
      int arow = 0;
      unsigned eofs = 0;   // the host has checked that B * T * Hj fits 32 bits
      if (row < n_rows) {
        const int a = row >= W ? 1 : 0, j = row - a * W;   // at most two utterances
        const int4 st = sh.slot[a];
        arow = st.x;
        eofs = ((unsigned)st.x * (unsigned)c.T + (unsigned)(st.y + j < st.z ? st.y + j : 0)) * (unsigned)Hj;
      }
      const float *er = c.e + eofs + kofs;
      float4 ev[ns32][2];
#pragma unroll
      for (int i = 0; i < ns32; ++i) {
        ev[i][0] = *reinterpret_cast<const float4 *>(er + i * 32);
        ev[i][1] = *reinterpret_cast<const float4 *>(er + i * 32 + 4);
      }
      // Touch the lines of the window after this one, so that they sit in L2 when it is their turn.  The
      // values are consumed one iteration later (each into a register of its own: nothing waits for them here).
      {
        const int lines_per_row = (Hj * 4 + 127) / 128;   // at most 32: eight rows per step, 32 lanes each
        // every lane issues every load, with its row and line clamped into the utterance's frames
        const int l = min(tid & 31, lines_per_row - 1);
#pragma unroll
        for (int a = 0; a < kLoopMaxB; ++a)
          if (a < na) {
            const int4 st = sh.slot[a];
#pragma unroll
            for (int i2 = 0; i2 < kTouchSteps; ++i2) {
              const int tr = max(min(st.y + W + (tid >> 5) + 8 * i2, st.z - 1), 0);
              pend[a * kTouchSteps + i2] = c.e[((unsigned)st.x * (unsigned)c.T + (unsigned)tr) * (unsigned)Hj + (unsigned)(l * 32)];
            }
          }
      }
      float dot = 0.f, nrm = 0.f;
      const float *pr = pfull + (size_t)arow * Hj + kofs, *wr = wbl + kofs;
      // the LDS operands of a step (projection, blank column) are read one step ahead, into registers that take turns
      float4 po[2][2], wo[2][2];
      auto read_ops = [&](int set, int i) {
        const int ofs = min(i, ns32 - 1) * 32;   // past the end: the last step again, never used
        po[set][0] = *reinterpret_cast<const float4 *>(pr + ofs); po[set][1] = *reinterpret_cast<const float4 *>(pr + ofs + 4);
        wo[set][0] = *reinterpret_cast<const float4 *>(wr + ofs); wo[set][1] = *reinterpret_cast<const float4 *>(wr + ofs + 4);
      };
      read_ops(0, 0);
#pragma unroll
      for (int i = 0; i < ns32; ++i) {
        read_ops((i + 1) & 1, i + 1);
        const float4 p0 = po[i & 1][0], p1 = po[i & 1][1], w0 = wo[i & 1][0], w1 = wo[i & 1][1];
        float x[8];
        x[0] = fmaxf(ev[i][0].x + p0.x, 0.f); x[1] = fmaxf(ev[i][0].y + p0.y, 0.f);
        x[2] = fmaxf(ev[i][0].z + p0.z, 0.f); x[3] = fmaxf(ev[i][0].w + p0.w, 0.f);
        x[4] = fmaxf(ev[i][1].x + p1.x, 0.f); x[5] = fmaxf(ev[i][1].y + p1.y, 0.f);
        x[6] = fmaxf(ev[i][1].z + p1.z, 0.f); x[7] = fmaxf(ev[i][1].w + p1.w, 0.f);
        dot = fmaf(x[0], w0.x, dot); dot = fmaf(x[1], w0.y, dot); dot = fmaf(x[2], w0.z, dot); dot = fmaf(x[3], w0.w, dot);
        dot = fmaf(x[4], w1.x, dot); dot = fmaf(x[5], w1.y, dot); dot = fmaf(x[6], w1.z, dot); dot = fmaf(x[7], w1.w, dot);
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) nrm = fmaf(x[e2], x[e2], nrm);
        const u32x4 zu = u32x4{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
        const bf16x8 zf = __builtin_bit_cast(bf16x8, zu);
        facc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(zf, bfrag16[0][i], facc[0], 0, 0, 0);
        facc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(zf, bfrag16[1][i], facc[1], 0, 0, 0);
      }
      dot += __shfl_xor(dot, 16, kWave); nrm += __shfl_xor(nrm, 16, kWave);
      dot += __shfl_xor(dot, 32, kWave); nrm += __shfl_xor(nrm, 32, kWave);
      // partial sums of this wave's quarter of K: fred[wave][tile][r][80] (register r of lane l: row 4 * (l >> 4) + r,
      // column 16 * tile + (l & 15); 80 floats per r so that the readers below hit different banks), then
      // fbn[wave][blank part, squared norm][row]
      float *fred = reinterpret_cast<float *>(zs), *fbn = fred + 4 * 2 * 4 * 80;   // kFusedRedFloats in all
#pragma unroll
      for (int t = 0; t < 2; ++t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) fred[((wave * 2 + t) * 4 + r) * 80 + lane] = facc[t][r];
      }
      if (lane < 16) {
        fbn[(wave * 2 + 0) * 16 + lane] = dot;
        fbn[(wave * 2 + 1) * 16 + lane] = nrm;
      }
      __syncthreads();
      const long long t1 = dbg ? wall_clock64() : 0;
      if (dbg) tsum[0] += t1 - t0;
      // wave w finishes rows 4w .. 4w + 3: lane = (row 4w + (lane >> 4), column lane & 15 of either tile)
      {
        const int rr = lane >> 4, cj = lane & 15, orow = 4 * wave + rr;
        float k1 = kKeyNone, k2 = kKeyNone;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          float v = bias16[t];
#pragma unroll
          for (int w2 = 0; w2 < 4; ++w2) v += fred[((w2 * 2 + t) * 4 + rr) * 80 + 16 * wave + cj];
          push_top2(k1, k2, make_key(ok16[t] ? v : kKeyNone, 16 * t + cj));
        }
        merge_top2(k1, k2, dpp_f32<kDppRowMirror>(k1), dpp_f32<kDppRowMirror>(k2));
        merge_top2(k1, k2, dpp_f32<kDppRowHalfMirror>(k1), dpp_f32<kDppRowHalfMirror>(k2));
        merge_top2(k1, k2, dpp_f32<kDppQuadXor2>(k1), dpp_f32<kDppQuadXor2>(k2));
        merge_top2(k1, k2, dpp_f32<kDppQuadXor1>(k1), dpp_f32<kDppQuadXor1>(k2));
        if (tagged) k2 = key_with_tag(k2, (it >> 1) & 1);
        if (has_cols && cj == 0) st_shared_f32x2(&parts[(size_t)orow * c.nparts_tiny + g], make_float2(k1, k2), near);
      }
      if (tid < 16 && tid < n_rows) {
        float d2 = b_blank, n2 = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) { d2 += fbn[(w2 * 2 + 0) * 16 + tid]; n2 += fbn[(w2 * 2 + 1) * 16 + tid]; }
        sh.blank[tid] = d2;
        sh.znorm[tid] = sqrtf(n2);
      }
      if (dbg) tsum[1] += wall_clock64() - t1;
    } else {
      // ---- window rows into LDS with their fp32 blank logit and norm (every workgroup: all rows)
      for (int q0 = 0; q0 < 8; q0 += 4) {
        if (q0 * 4 >= n_rows) continue;   // no window rows in this pass (what those rows of z hold is never looked at)
        float4 ev[4][KI];
        bool valid[4];
        int arow[4];
  #pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = wave + 4 * (q0 + q);
          valid[q] = false;
          arow[q] = 0;
          const float *er = c.e;
          if (row < n_rows) {
            const int a = row >= W ? 1 : 0, j = row - a * W;   // at most two utterances
            const int4 st = sh.slot[a];
            valid[q] = st.y + j < st.z;
            arow[q] = st.x;
            er = c.e + ((unsigned)st.x * (unsigned)c.T + (unsigned)(valid[q] ? st.y + j : 0)) * (unsigned)Hj;   // fits 32 bits: checked by the host
          }
  #pragma unroll
          for (int i = 0; i < KI; ++i) {
            const int k = lane * 4 + 256 * i;
            ev[q][i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (valid[q] && k < Hj) ev[q][i] = *reinterpret_cast<const float4 *>(er + k);
          }
        }
        float dn[8];   // [q][blank-logit part, squared norm]
  #pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = wave + 4 * (q0 + q);
          float dot = 0.f, nrm = 0.f;
  #pragma unroll
          for (int i = 0; i < KI; ++i) {
            const int k = lane * 4 + 256 * i;
            if (k < Hj && row < n_rows) {   // rows past the windows: what z holds there is never looked at
              float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
              if (valid[q]) {
                const float4 pv = *reinterpret_cast<const float4 *>(pfull + (size_t)arow[q] * Hj + k);
                x.x = fmaxf(ev[q][i].x + pv.x, 0.f); x.y = fmaxf(ev[q][i].y + pv.y, 0.f);
                x.z = fmaxf(ev[q][i].z + pv.z, 0.f); x.w = fmaxf(ev[q][i].w + pv.w, 0.f);
              }
              *reinterpret_cast<uint2 *>(zs + (size_t)row * zstride + k) = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
              const float4 wb = wblank[i];
              dot = fmaf(x.x, wb.x, dot); dot = fmaf(x.y, wb.y, dot); dot = fmaf(x.z, wb.z, dot); dot = fmaf(x.w, wb.w, dot);
              nrm = fmaf(x.x, x.x, nrm); nrm = fmaf(x.y, x.y, nrm); nrm = fmaf(x.z, x.z, nrm); nrm = fmaf(x.w, x.w, nrm);
            }
          }
          dn[2 * q] = dot;
          dn[2 * q + 1] = nrm;
        }
        const float tot = wave_sum8_scatter(dn, lane);   // lane 4q: row q's dot; lane 4q + 16: its squared norm
        const int rowq = wave + 4 * (q0 + ((lane >> 2) & 3));
        if (rowq < n_rows && (lane & 0x23) == 0) {
          if (lane & 16) sh.znorm[rowq] = sqrtf(tot);
          else sh.blank[rowq] = tot + b_blank;
        }
      }
      // Touch the lines of the window after this one, so that they sit in L2 when it is their turn.  The
      // values are consumed one iteration later (each into a register of its own: nothing waits for them here).
      {
        const int lines_per_row = (Hj * 4 + 127) / 128;   // at most 32: eight rows per step, 32 lanes each
        // every lane issues every load, with its row and line clamped into the utterance's frames: a load
        // under a lane's condition would have to merge with the register's old value, and wait for it
        const int l = min(tid & 31, lines_per_row - 1);
#pragma unroll
        for (int a = 0; a < kLoopMaxB; ++a)
          if (a < na) {
            const int4 st = sh.slot[a];
#pragma unroll
            for (int i2 = 0; i2 < kTouchSteps; ++i2) {
              const int tr = max(min(st.y + W + (tid >> 5) + 8 * i2, st.z - 1), 0);
              pend[a * kTouchSteps + i2] = c.e[((unsigned)st.x * (unsigned)c.T + (unsigned)tr) * (unsigned)Hj + (unsigned)(l * 32)];
            }
          }
      }
      __syncthreads();
      const long long t1 = dbg ? wall_clock64() : 0;
      if (dbg) { tsum[0] += t1 - t0; }
      // ---- this workgroup's 32 columns: K split over the four waves, W_out from registers
      if (has_cols) {
        f32x16 acc;
  #pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        const bf16_t *zrow = zs + (size_t)min(lane & 31, lp.zrows - 1) * zstride + k0 + (lane >> 5) * 8;   // rows past the region repeat its last row; never looked at
  #pragma unroll
        for (int i = 0; i < kTinyPrefetch; ++i)
          if (i < nk) {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(zrow + i * 16);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bfrag[i], acc, 0, 0, 0);
          }
        __syncthreads();   // every wave is done with z: its LDS takes the K-split partial sums
        float *red = reinterpret_cast<float *>(zs);   // [wave][r][lane]
  #pragma unroll
        for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[r];
        __syncthreads();
        if (wave == 0) {
          float k1[16], k2[16];
  #pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = col_bias;
  #pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) v += red[(w2 * 16 + r) * 64 + lane];
            k1[r] = make_key(col_ok ? v : kKeyNone, cip);
            k2[r] = kKeyNone;
          }
          float o1[1], o2[1];
          RowTop2<16, 0>::run(k1, k2, lane, o1, o2);
          const int s0 = rowtop2_first_slot<16>(lane);
          st_shared_f32x2(&parts[(size_t)acc_row(0, s0, lane) * c.nparts_tiny + g], make_float2(o1[0], o2[0]), near);
        }
      }
      if (dbg) tsum[1] += wall_clock64() - t1;
    }
    const long long t2 = dbg ? wall_clock64() : 0;
    if (tagged) __syncthreads();                           // exchange 1: tagged keys, asked for until they are this iteration's;
    else if (!loop_barrier(lp, g, near, passed, ls)) return;   // ... otherwise behind a barrier: every row's keys are in memory
    const long long t3 = dbg ? wall_clock64() : 0;
    // ---- the decisions, taken alike by every workgroup; workgroup 0 writes the outputs
    // With at most 64 parts per row and 4 rows per wave the decision only looks at the keys its
    // caller hands it, which are read here straight from the exchange buffer; otherwise the keys
    // are copied to LDS first.
    float2 *lparts = reinterpret_cast<float2 *>(zs);
    if (!direct) {
      for (int i = tid; i < n_rows * c.nparts_tiny; i += 256) lparts[i] = ld_shared_f32x2(parts + i);
      __syncthreads();
    }
    int n_emit = 0;
    if (quad && na == 1) {
      // One utterance: its rows four per wave, then first non-blank row, update, lists and counters in one
      // go by wave 0: two workgroup barriers in all.
      const int4 st = sh.slot[0];
      const int cnt0 = sh.cnt[0];   // read on this side of the workgroup barrier below: wave 0 writes the new count right behind it
      const int s = lane & 15, j = wave + (lane >> 4) * 4;
      float2 kA, kB;
      const bool fresh = read_quad_keys(parts, j, j < W, s, (it >> 1) & 1, kA, kB);
      float vb = 0.f, zn = 0.f;
      if (j < W) {
        vb = sh.blank[j];
        zn = sh.znorm[j];
      }
      auto reload = [&](int r, int part) {
        float2 k = ld_shared_f32x2(parts + (size_t)r * c.nparts_tiny + part);
        if (tagged) k.y = key_with_tag(k.y, 0);
        return k;
      };
      int rechecked = 0;
      if (fresh) rechecked = decide_rows_quad<bf16_t>(m, cl, 0, st, c.nparts_tiny, kTinyCols, kA, kB, vb, zn, j, reload, sh);
      if (lane == 0) ls.rechecked[wave] = fresh ? rechecked : -1;
      __syncthreads();
      // what the rest needs from LDS, asked for in one go: the waves' verdicts and the rows' labels
      const int v0 = ls.rechecked[0], v1 = ls.rechecked[1], v2 = ls.rechecked[2], v3 = ls.rechecked[3];
      const int lab = sh.label[lane & 15];
      if ((v0 | v1 | v2 | v3) < 0) return;   // some wave gave up waiting for keys
      // Wave 0 applies the outcome to the loop's own state; in workgroup 0 wave 1 works out the same outcome beside
      // it and does what only the caller sees: the outputs and the call's counters.
      if (wave == 0 || (wave == 1 && g == 0)) {
        const int n = min(W, st.z - st.y);
        const unsigned long long mask = __ballot(lane < n && lab != m.V);
        const int i = mask ? __ffsll((long long)mask) - 1 : -1;   // smallest i with labels[i] != blank
        const int label_i = i < 0 ? m.V : __builtin_amdgcn_readlane(lab, i);
        if (lane == 0) {
          const WindowOutcome wo = window_outcome(cl, st, cnt0, n, i, label_i, m.V, v0 + v1 + v2 + v3, wave == 1);
          if (wave == 0) {
            ls.n_act = wo.flag & 1;
            ls.n_emit = (wo.flag >> 1) & 1;
            if (wo.flag & 2) { ls.emit_ub[0] = wo.slot.x; ls.emit_tok[0] = wo.tok; }
            if (wo.flag & 1) { sh.slot[0] = wo.slot; sh.cnt[0] = wo.cnt; }
          } else {
            const unsigned ev = wo.ev;
            // this thread's registers take the counters (a chain of read-modify-writes in LDS would be a microsecond)
            rs[ST_ROWS] += ev & 127u; rs[ST_USEFUL] += (ev >> 7) & 127u; rs[ST_RECHECK] += (ev >> 21) & 127u;
            rs[ST_LABELS] += (ev >> 28) & 1u; rs[ST_FORCED] += (ev >> 29) & 1u; rs[ST_OVERFLOW] += (ev >> 30) & 1u;
            rs[ST_ITER] += 1u; rs[ST_WINDOWS] += 1u;
            atomicAdd(&lstats[kStatJump0 + ((ev >> 14) & 127u)], 1ull);   // nobody waits for the sum
          }
        }
      }
      __syncthreads();
      na = ls.n_act;
      n_emit = ls.n_emit;
    } else {
    for (int a = 0; a < na; ++a) {
      RowsAhead ahead;
      if (quad) {
        const int s = lane & 15, j = wave + (lane >> 4) * 4, row = a * W + j;
        float2 kA, kB;
        const bool fresh = read_quad_keys(parts, row, j < W, s, (it >> 1) & 1, kA, kB);
        if (tagged && !__syncthreads_and(fresh)) return;   // some wave gave up waiting for keys
        float vb = 0.f, zn = 0.f;
        if (j < W) {
          vb = sh.blank[row];
          zn = sh.znorm[row];
        }
        auto reload = [&](int r, int part) {
          float2 k = ld_shared_f32x2(parts + (size_t)r * c.nparts_tiny + part);
          if (tagged) k.y = key_with_tag(k.y, 0);
          return k;
        };
        const int rechecked = decide_rows_quad<bf16_t>(m, cl, a, sh.slot[a], c.nparts_tiny, kTinyCols, kA, kB, vb, zn, j, reload, sh);
        decide_utterance<bf16_t, true>(m, cl, a, sh.slot[a], sh.cnt[a], 0, c.nparts_tiny, c.nparts_tiny, kTinyCols, ahead, sh,
                                       g == 0, true, rechecked);
        continue;
      }
#pragma unroll
      for (int q = 0; q < kRowsAhead; ++q) {
        const int j = wave + q * 4, row = a * W + j;
        ahead.kk0[q] = no_keys();
        ahead.vb[q] = 0.f; ahead.zn[q] = 0.f;
        if (j < W) {
          if (lane < c.nparts_tiny) {
            const float2 k2 = direct ? ld_shared_f32x2(parts + (size_t)row * c.nparts_tiny + lane) : lparts[(size_t)row * c.nparts_tiny + lane];
            ahead.kk0[q].x = k2.x;
            ahead.kk0[q].y = k2.y;
          }
          ahead.vb[q] = sh.blank[row];
          ahead.zn[q] = sh.znorm[row];
        }
      }
      decide_utterance<bf16_t, true>(m, cl, a, sh.slot[a], sh.cnt[a], 0, c.nparts_tiny, c.nparts_tiny, kTinyCols, ahead, sh,
                                     g == 0);
    }
    if (wave == 0) {
      // survivors keep their order; the emit list is the survivors that produced a label
      if (lane == 0) {
        int n_act = 0, n_em = 0;
        for (int a = 0; a < na; ++a) {
          const int f = sh.flag[a];
          if (f & 2) { ls.emit_ub[n_em] = sh.slot[a].x; ls.emit_tok[n_em] = sh.tok[a]; ++n_em; }
          if (f & 1) { ls.nslot[n_act] = sh.slot[a]; ls.ncnt[n_act] = sh.cnt[a]; ++n_act; }
          if (g == 0) {   // the window's counters (see decide_utterance for the packing)
            const unsigned ev = sh.event[a];
            lstats[ST_ROWS] += ev & 127u; lstats[ST_USEFUL] += (ev >> 7) & 127u; lstats[ST_RECHECK] += (ev >> 21) & 127u;
            lstats[ST_LABELS] += (ev >> 28) & 1u; lstats[ST_FORCED] += (ev >> 29) & 1u; lstats[ST_OVERFLOW] += (ev >> 30) & 1u;
            lstats[kStatJump0 + ((ev >> 14) & 127u)] += 1ull;
          }
        }
        if (g == 0) { lstats[ST_ITER] += 1ull; lstats[ST_WINDOWS] += (unsigned long long)na; }
        ls.n_act = n_act;
        ls.n_emit = n_em;
      }
    }
    __syncthreads();
    na = ls.n_act;
    n_emit = ls.n_emit;
    if (tid < na) { sh.slot[tid] = ls.nslot[tid]; sh.cnt[tid] = ls.ncnt[tid]; }
    __syncthreads();
    }
    const long long t4 = dbg ? wall_clock64() : 0;
    if (dbg) { tsum[2] += t3 - t2; tsum[3] += t4 - t3; ++n_it; }
    if (n_emit == 0 || na == 0) continue;
    // ---- one LSTM step for the utterances that emitted: this workgroup's units, weights from LDS
    // thread 4u + gate: that gate of the workgroup's unit u (the label's input sums are one coalesced read)
    for (int r = 0; r < n_emit; ++r) {
      const int ub = ls.emit_ub[r], tok = ls.emit_tok[r];
      if (tid < nr) {
        const int ul = tid >> 2, gate = tid & 3, unit = unit0 + ul;
        const bool ok = unit < Hp;
        float pre = 0.f;
        if (ok) pre = recs[ub * nr + tid] + m.emb_gates[(unsigned)tok * 4u * (unsigned)Hp + (unsigned)(unit0 * 4 + tid)];   // fits 32 bits: checked by the host
        const float act = gate == 2 ? tanhf(pre) : 1.f / (1.f + expf(-pre));
        const int base = lane & ~3;
        const float ig = __shfl(act, base, kWave), fg = __shfl(act, base + 1, kWave);
        const float gg = __shfl(act, base + 2, kWave), og = __shfl(act, base + 3, kWave);
        if (gate == 0 && ok) {
          const float cn = fg * cst[ub * lp.upw + ul] + ig * gg;
          cst[ub * lp.upw + ul] = cn;
          st_shared_f32(&lp.h_x[(size_t)ub * Hp + unit], og * tanhf(cn), near);
        }
      }
    }
    const long long t5 = dbg ? wall_clock64() : 0;
    if (!loop_barrier(lp, g, near, passed, ls)) return;   // exchange 2: the new hidden vectors
    const long long t6 = dbg ? wall_clock64() : 0;
    for (int r = 0; r < n_emit; ++r) {
      const int ub = ls.emit_ub[r];
      for (int k = tid * 2; k < Hp; k += 512) put_h2(ub * Hp + k, ld_shared_f32x2(reinterpret_cast<const float2 *>(&lp.h_x[(size_t)ub * Hp + k])));
    }
    __syncthreads();
    // ---- this workgroup's rows of the prediction projection; the recurrent sums of the next step, which
    // want the same new vectors, in the same pass (rows nr .. nr + ppw - 1 and 0 .. nr - 1 of the weights
    // in LDS), or, in the fused form, put off to the time the next window's loads take
    const int prow_red = FUSED ? 0 : nr;
    if constexpr (FUSED) weight_rows_times_h(wp, lp.ppw);
    else weight_rows_times_h(wl, nr + lp.ppw);
    __syncthreads();
    if (tid < lp.ppw && prow0 + tid < Hj) {
      const int j = prow0 + tid;
      const float bj = m.b_pred[j];
      for (int r = 0; r < n_emit; ++r) {
        const int ub = ls.emit_ub[r];
        st_shared_f32(&lp.p_x[(size_t)ub * Hj + j], red_sum(prow_red + tid, ub) + bj, near);
      }
    }
    const long long t7 = dbg ? wall_clock64() : 0;
    loop_arrive(lp, g, near, passed);                     // exchange 3: the new projections ...
    long long t8 = 0;
    if constexpr (FUSED) {
      // ... and, while wave 0 watches the arrivals and then copies the new projections in, each other wave renews
      // the recurrent sums of a block of 32 gate rows over the whole of K (they are wanted by the next label's
      // step, not before)
      const unsigned epoch = ++passed;
      if (wave >= 1) {
        recurrent_block(wave - 1, n_emit);
      } else if (loop_poll(lp, epoch, ls)) {
        asm volatile("" ::: "memory");   // the exchange reads that follow stay behind the wait
        t8 = dbg ? wall_clock64() : 0;
        constexpr int KP = 2 * ns32;   // Hj = 128 NS = 64 KP
        for (int r = 0; r < n_emit; ++r) {
          const int ub = ls.emit_ub[r];
          float pv[KP];
#pragma unroll
          for (int i = 0; i < KP; ++i) pv[i] = ld_shared_f32(&lp.p_x[(unsigned)(ub * Hj + lane + 64 * i)]);
#pragma unroll
          for (int i = 0; i < KP; ++i) pfull[ub * Hj + lane + 64 * i] = pv[i];
        }
      }
      __syncthreads();
      if (!ls.ok) return;
    } else {
      if (tid < nr) {                                     // ... and, while the arrivals travel, the recurrent sums are put by
        for (int r = 0; r < n_emit; ++r) {
          const int ub = ls.emit_ub[r];
          recs[ub * nr + tid] = red_sum(tid, ub);
        }
      }
      if (!loop_wait(lp, passed, ls)) return;
      t8 = dbg ? wall_clock64() : 0;
      for (int r = 0; r < n_emit; ++r) {
        const int ub = ls.emit_ub[r];
        for (int k = tid; k < Hj; k += 256) pfull[(size_t)ub * Hj + k] = ld_shared_f32(&lp.p_x[(size_t)ub * Hj + k]);
      }
      __syncthreads();
    }
    if (dbg) {
      const long long t9 = wall_clock64();
      tsum[4] += t5 - t4; tsum[5] += t6 - t5; tsum[6] += t7 - t6; tsum[7] += t8 - t7; tsum[8] += t9 - t8; ++n_em_it;
    }
  }
  if (dbg) {
    for (int i = 0; i < 9; ++i) c.dbg[i] += tsum[i];
    c.dbg[10] += n_it; c.dbg[11] += n_em_it;
  }
  __syncthreads();
  if (g == 0) {
    if (tid == 64)   // the thread that kept the counters of the windows of single utterances
      for (int i = 0; i < kStatJump0; ++i) lstats[i] += rs[i];
    __syncthreads();
    for (int i = tid; i < kNumStats; i += 256) c.stats[i] = lstats[i];
    if (tid == 0) {
      c.n_active[0] = na;   // zero unless max_iters ran out
      c.n_active[1] = na;
    }
  }
  if (warm == 1.2345e-30f && lp.spin_limit == 0u) lp.h_x[0] = warm;   // keeps the warming loads alive; never true
}

}  // namespace wind
