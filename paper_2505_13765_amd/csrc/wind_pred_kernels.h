// The prediction network: the load-time table of the first layer's input sums, LSTM layers and the
// projection in three implementations (fp32 FMA, low-latency wave-per-unit, hi/lo-split bf16 MFMA tiles).
#pragma once
#include "wind_types.h"

namespace wind {

// ---------------------------------------------------------------------------------------------
// Column slices of 32 labels: the unit in which the resident loop kernel's workgroups own W_out.
constexpr int kTinyCols = 32;
constexpr int kTinyMaxHj = 1024;    // the loop kernel keeps its window rows in registers, then LDS
constexpr int kTinyPrefetch = 16;   // W_out fragments (K steps of 16) a wave of that kernel keeps in registers

// ---------------------------------------------------------------------------------------------
// Load time: out[v][r] = bias[r] + sum_k w[r][k] * emb[v][k] for v < nv, r < nr (fp32 accumulation,
// k ascending).  Plain LDS-tiled product, 64 x 64 outputs per workgroup, 4 x 4 per thread.
template <class WT>
__global__ __launch_bounds__(256) void emb_gates_kernel(const WT *emb, const WT *w, const float *bias, float *out,
                                                        int nv, int nr, int E) {
  __shared__ float as[16][65], bs[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int v0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < E; k0 += 16) {
    for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
      const int row = idx >> 4, kk = idx & 15, k = k0 + kk;
      as[kk][row] = (v0 + row < nv && k < E) ? ldw(emb, (size_t)(v0 + row) * E + k) : 0.f;
      bs[kk][row] = (r0 + row < nr && k < E) ? ldw(w, (size_t)(r0 + row) * E + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = as[kk][ty * 4 + i]; b[i] = bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int v = v0 + ty * 4 + i, r = r0 + tx * 4 + j;
      if (v < nv && r < nr) out[(size_t)v * nr + r] = acc[i][j] + bias[r];
    }
}

// ---------------------------------------------------------------------------------------------
// One LSTM cell for the utterances on the emit list.  One wave per hidden unit: its four gate rows
// are dotted with [x ; h_prev] of R utterances at a time (weights are read once per group).
//   x = the new h of the layer below; layer 0 has no x part, the emitted label's row of emb_gates
//   carries its input sums and biases.
template <class WT, int R>
__global__ __launch_bounds__(256) void lstm_layer_kernel(ModelDev m, CallDev c, int layer) {
  const int n_emit = *c.n_emit;
  if (n_emit == 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int unit = blockIdx.x * 4 + wave;
  if (unit >= m.Hp) return;
  const int Hp = m.Hp, in = layer == 0 ? 0 : Hp, K = in + Hp;
  const WT *w = reinterpret_cast<const WT *>(m.w_cat[layer]) + (size_t)unit * 4 * K;
  const float *bias = m.b_cat[layer] + unit * 4;
  const size_t lofs = (size_t)layer * c.B * Hp;
  constexpr int VEC = sizeof(WT) == 2 ? 2 : 1;

  for (int r0 = 0; r0 < n_emit; r0 += R) {
    float acc[4][R];
    int ub[R];
    const float *xg[R];  // layer 0: the label's row of input gate sums
    const float *xh[R];  // deeper layers: new hidden vector of the layer below
    const float *hp[R];  // this layer's previous hidden vector
#pragma unroll
    for (int r = 0; r < R; ++r) {
      ub[r] = c.emit_idx[min(r0 + r, n_emit - 1)];
      xg[r] = m.emb_gates + (size_t)c.emit_list_tok[min(r0 + r, n_emit - 1)] * 4 * Hp + unit * 4;
      xh[r] = c.hn + (layer == 0 ? 0 : lofs - (size_t)c.B * Hp) + (size_t)ub[r] * Hp;
      hp[r] = c.h + lofs + (size_t)ub[r] * Hp;
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g][r] = 0.f;
    }
    for (int k = lane * VEC; k < K; k += 64 * VEC) {
      float wv[4][VEC];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if constexpr (VEC == 2) {
          const float2 t2 = ldw2(w, (size_t)g * K + k);
          wv[g][0] = t2.x; wv[g][1] = t2.y;
        } else {
          wv[g][0] = ldw(w, (size_t)g * K + k);
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float xv[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
          const int kk = k + q;
          xv[q] = kk < in ? xh[r][kk] : hp[r][kk - in];
        }
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int q = 0; q < VEC; ++q) acc[g][r] = fmaf(wv[g][q], xv[q], acc[g][r]);
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g][r] = wave_sum(acc[g][r]);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (lane == r && r0 + r < n_emit) {
        const size_t si = lofs + (size_t)ub[r] * Hp + unit;
        const float *add = layer == 0 ? xg[r] : bias;
        const float ig = 1.f / (1.f + expf(-(acc[0][r] + add[0])));
        const float fg = 1.f / (1.f + expf(-(acc[1][r] + add[1])));
        const float gg = tanhf(acc[2][r] + add[2]);
        const float og = 1.f / (1.f + expf(-(acc[3][r] + add[3])));
        const float cn = fg * c.c[si] + ig * gg;
        c.c[si] = cn;
        c.hn[si] = og * tanhf(cn);
      }
    }
  }
}

// p[b,:] = W_pred h_top + b_pred for the utterances on the emit list; also commits the new hidden
// vectors (hn -> h) now that every layer has read the old ones.
template <class WT, int R>
__global__ __launch_bounds__(256) void pred_proj_kernel(ModelDev m, CallDev c) {
  const int n_emit = *c.n_emit;
  if (n_emit == 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int Hp = m.Hp;
  // commit: grid-strided copy over [L][n_emit][Hp]
  {
    const size_t total = (size_t)m.L * n_emit * Hp;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
      const int k = (int)(i % Hp);
      const size_t q = i / Hp;
      const int r = (int)(q % n_emit), l = (int)(q / n_emit);
      const size_t si = ((size_t)l * c.B + c.emit_idx[r]) * Hp + k;
      c.h[si] = c.hn[si];
    }
  }
  const int j = blockIdx.x * 4 + wave;
  if (j >= m.Hj) return;
  const WT *w = reinterpret_cast<const WT *>(m.w_pred) + (size_t)j * Hp;
  const float *htop = c.hn + (size_t)(m.L - 1) * c.B * Hp;
  constexpr int VEC = sizeof(WT) == 2 ? 2 : 1;
  for (int r0 = 0; r0 < n_emit; r0 += R) {
    float acc[R];
    int ub[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { ub[r] = c.emit_idx[min(r0 + r, n_emit - 1)]; acc[r] = 0.f; }
    for (int k = lane * VEC; k < Hp; k += 64 * VEC) {
      float wv[VEC];
      if constexpr (VEC == 2) { const float2 t2 = ldw2(w, k); wv[0] = t2.x; wv[1] = t2.y; }
      else wv[0] = ldw(w, k);
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[r] = fmaf(wv[q], htop[(size_t)ub[r] * Hp + k + q], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      acc[r] = wave_sum(acc[r]);
      if (lane == r && r0 + r < n_emit) c.p[(size_t)ub[r] * m.Hj + j] = acc[r] + m.b_pred[j];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Low-latency prediction network for a handful of emitting utterances (bf16 models).  The cost of
// a step at batch 1 is not arithmetic but dependent memory round trips, about a microsecond each
// on this chip, so these kernels are built to need two: first the emit list (count, utterance ids
// and tokens, read side by side), then everything else at once: each lane's share of the weight
// rows as 16-byte loads, the input / hidden vectors, the cell state.
constexpr int kSmallKSteps = 4;   // lanes cover K in steps of 512: K = in + Hp <= 2048

__device__ __forceinline__ void unpack_bf16x8(const u32x4 &v, float (&o)[8]) {
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
  o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xFFFF0000u);
  o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

template <int R>
__global__ __launch_bounds__(256) void lstm_small_kernel(ModelDev m, CallDev c, int layer) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int unit = blockIdx.x * 4 + wave;
  const int Hp = m.Hp, in = layer == 0 ? 0 : Hp, K = in + Hp;   // layer 0: input sums come from emb_gates
  const size_t lofs = (size_t)layer * c.B * Hp;
  // round trip 1: the emit list (entries past n_emit hold valid, stale ids: harmless to read)
  const int n_emit = *c.n_emit;
  int ub0[R], tok0[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int idx = r < c.B ? r : c.B - 1;
    ub0[r] = c.emit_idx[idx];
    tok0[r] = c.emit_list_tok[idx];
  }
  // weights do not depend on the list: they go out in the same breath
  const bf16_t *w = reinterpret_cast<const bf16_t *>(m.w_cat[layer]) + (size_t)(unit < Hp ? unit : 0) * 4 * K;
  u32x4 wv[4][kSmallKSteps];
#pragma unroll
  for (int s2 = 0; s2 < kSmallKSteps; ++s2) {
    const int k = lane * 8 + 512 * s2;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      wv[g][s2] = u32x4{0u, 0u, 0u, 0u};
      if (k < K) wv[g][s2] = *reinterpret_cast<const u32x4 *>(w + (size_t)g * K + k);
    }
  }
  if (n_emit == 0 || unit >= Hp) return;
  const float *bias = m.b_cat[layer] + unit * 4;
  for (int r0 = 0; r0 < n_emit; r0 += R) {
    int ub[R], tok[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (r0 == 0) { ub[r] = ub0[r]; tok[r] = tok0[r]; }
      else { const int idx = min(r0 + r, n_emit - 1); ub[r] = c.emit_idx[idx]; tok[r] = c.emit_list_tok[idx]; }
    }
    // round trip 2: inputs, previous hidden vectors, cell state, the label's input gate sums
    float xv[R][kSmallKSteps][8];
    float cprev[R];
    float4 add[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const size_t si = lofs + (size_t)ub[r] * Hp;
      cprev[r] = c.c[si + unit];
      add[r] = *reinterpret_cast<const float4 *>(layer == 0 ? m.emb_gates + (size_t)tok[r] * 4 * Hp + unit * 4 : bias);
#pragma unroll
      for (int s2 = 0; s2 < kSmallKSteps; ++s2) {
        const int k = lane * 8 + 512 * s2;
#pragma unroll
        for (int q = 0; q < 8; ++q) xv[r][s2][q] = 0.f;
        if (k < in) {
          const f32x4 *src = reinterpret_cast<const f32x4 *>(c.hn + si - (size_t)c.B * Hp + k);
          const f32x4 a = src[0], b2 = src[1];
          xv[r][s2][0] = a.x; xv[r][s2][1] = a.y; xv[r][s2][2] = a.z; xv[r][s2][3] = a.w;
          xv[r][s2][4] = b2.x; xv[r][s2][5] = b2.y; xv[r][s2][6] = b2.z; xv[r][s2][7] = b2.w;
        } else if (k < K) {
          const f32x4 *src = reinterpret_cast<const f32x4 *>(c.h + si + (k - in));
          const f32x4 a = src[0], b2 = src[1];
          xv[r][s2][0] = a.x; xv[r][s2][1] = a.y; xv[r][s2][2] = a.z; xv[r][s2][3] = a.w;
          xv[r][s2][4] = b2.x; xv[r][s2][5] = b2.y; xv[r][s2][6] = b2.z; xv[r][s2][7] = b2.w;
        }
      }
    }
    float acc[4][R];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int r = 0; r < R; ++r) acc[g][r] = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < kSmallKSteps; ++s2)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float wf[8];
        unpack_bf16x8(wv[g][s2], wf);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[g][r] = fmaf(wf[q], xv[r][s2][q], acc[g][r]);
      }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g][r] = wave_sum(acc[g][r]);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (lane == r && r0 + r < n_emit) {
        const size_t si = lofs + (size_t)ub[r] * Hp + unit;
        const float ig = 1.f / (1.f + expf(-(acc[0][r] + add[r].x)));
        const float fg = 1.f / (1.f + expf(-(acc[1][r] + add[r].y)));
        const float gg = tanhf(acc[2][r] + add[r].z);
        const float og = 1.f / (1.f + expf(-(acc[3][r] + add[r].w)));
        const float cn = fg * cprev[r] + ig * gg;
        c.c[si] = cn;
        c.hn[si] = og * tanhf(cn);
      }
    }
  }
}

template <int R>
__global__ __launch_bounds__(256) void pred_small_kernel(ModelDev m, CallDev c) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int Hp = m.Hp, j = blockIdx.x * 4 + wave;
  const int n_emit = *c.n_emit;
  int ub0[R];
#pragma unroll
  for (int r = 0; r < R; ++r) ub0[r] = c.emit_idx[r < c.B ? r : c.B - 1];
  const bf16_t *w = reinterpret_cast<const bf16_t *>(m.w_pred) + (size_t)(j < m.Hj ? j : 0) * Hp;
  u32x4 wv[kSmallKSteps];
#pragma unroll
  for (int s2 = 0; s2 < kSmallKSteps; ++s2) {
    const int k = lane * 8 + 512 * s2;
    wv[s2] = u32x4{0u, 0u, 0u, 0u};
    if (k < Hp) wv[s2] = *reinterpret_cast<const u32x4 *>(w + k);
  }
  if (n_emit == 0) return;
  {  // commit the new hidden vectors: every layer has read the old ones by now
    const size_t total = (size_t)m.L * n_emit * Hp;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
      const int k = (int)(i % Hp);
      const size_t q = i / Hp;
      const int r = (int)(q % n_emit), l = (int)(q / n_emit);
      const size_t si = ((size_t)l * c.B + c.emit_idx[r]) * Hp + k;
      c.h[si] = c.hn[si];
    }
  }
  if (j >= m.Hj) return;
  const float *htop = c.hn + (size_t)(m.L - 1) * c.B * Hp;
  const float bias = m.b_pred[j];
  for (int r0 = 0; r0 < n_emit; r0 += R) {
    float acc[R];
    int ub[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      ub[r] = r0 == 0 ? ub0[r] : c.emit_idx[min(r0 + r, n_emit - 1)];
      acc[r] = 0.f;
    }
#pragma unroll
    for (int s2 = 0; s2 < kSmallKSteps; ++s2) {
      const int k = lane * 8 + 512 * s2;
      float wf[8];
      unpack_bf16x8(wv[s2], wf);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (k < Hp) {
          const f32x4 *src = reinterpret_cast<const f32x4 *>(htop + (size_t)ub[r] * Hp + k);
          const f32x4 a = src[0], b2 = src[1];
          acc[r] = fmaf(wf[0], a.x, acc[r]); acc[r] = fmaf(wf[1], a.y, acc[r]); acc[r] = fmaf(wf[2], a.z, acc[r]);
          acc[r] = fmaf(wf[3], a.w, acc[r]); acc[r] = fmaf(wf[4], b2.x, acc[r]); acc[r] = fmaf(wf[5], b2.y, acc[r]);
          acc[r] = fmaf(wf[6], b2.z, acc[r]); acc[r] = fmaf(wf[7], b2.w, acc[r]);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      acc[r] = wave_sum(acc[r]);
      if (lane == r && r0 + r < n_emit) c.p[(size_t)ub[r] * m.Hj + j] = acc[r] + bias;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The prediction network for large batches on the direct-to-LDS MFMA tile core.  The activations
// are fp32 values carried as bf16 hi + lo (hi = RNE(x), lo = RNE(x - hi): relative error 2^-17,
// the size of fp32 accumulation noise over these K); products with the bf16 weights are exact and
// the accumulation is fp32.  The split costs rows, not K.  Hidden vectors are kept in memory
// already split (hb_*), so the GEMM operands are plain bf16 rows that the loads can fetch without
// a conversion pass; rows are gathered through the
// emit list by giving every lane its own source address.  A tile's first R rows are the hi parts
// of R utterances, the next R rows their lo parts; K runs over [x | h_prev].
template <class Cfg>
struct PredRows {
  const bf16_t *px[Cfg::LPW];   // x part at K = 0 (embedding row, or hi/lo of the layer below, or zeros)
  const bf16_t *ph[Cfg::LPW];   // h part at K = in
  int xstep[Cfg::LPW];          // 1: advance with K; 0: the shared zero row
  int kin;                      // K steps of the x part
  __device__ __forceinline__ const bf16_t *operator()(int i, int, int, int kt, int BK) const {
    return kt < kin ? px[i] + kt * BK * xstep[i] : ph[i] + (kt - kin) * BK;
  }
};

// pre = 0: the whole step of a layer, [x | h_prev] against [w_ih | w_hh]; new hidden vectors go to hbn_*.
// pre = 1 (layers above the first, c.rec in use): only the input half, x = the layer below's new
// vector, on top of the recurrent sums in c.rec; nobody reads this layer's old vector any more, so the
// new one is written in place (hb_*).
// pre = 2 (CallDev::slot_rows; layers above the first): as pre = 1, with the rows taken by slot.  Row a of the
// launch is the a-th active utterance of the iteration (parity: which half of the slot table), its input
// vector the layer below's row a of hbn_*, whether that utterance emitted or not; res_aux[a] says which
// utterance it is and whether it steps.  Nothing about the rows' addresses depends on a load, so the
// operands are asked for first and the slot's data travel in the same round trip.  The new vector goes to
// row a of this layer in hbn_* (and in place to hb_*).
template <class Cfg>
__device__ __forceinline__ void lstm_layer_slot_rows(const ModelDev &m, const CallDev &c, int layer, int parity, unsigned char *smem_raw) {
  constexpr int R = Cfg::BM / 2, UB = Cfg::BN / 4, TS = Cfg::BN + 4;
  const int row0 = blockIdx.y * R, n0 = blockIdx.x * Cfg::BN;
  const int Hp = m.Hp, in = Hp, K = in + Hp;
  const size_t lofs = (size_t)layer * c.B * Hp;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  PredRows<Cfg> rows;
  rows.kin = in / Cfg::BK;
#pragma unroll
  for (int i = 0; i < Cfg::LPW; ++i) {
    const int row = (wave * Cfg::LPW + i) * Cfg::RPI + lane / Cfg::CPR;
    const int chunk = (lane % Cfg::CPR) ^ lds_swizzle<Cfg::CPR>(row);
    rows.px[i] = c.hb_zero; rows.ph[i] = c.hb_zero; rows.xstep[i] = 0;
    if (row < Cfg::BM) {
      const int part = row >= R, slot = min(row0 + (part ? row - R : row), c.B - 1);
      rows.px[i] = (part ? c.hbn_lo : c.hbn_hi) + lofs - (size_t)c.B * Hp + (size_t)slot * Hp + chunk * 8;
      rows.xstep[i] = 1;
    }
  }
  f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
  constexpr int EPI = (R * UB + Cfg::NT - 1) / Cfg::NT;   // (row, unit) pairs per thread in the epilogue
  int ub_e[EPI], tok_e[EPI];
  float c_prev[EPI];
  float4 add_e[EPI], rec_e[EPI];
  bool drop = false;
  const float *bias = m.b_cat_t[layer] + n0;
  // asked for ahead of the operand stages, and not waited for before them (loads return in order: what is
  // older than the stages does not disturb the tile core's counting of its own loads)
  const int na = c.n_active[parity];
  const int *slot_ub = reinterpret_cast<const int *>(c.res_aux);   // per slot: the utterance if it steps, else -1
  int info[EPI];
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    info[q] = slot_ub[min(row0 + min((tid + q * Cfg::NT) / UB, R - 1), c.B - 1)];   // slots past the count: stale, not used
    const int u = (tid + q * Cfg::NT) % UB;
    add_e[q] = make_float4(bias[u], bias[UB + u], bias[2 * UB + u], bias[3 * UB + u]);
  }
  __builtin_amdgcn_sched_barrier(0);
  auto slot_data = [&]() {
    drop = row0 >= na;
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
      const bool live = row0 + min((tid + q * Cfg::NT) / UB, R - 1) < na;
      tok_e[q] = live ? info[q] : -1;   // >= 0: steps
      ub_e[q] = tok_e[q] >= 0 ? tok_e[q] : 0;
    }
    if (drop) return;
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
      const int u = (tid + q * Cfg::NT) % UB;
      c_prev[q] = 0.f;
      rec_e[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (tok_e[q] >= 0) {   // requested here, looked at in the epilogue
        c_prev[q] = c.c[lofs + (size_t)ub_e[q] * Hp + (n0 >> 2) + u];
        rec_e[q] = *reinterpret_cast<const float4 *>(c.rec + ((size_t)layer * c.B + ub_e[q]) * 4 * Hp + n0 + 4 * u);
      }
    }
  };
  gemm_mainloop_dma_src<Cfg>(rows, reinterpret_cast<const bf16_t *>(m.w_cat_t[layer]) + (size_t)n0 * K, in, smem_raw, acc, slot_data,
                             K, &drop);
  if (drop) return;
  __syncthreads();   // every wave is done with the ring: reuse it for the gate tile
  float *tile = reinterpret_cast<float *>(smem_raw);
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        tile[(wm * Cfg::WM + acc_row(mi, r, lane)) * TS + wn * Cfg::WN + ni * 32 + (lane & 31)] = acc[mi][ni][r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    const int idx = tid + q * Cfg::NT;
    const int r = idx / UB, u = idx - r * UB;
    if (idx >= R * UB || tok_e[q] < 0) continue;
    const float *hi = tile + r * TS + u, *lo = tile + (R + r) * TS + u;
    const float gi = hi[0] + lo[0] + (add_e[q].x + rec_e[q].x);
    const float gf = hi[UB] + lo[UB] + (add_e[q].y + rec_e[q].y);
    const float gg = hi[2 * UB] + lo[2 * UB] + (add_e[q].z + rec_e[q].z);
    const float go = hi[3 * UB] + lo[3 * UB] + (add_e[q].w + rec_e[q].w);
    const size_t si = lofs + (size_t)ub_e[q] * Hp + (n0 >> 2) + u;
    const float ig = 1.f / (1.f + expf(-gi)), fg = 1.f / (1.f + expf(-gf));
    const float og = 1.f / (1.f + expf(-go));
    const float cn = fg * c_prev[q] + ig * tanhf(gg);
    c.c[si] = cn;
    const float hv = og * tanhf(cn);
    store_hi_lo(c.hb_hi, c.hb_lo, si, hv);
    store_hi_lo(c.hbn_hi, c.hbn_lo, lofs + (size_t)(row0 + r) * Hp + (n0 >> 2) + u, hv);
  }
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) void lstm_layer_dma_kernel(ModelDev m, CallDev c, int layer, int pre, int parity) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  if (pre == 2) {
    lstm_layer_slot_rows<Cfg>(m, c, layer, parity, smem_raw);
    return;
  }
  constexpr int R = Cfg::BM / 2, UB = Cfg::BN / 4, TS = Cfg::BN + 4;
  // grid = (column tiles, row tiles): workgroups with consecutive ids share the row tile, and the
  // row tiles of one column tile land on the same XCD (id mod 8), which then fetches that slice of
  // the weights once
  const int row0 = blockIdx.y * R;
  const int n0 = blockIdx.x * Cfg::BN;
  const int Hp = m.Hp, in = layer == 0 ? 0 : Hp, K = in + Hp;   // layer 0: input sums come from emb_gates
  const size_t lofs = (size_t)layer * c.B * Hp;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // round trip 1: the emit count and the list entries this thread will need (entries past the
  // count hold stale but valid ids, so the reads need not wait for the count)
  const int n_emit = *c.n_emit;
  int ub_row[Cfg::LPW];
#pragma unroll
  for (int i = 0; i < Cfg::LPW; ++i) {
    const int row = (wave * Cfg::LPW + i) * Cfg::RPI + lane / Cfg::CPR;
    const int r = row < Cfg::BM ? (row >= R ? row - R : row) : 0;
    ub_row[i] = c.emit_idx[min(row0 + r, c.B - 1)];
  }
  constexpr int EPI = (R * UB + Cfg::NT - 1) / Cfg::NT;   // (utterance, unit) pairs per thread in the epilogue
  int ub_e[EPI], tok_e[EPI];
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    const int r = min((tid + q * Cfg::NT) / UB, R - 1);
    ub_e[q] = c.emit_idx[min(row0 + r, c.B - 1)];
    tok_e[q] = c.emit_list_tok[min(row0 + r, c.B - 1)];
  }
  if (row0 >= n_emit) return;
  // round trip 2, requested ahead of the tile core's loads and used after it: cell state and the
  // additive term (bias, or the label's row of input gate sums) of this thread's pairs
  const float *bias = m.b_cat_t[layer] + n0;
  float c_prev[EPI];
  float4 add_e[EPI], rec_e[EPI];   // both only looked at in the epilogue: no wait for them ahead of the tile core
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    const int idx = tid + q * Cfg::NT, u = idx % UB;
    c_prev[q] = c.c[lofs + (size_t)ub_e[q] * Hp + (n0 >> 2) + u];
    add_e[q] = make_float4(bias[u], bias[UB + u], bias[2 * UB + u], bias[3 * UB + u]);
    if (layer == 0) add_e[q] = *reinterpret_cast<const float4 *>(m.emb_gates + (size_t)tok_e[q] * 4 * Hp + n0 + 4 * u);
    rec_e[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (pre) rec_e[q] = *reinterpret_cast<const float4 *>(c.rec + ((size_t)layer * c.B + ub_e[q]) * 4 * Hp + n0 + 4 * u);
  }
  __builtin_amdgcn_sched_barrier(0);   // these requests stay ahead of the tile core's
  PredRows<Cfg> rows;
  rows.kin = in / Cfg::BK;
#pragma unroll
  for (int i = 0; i < Cfg::LPW; ++i) {
    const int row = (wave * Cfg::LPW + i) * Cfg::RPI + lane / Cfg::CPR;
    const int chunk = (lane % Cfg::CPR) ^ lds_swizzle<Cfg::CPR>(row);
    rows.px[i] = c.hb_zero; rows.ph[i] = c.hb_zero; rows.xstep[i] = 0;
    if (row < Cfg::BM) {
      const int part = row >= R;
      const size_t si = lofs + (size_t)ub_row[i] * Hp;
      if (layer > 0) {
        rows.px[i] = (pre ? (part ? c.hb_lo : c.hb_hi) : (part ? c.hbn_lo : c.hbn_hi)) + si - (size_t)c.B * Hp + chunk * 8;
        rows.xstep[i] = 1;
      }
      rows.ph[i] = (part ? c.hb_lo : c.hb_hi) + si + chunk * 8;
    }
  }
  f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
  gemm_mainloop_dma_src<Cfg>(rows, reinterpret_cast<const bf16_t *>(m.w_cat_t[layer]) + (size_t)n0 * K, pre ? in : K, smem_raw,
                             acc, NoInit{}, K);
  __syncthreads();   // every wave is done with the ring: reuse it for the gate tile

  float *tile = reinterpret_cast<float *>(smem_raw);
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        tile[(wm * Cfg::WM + acc_row(mi, r, lane)) * TS + wn * Cfg::WN + ni * 32 + (lane & 31)] = acc[mi][ni][r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    const int idx = tid + q * Cfg::NT;
    const int r = idx / UB, u = idx - r * UB;
    if (idx >= R * UB || row0 + r >= n_emit) continue;
    const float *hi = tile + r * TS + u, *lo = tile + (R + r) * TS + u;
    const float gi = hi[0] + lo[0] + (add_e[q].x + rec_e[q].x);
    const float gf = hi[UB] + lo[UB] + (add_e[q].y + rec_e[q].y);
    const float gg = hi[2 * UB] + lo[2 * UB] + (add_e[q].z + rec_e[q].z);
    const float go = hi[3 * UB] + lo[3 * UB] + (add_e[q].w + rec_e[q].w);
    const size_t si = lofs + (size_t)ub_e[q] * Hp + (n0 >> 2) + u;
    const float ig = 1.f / (1.f + expf(-gi)), fg = 1.f / (1.f + expf(-gf));
    const float og = 1.f / (1.f + expf(-go));
    const float cn = fg * c_prev[q] + ig * tanhf(gg);
    c.c[si] = cn;
    if (pre) store_hi_lo(c.hb_hi, c.hb_lo, si, og * tanhf(cn));
    else store_hi_lo(c.hbn_hi, c.hbn_lo, si, og * tanhf(cn));
  }
}

// One tile of c.rec: the recurrent gate sums w_hh . h of `layer` for the R utterances from row0 of
// the emit list and the tile's 64 gate rows, from the hidden vectors in hb_* (already the new ones).
template <class Cfg>
__device__ __forceinline__ void lstm_rec_tile(const ModelDev &m, const CallDev &c, int layer, int n0, int row0, int n_emit,
                                              const int (&ub_row)[Cfg::LPW], unsigned char *smem_raw) {
  constexpr int R = Cfg::BM / 2, UB = Cfg::BN / 4, TS = Cfg::BN + 4;
  const int Hp = m.Hp, in = layer == 0 ? 0 : Hp, K = in + Hp;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the utterances of this thread's rows in the epilogue, requested ahead of the tile core
  constexpr int EPI = (R * UB + Cfg::NT - 1) / Cfg::NT;
  int ub_e[EPI];
#pragma unroll
  for (int q = 0; q < EPI; ++q) ub_e[q] = c.emit_idx[min(row0 + min((tid + q * Cfg::NT) / UB, R - 1), c.B - 1)];
  PredRows<Cfg> rows;
  rows.kin = 0;
#pragma unroll
  for (int i = 0; i < Cfg::LPW; ++i) {
    const int row = (wave * Cfg::LPW + i) * Cfg::RPI + lane / Cfg::CPR;
    const int chunk = (lane % Cfg::CPR) ^ lds_swizzle<Cfg::CPR>(row);
    rows.px[i] = c.hb_zero; rows.ph[i] = c.hb_zero; rows.xstep[i] = 0;
    if (row < Cfg::BM) rows.ph[i] = (row >= R ? c.hb_lo : c.hb_hi) + ((size_t)layer * c.B + ub_row[i]) * Hp + chunk * 8;
  }
  f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
  // the h columns of the tile's rows of [w_ih | w_hh]
  gemm_mainloop_dma_src<Cfg>(rows, reinterpret_cast<const bf16_t *>(m.w_cat_t[layer]) + (size_t)n0 * K + in, Hp, smem_raw, acc,
                             NoInit{}, K);
  __syncthreads();
  float *tile = reinterpret_cast<float *>(smem_raw);
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        tile[(wm * Cfg::WM + acc_row(mi, r, lane)) * TS + wn * Cfg::WN + ni * 32 + (lane & 31)] = acc[mi][ni][r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    const int idx = tid + q * Cfg::NT, r = idx / UB, u = idx - r * UB;
    if (idx >= R * UB || row0 + r >= n_emit) continue;
    const float *hi = tile + r * TS + u, *lo = tile + (R + r) * TS + u;
    const float4 g = make_float4(hi[0] + lo[0], hi[UB] + lo[UB], hi[2 * UB] + lo[2 * UB], hi[3 * UB] + lo[3 * UB]);
    *reinterpret_cast<float4 *>(c.rec + ((size_t)layer * c.B + ub_e[q]) * 4 * Hp + n0 + 4 * u) = g;
  }
}

// pre = 0: the projection of the new top-layer vectors in hbn_*, then the new vectors of all layers
// are committed to hb_*.  pre = 1 (c.rec in use): the new vectors are in hb_* already; column tiles
// from proj_tiles on do not project but renew c.rec, layer by layer, for the utterances that emitted.
template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) void pred_proj_dma_kernel(ModelDev m, CallDev c, int pre, int proj_tiles) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  constexpr int R = Cfg::BM / 2, TS = Cfg::BN + 4;
  const int Hp = m.Hp, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // grid = (column tiles, row tiles): workgroups with consecutive ids share the row tile, and the
  // row tiles of one column tile land on the same XCD (id mod 8), which then fetches that slice of
  // the weights once
  const int row0 = blockIdx.y * R;
  const int n0 = blockIdx.x * Cfg::BN;
  // one round trip for the emit count and the list entries (entries past the count are stale but valid)
  const int n_emit = *c.n_emit;
  int ub_row[Cfg::LPW];
#pragma unroll
  for (int i = 0; i < Cfg::LPW; ++i) {
    const int row = (wave * Cfg::LPW + i) * Cfg::RPI + lane / Cfg::CPR;
    const int r = row < Cfg::BM ? (row >= R ? row - R : row) : 0;
    ub_row[i] = c.emit_idx[min(row0 + r, c.B - 1)];
  }
  if (n_emit == 0) return;
  if ((int)blockIdx.x >= proj_tiles) {
    if (row0 >= n_emit) return;
    const int tiles_per_layer = 4 * Hp / Cfg::BN, ct = (int)blockIdx.x - proj_tiles;
    lstm_rec_tile<Cfg>(m, c, ct / tiles_per_layer, (ct % tiles_per_layer) * Cfg::BN, row0, n_emit, ub_row, smem_raw);
    return;
  }
  if (row0 < n_emit) {
    // epilogue inputs, requested ahead of the tile core: this thread's column bias and the utterances of
    // its rows (a thread keeps one column and every (NT / BN)-th row)
    static_assert(Cfg::NT % Cfg::BN == 0 && R % (Cfg::NT / Cfg::BN) == 0, "epilogue mapping");
    constexpr int RSTEP = Cfg::NT / Cfg::BN, RPT = R / RSTEP;
    const int ecol = tid % Cfg::BN, erow = tid / Cfg::BN;
    const float bias_e = n0 + ecol < m.Hj ? m.b_pred[n0 + ecol] : 0.f;
    int ub_e[RPT];
#pragma unroll
    for (int q = 0; q < RPT; ++q) ub_e[q] = c.emit_idx[min(row0 + erow + q * RSTEP, c.B - 1)];
    const size_t top = (size_t)(m.L - 1) * c.B * Hp;
    PredRows<Cfg> rows;
    rows.kin = 0;
#pragma unroll
    for (int i = 0; i < Cfg::LPW; ++i) {
      const int row = (wave * Cfg::LPW + i) * Cfg::RPI + lane / Cfg::CPR;
      const int chunk = (lane % Cfg::CPR) ^ lds_swizzle<Cfg::CPR>(row);
      rows.px[i] = c.hb_zero; rows.ph[i] = c.hb_zero; rows.xstep[i] = 0;
      if (row < Cfg::BM)
        rows.ph[i] = (pre ? (row >= R ? c.hb_lo : c.hb_hi) : (row >= R ? c.hbn_lo : c.hbn_hi)) + top + (size_t)ub_row[i] * Hp + chunk * 8;
    }
    f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
    gemm_mainloop_dma_src<Cfg>(rows, reinterpret_cast<const bf16_t *>(m.w_pred) + (size_t)n0 * Hp, Hp, smem_raw, acc);
    __syncthreads();
    float *tile = reinterpret_cast<float *>(smem_raw);
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          tile[(wm * Cfg::WM + acc_row(mi, r, lane)) * TS + wn * Cfg::WN + ni * 32 + (lane & 31)] = acc[mi][ni][r];
    __syncthreads();
#pragma unroll
    for (int q = 0; q < RPT; ++q) {
      const int r = erow + q * RSTEP;
      if (row0 + r >= n_emit || n0 + ecol >= m.Hj) continue;
      c.p[(size_t)ub_e[q] * m.Hj + n0 + ecol] = tile[r * TS + ecol] + tile[(R + r) * TS + ecol] + bias_e;
    }
  }
  if (!pre) {  // commit the new hidden vectors (hi and lo): every layer has read the old ones by now.  Last,
     // so that the copy's round trips do not delay the projection.
    const size_t total = (size_t)m.L * n_emit * Hp;
    const size_t nthreads = (size_t)gridDim.x * gridDim.y * Cfg::NT;
    for (size_t i = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * Cfg::NT + tid; i < total; i += nthreads) {
      const int k = (int)(i % Hp);
      const size_t q = i / Hp;
      const int r = (int)(q % n_emit), l = (int)(q / n_emit);
      const size_t si = ((size_t)l * c.B + c.emit_idx[r]) * Hp + k;
      c.hb_hi[si] = c.hbn_hi[si];
      c.hb_lo[si] = c.hbn_lo[si];
    }
  }
}

}  // namespace wind
