// Scoring step of WIND beam search (section "A Novel Beam-search Algorithm for WIND": Eq. 1 and the
// step of Algorithm 3 that scores a window) for Bh hypotheses that sit on the same frame:
//   logits[b, t, :] = joiner(enc_window[t], dec_out[b])            t < n
//   log P'(v, t)    = log softmax(logits[b, t])[v] + sum_{t' < t} log softmax(logits[b, t'])[blank]
//   log P'(blank, n-1) = sum_{t' < n} log softmax(logits[b, t'])[blank];   P'(blank, t < n-1) = 0
//   the K best (label, jump) pairs of every hypothesis under P'
// Order among equal scores: earlier frame, then lower label.  The logits take the same route as in
// the greedy path (bf16 models: hidden vector rounded to bf16, bf16 MFMA, fp32 accumulation; fp32
// models: fp32 FMA; bf16 models on request: fp32 hidden vector split into two bf16 vectors, both
// through the MFMA pass); everything after them is fp32.
#pragma once
#include "wind_kernels.h"

namespace wind {

constexpr int kBeamMaxK = 32;
constexpr int kBeamMaxWindow = 64;

// Eight consecutive weights as floats: one 16-byte load for bf16 storage, two for fp32.
__device__ __forceinline__ void ldw8(const bf16_t *w, size_t i, float (&o)[8]) {
  unpack_bf16x8(*reinterpret_cast<const u32x4 *>(w + i), o);
}
__device__ __forceinline__ void ldw8(const float *w, size_t i, float (&o)[8]) {
  const float4 a = *reinterpret_cast<const float4 *>(w + i), b = *reinterpret_cast<const float4 *>(w + i + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

// Which table row (or label) belongs to entry b of a launch: b itself, an entry of a device list, or
// one of up to 32 values carried in the launch's own arguments (no copy to the device needed).
constexpr int kBeamInline = 32;
struct BeamIndex {
  const int *ptr;
  int n_inline;
  int inl[kBeamInline];
  __device__ __forceinline__ int operator()(int b) const { return ptr ? ptr[b] : (n_inline ? inl[b] : b); }
};

// out[r, j] = bias[j] + sum_k w[j, k] * x[r, k]: one wave per output j and group of R rows, so that a
// weight row is read once per group.  ROUND_X rounds x to bf16 first (what the encoder projection
// of a bf16 model does with its input).  grid = (ceil(n_out / 4), ceil(rows / R)).
template <class WT, bool ROUND_X, int R>
__global__ __launch_bounds__(256) void beam_linear_kernel(const WT *w, const float *bias, const float *x, float *out,
                                                          int rows, int n_out, int K) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 4 + wave, r0 = blockIdx.y * R;
  if (j >= n_out) return;
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  for (int k = lane; k < K; k += 64) {
    const float wv = ldw(w, (size_t)j * K + k);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float xv = x[(size_t)min(r0 + r, rows - 1) * K + k];
      if (ROUND_X) xv = bf16_bits_to_f32(f32_to_bf16_bits(xv));
      acc[r] = fmaf(wv, xv, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float tot = wave_sum(acc[r]);
    if (lane == 0 && r0 + r < rows) out[(size_t)(r0 + r) * n_out + j] = tot + bias[j];
  }
}

// Row (b, t) of the joiner's hidden layer, relu(e[t] + p[row pi(b)]), as bf16 for the MFMA pass.  With
// z_lo the remainder after rounding is stored as a second bf16 vector (see joint_mfma_store_kernel).
__global__ __launch_bounds__(256) void beam_hidden_kernel(const float *e, const float *p, BeamIndex pi, bf16_t *z,
                                                          bf16_t *z_lo, int n, int Hj) {
  const int row = blockIdx.x, b = row / n, t = row - b * n;
  const float *pr = p + (size_t)pi(b) * Hj;
  for (int k = threadIdx.x; k < Hj; k += 256) {
    const float v = fmaxf(e[(size_t)t * Hj + k] + pr[k], 0.f);
    const unsigned short hi = f32_to_bf16_bits(v);
    z[(size_t)row * Hj + k] = (bf16_t)hi;
    if (z_lo) z_lo[(size_t)row * Hj + k] = (bf16_t)f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
  }
}

// Logits of row (b, t) by fp32 FMA on an fp32 hidden vector, one workgroup per row: fp32 models, and
// bf16 models when the caller asks for decisions that do not depend on rounding the hidden vector.
template <class WT>
__global__ __launch_bounds__(256) void beam_logits_kernel(ModelDev m, const float *e, const float *p, BeamIndex pi, int n,
                                                          float *logits) {
  extern __shared__ float zs[];
  const int row = blockIdx.x, b = row / n, t = row - b * n;
  const float *pr = p + (size_t)pi(b) * m.Hj;
  for (int k = threadIdx.x; k < m.Hj; k += 256) zs[k] = fmaxf(e[(size_t)t * m.Hj + k] + pr[k], 0.f);
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const WT *w = reinterpret_cast<const WT *>(m.w_out);
  for (int v = wave; v <= m.V; v += 4) {
    float a = 0.f;
    for (int k = lane; k < m.Hj; k += 64) a = fmaf(ldw(w, (size_t)v * m.Hj + k), zs[k], a);
    a = wave_sum(a);
    if (lane == 0) logits[(size_t)row * (m.V + 1) + v] = a + m.b_out[v];
  }
}

// Few rows (bf16 models, Hj <= 1024): logits of one block of 32 rows x 32 columns per workgroup.  The
// workgroup builds its hidden rows relu(e[t] + p[pi(b)]) in LDS itself (no separate pass, no trip
// through memory), its four waves split K and read their W_out fragments straight from memory into
// MFMA operands, all loads in flight at once; the four partial tiles are added through LDS.  With
// `split` the remainder of the bf16 rounding is kept as a second vector and multiplied as well.
// grid = (ceil((V+1) / 32), ceil(rows / 32)); dynamic LDS = (split ? 2 : 1) * 32 * (Hj + 8) * 2 bytes,
// at least 16 KB.
constexpr int kBeamTinyMaxHj = 1024;
constexpr int kBeamTinyMaxRows = 256;
__global__ __launch_bounds__(256) void beam_logits_tiny_kernel(ModelDev m, const float *e, const float *p, BeamIndex pi,
                                                               int n, int rows, int split, float *logits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Hj = m.Hj, V1 = m.V + 1;
  const int n0 = blockIdx.x * 32, row0 = blockIdx.y * 32;
  const int nk = Hj / 64, k0 = wave * (Hj / 4);   // this wave's K steps of 16 and where they start
  const bf16_t *wrow = reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)(n0 + (lane & 31)) * Hj + k0 + (lane >> 5) * 8;
  constexpr int kMaxSteps = kBeamTinyMaxHj / 64;
  bf16x8 bfrag[kMaxSteps];
#pragma unroll
  for (int i = 0; i < kMaxSteps; ++i)
    if (i < nk) bfrag[i] = *reinterpret_cast<const bf16x8 *>(wrow + i * 16);
  const int zstride = Hj + 8;   // bf16 elements; an odd number of 16-byte units, so fragment reads spread over the banks
  bf16_t *zs = reinterpret_cast<bf16_t *>(smem_raw), *zl = zs + 32 * zstride;
  // hidden rows: a wave takes rows wave, wave + 4, ...
  for (int r = wave; r < 32; r += 4) {
    const int row = row0 + r;
    const bool valid = row < rows;
    const int b = valid ? row / n : 0, t = valid ? row - b * n : 0;
    const float *er = e + (size_t)t * Hj, *pr = p + (size_t)pi(b) * Hj;
    for (int k = lane * 4; k < Hj; k += 256) {
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (valid) {
        const float4 ev = *reinterpret_cast<const float4 *>(er + k), pv = *reinterpret_cast<const float4 *>(pr + k);
        x = make_float4(fmaxf(ev.x + pv.x, 0.f), fmaxf(ev.y + pv.y, 0.f), fmaxf(ev.z + pv.z, 0.f), fmaxf(ev.w + pv.w, 0.f));
      }
      const unsigned h01 = pack_bf16x2(x.x, x.y), h23 = pack_bf16x2(x.z, x.w);
      *reinterpret_cast<uint2 *>(zs + (size_t)r * zstride + k) = make_uint2(h01, h23);
      if (split) {
        const float r0 = x.x - __uint_as_float(h01 << 16), r1 = x.y - __uint_as_float(h01 & 0xFFFF0000u);
        const float r2 = x.z - __uint_as_float(h23 << 16), r3 = x.w - __uint_as_float(h23 & 0xFFFF0000u);
        *reinterpret_cast<uint2 *>(zl + (size_t)r * zstride + k) = make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
      }
    }
  }
  __syncthreads();
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const bf16_t *zrow = zs + (size_t)(lane & 31) * zstride + k0 + (lane >> 5) * 8;
#pragma unroll
  for (int i = 0; i < kMaxSteps; ++i) {
    if (i < nk) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(zrow + i * 16), bfrag[i], acc, 0, 0, 0);
      if (split)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(zrow + 32 * zstride + i * 16), bfrag[i],
                                                      acc, 0, 0, 0);
    }
  }
  __syncthreads();   // every wave is done with the hidden rows: their LDS now takes the partial tiles
  float *red = reinterpret_cast<float *>(smem_raw);   // [wave][r][lane]
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[r];
  __syncthreads();
  const int col = n0 + (lane & 31);
  if (col >= V1) return;
  const float bias = m.b_out[col];
#pragma unroll
  for (int q = 0; q < 4; ++q) {   // wave w adds up and stores accumulator registers 4w .. 4w+3
    const int r = wave * 4 + q;
    const float v = (red[r * 64 + lane] + red[(16 + r) * 64 + lane]) + (red[(32 + r) * 64 + lane] + red[(48 + r) * 64 + lane]);
    const int row = row0 + acc_row(0, r, lane);
    if (row < rows) logits[(size_t)row * V1 + col] = v + bias;
  }
}

// out[r] = log softmax(logits[r, :])[tok[r]]: one workgroup per row.
__global__ __launch_bounds__(256) void beam_token_logp_kernel(const float *logits, int V1, BeamIndex tok, float *out) {
  __shared__ float s_f[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *row = logits + (size_t)blockIdx.x * V1;
  float mx = -INFINITY;
  for (int v = tid; v < V1; v += 256) mx = fmaxf(mx, row[v]);
  mx = wave_max_f32(mx);
  if (lane == 0) s_f[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
  __syncthreads();
  float sum = 0.f;
  for (int v = tid; v < V1; v += 256) sum += expf(row[v] - mx);
  sum = wave_sum(sum);
  if (lane == 0) s_f[wave] = sum;
  __syncthreads();
  if (tid == 0) out[blockIdx.x] = row[tok(blockIdx.x)] - (mx + logf((s_f[0] + s_f[1]) + (s_f[2] + s_f[3])));
}

// ---------------------------------------------------------------------------------------------
// Prediction network for the hypotheses of a beam search.  States live in a pool of slots,
// h and c as [slot][L][Hp], the projected output p as [slot][Hj]; a step reads the parent's slot
// and writes the child's, so that every label sequence the search has touched keeps its state.
// One wave per hidden unit, R rows at a time (a weight row is read once per group), fp32 FMA.
template <class WT, int R>
__global__ __launch_bounds__(256) void beam_lstm_layer_kernel(ModelDev m, float *h, float *c, int layer, int rows,
                                                              BeamIndex parent, BeamIndex child, BeamIndex tok) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int unit = blockIdx.x * 4 + wave;
  if (unit >= m.Hp) return;
  const int Hp = m.Hp, in = layer == 0 ? 0 : Hp, K = in + Hp;
  const size_t slot_sz = (size_t)m.L * Hp;
  const WT *w = reinterpret_cast<const WT *>(m.w_cat[layer]) + (size_t)unit * 4 * K;
  for (int r0 = 0; r0 < rows; r0 += R) {
    float acc[4][R];
    const float *xh[R], *hp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int rr = min(r0 + r, rows - 1);
      xh[r] = h + (size_t)child(rr) * slot_sz + (size_t)(layer > 0 ? layer - 1 : 0) * Hp;   // new h of the layer below
      hp[r] = h + (size_t)parent(rr) * slot_sz + (size_t)layer * Hp;
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g][r] = 0.f;
    }
    // lane r finishes row r: its additive term (layer 0: the label's row of emb_gates, which carries the
    // input sums and both biases) and the parent's cell value are requested here, ahead of the dot
    // products, so that they do not cost a round trip of their own at the end
    float4 addv = make_float4(0.f, 0.f, 0.f, 0.f);
    float cprev = 0.f;
    if (lane < R && r0 + lane < rows) {
      addv = *reinterpret_cast<const float4 *>(layer == 0 ? m.emb_gates + (size_t)tok(r0 + lane) * 4 * Hp + unit * 4
                                                          : m.b_cat[layer] + unit * 4);
      cprev = c[(size_t)parent(r0 + lane) * slot_sz + (size_t)layer * Hp + unit];
    }
    if ((Hp & 7) == 0) {
      // eight weights of each gate row and eight inputs per lane and step: 16- and 32-byte loads
      for (int k = lane * 8; k < K; k += 512) {
        float wv[4][8];
#pragma unroll
        for (int g = 0; g < 4; ++g) ldw8(w, (size_t)g * K + k, wv[g]);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float *xp = k < in ? xh[r] + k : hp[r] + (k - in);
          const float4 x0 = *reinterpret_cast<const float4 *>(xp), x1 = *reinterpret_cast<const float4 *>(xp + 4);
          const float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[g][r] = fmaf(wv[g][q], xv[q], acc[g][r]);
        }
      }
    } else {
      for (int k = lane; k < K; k += 64) {
        float wv[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) wv[g] = ldw(w, (size_t)g * K + k);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float xv = k < in ? xh[r][k] : hp[r][k - in];
#pragma unroll
          for (int g = 0; g < 4; ++g) acc[g][r] = fmaf(wv[g], xv, acc[g][r]);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g][r] = wave_sum(acc[g][r]);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (lane == r && r0 + r < rows) {
        const float ig = 1.f / (1.f + expf(-(acc[0][r] + addv.x)));
        const float fg = 1.f / (1.f + expf(-(acc[1][r] + addv.y)));
        const float gg = tanhf(acc[2][r] + addv.z);
        const float og = 1.f / (1.f + expf(-(acc[3][r] + addv.w)));
        const size_t co = (size_t)child(r0 + r) * slot_sz + (size_t)layer * Hp + unit;
        const float cn = fg * cprev + ig * gg;
        c[co] = cn;
        h[co] = og * tanhf(cn);
      }
    }
  }
}

// p[child] = W_pred h_top[child] + b_pred for the new hypotheses.
template <class WT, int R>
__global__ __launch_bounds__(256) void beam_pred_kernel(ModelDev m, const float *h, float *p, int rows, BeamIndex child) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 4 + wave;
  if (j >= m.Hj) return;
  const int Hp = m.Hp;
  const size_t slot_sz = (size_t)m.L * Hp;
  const WT *w = reinterpret_cast<const WT *>(m.w_pred) + (size_t)j * Hp;
  for (int r0 = 0; r0 < rows; r0 += R) {
    float acc[R];
    const float *ht[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      ht[r] = h + (size_t)child(min(r0 + r, rows - 1)) * slot_sz + (size_t)(m.L - 1) * Hp;
      acc[r] = 0.f;
    }
    if ((Hp & 7) == 0) {
      for (int k = lane * 8; k < Hp; k += 512) {
        float wv[8];
        ldw8(w, k, wv);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float4 x0 = *reinterpret_cast<const float4 *>(ht[r] + k), x1 = *reinterpret_cast<const float4 *>(ht[r] + k + 4);
          const float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[r] = fmaf(wv[q], xv[q], acc[r]);
        }
      }
    } else {
      for (int k = lane; k < Hp; k += 64) {
        const float wv = ldw(w, k);
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = fmaf(wv, ht[r][k], acc[r]);
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float tot = wave_sum(acc[r]);
      if (lane == 0 && r0 + r < rows) p[(size_t)child(r0 + r) * m.Hj + j] = tot + m.b_pred[j];
    }
  }
}

// (score, frame, label) ordering of Algorithm 3's top-K: a comes before b
__device__ __forceinline__ bool beam_before(float sa, int ka, float sb, int kb) {
  return sa > sb || (sa == sb && ka < kb);   // k = frame * (V+1) + label: earlier frame, then lower label
}

// The same ordering on a pair of unsigned words that compare like integers: hi = the score's bits
// mapped so that larger floats give larger integers, lo = ~key (smaller key = larger word).
__device__ __forceinline__ unsigned beam_order_bits(float s) {
  const unsigned u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float beam_score_of(unsigned hi) {
  return __uint_as_float((hi & 0x80000000u) ? (hi & 0x7FFFFFFFu) : ~hi);
}
// Largest (hi, lo) pair of the wave, in every lane.  The pair is compared as one 64-bit integer.  DPP
// row permutations inside the rows of 16, then the four row winners by v_readlane: no trip through
// the LDS crossbar.
__device__ __forceinline__ void wave_max_pair(unsigned &hi, unsigned &lo) {
  unsigned long long v = ((unsigned long long)hi << 32) | lo;
#define WIND_PAIR_STEP(CTRL)                                                                                   \
  {                                                                                                             \
    const unsigned oh = (unsigned)dpp_i32<CTRL>((int)(v >> 32)), ol = (unsigned)dpp_i32<CTRL>((int)(unsigned)v); \
    const unsigned long long o = ((unsigned long long)oh << 32) | ol;                                           \
    v = o > v ? o : v;                                                                                          \
  }
  WIND_PAIR_STEP(kDppRowMirror)
  WIND_PAIR_STEP(kDppRowHalfMirror)
  WIND_PAIR_STEP(kDppQuadXor2)
  WIND_PAIR_STEP(kDppQuadXor1)
#undef WIND_PAIR_STEP
#pragma unroll
  for (int row = 0; row < 64; row += 16) {
    const unsigned oh = (unsigned)__builtin_amdgcn_readlane((int)(v >> 32), row);
    const unsigned ol = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, row);
    const unsigned long long o = ((unsigned long long)oh << 32) | ol;
    v = o > v ? o : v;
  }
  hi = (unsigned)(v >> 32);
  lo = (unsigned)v;
}

// One workgroup per hypothesis.  Pass 1: log-sum-exp of every row, blank log-probabilities and their
// running sum.  Pass 2: every thread keeps the K best of the entries it visits, sorted, in
// registers (KMAX slots).  Then every wave merges its 64 lists by K rounds of "best head", and wave
// 0 merges the four results.
template <int KMAX>
__global__ __launch_bounds__(256) void beam_score_kernel(const float *logits, int n, int V, int K, int *out_labels,
                                                         int *out_jumps, float *out_scores) {
  __shared__ float s_lse[kBeamMaxWindow], s_blank[kBeamMaxWindow], s_run[kBeamMaxWindow + 1];
  __shared__ unsigned s_hi[4][KMAX], s_lo[4][KMAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, V1 = V + 1;
  const float *lg = logits + (size_t)blockIdx.x * n * V1;
  // ---- pass 1: a wave takes rows wave, wave + 4, ...; one sweep per row with a running maximum and a
  // running sum of exponentials.  Loads go out 32 at a time: these rows come from the memory side,
  // and one dependent round trip per element would cost far more than the arithmetic.
  for (int t = wave; t < n; t += 4) {
    const float *row = lg + (size_t)t * V1;
    float mx = -INFINITY, sum = 0.f;
    for (int v0 = lane; v0 < V1; v0 += 64 * 32) {
      float x[32];
#pragma unroll
      for (int i = 0; i < 32; ++i) x[i] = v0 + 64 * i < V1 ? row[v0 + 64 * i] : -INFINITY;
      float cm = x[0];
#pragma unroll
      for (int i = 1; i < 32; ++i) cm = fmaxf(cm, x[i]);
      const float nm = fmaxf(mx, cm);
      float cs = 0.f;
      if (nm > -INFINITY) {
#pragma unroll
        for (int i = 0; i < 32; ++i) cs += expf(x[i] - nm);
        sum = sum * expf(mx - nm) + cs;
        mx = nm;
      }
    }
    const float wm = wave_max_f32(mx);
    sum = wave_sum(mx > -INFINITY ? sum * expf(mx - wm) : 0.f);
    if (lane == 0) {
      const float lse = wm + logf(sum);
      s_lse[t] = lse;
      s_blank[t] = row[V] - lse;   // log P(blank | t)
    }
  }
  __syncthreads();
  if (tid == 0) {
    float run = 0.f;
    for (int t = 0; t < n; ++t) {
      s_run[t] = run;                                   // blanks on every frame before t
      run += s_blank[t];
    }
    s_run[n] = run;                                     // blanks on every frame of the window
  }
  __syncthreads();
  // ---- pass 2: thread-local K best as ordered (hi, lo) words, best first; slots >= K stay empty
  unsigned lh[KMAX], ll[KMAX];
#pragma unroll
  for (int i = 0; i < KMAX; ++i) { lh[i] = 0u; ll[i] = 0u; }
  unsigned thr_h = 0u, thr_l = 0u;   // the K-th slot: what an entry has to beat to get in
  auto offer = [&](float s, int key) {
    unsigned h = beam_order_bits(s), l = ~(unsigned)key;
    if (!(h > thr_h || (h == thr_h && l > thr_l))) return;
    // one pass of compare-and-swap down the list: the new entry sinks to its place, the last one drops out
#pragma unroll
    for (int i = 0; i < KMAX; ++i) {
      const bool better = i < K && (h > lh[i] || (h == lh[i] && l > ll[i]));
      const unsigned th = lh[i], tl = ll[i];
      lh[i] = better ? h : th; ll[i] = better ? l : tl;
      h = better ? th : h; l = better ? tl : l;
      if (i == K - 1) { thr_h = lh[i]; thr_l = ll[i]; }
    }
  };
  for (int t = 0; t < n; ++t) {
    const float *row = lg + (size_t)t * V1;
    const float add = s_run[t] - s_lse[t];
    for (int v0 = tid; v0 < V; v0 += 256 * 32) {
      float x[32];
#pragma unroll
      for (int i = 0; i < 32; ++i) x[i] = v0 + 256 * i < V ? row[v0 + 256 * i] : -INFINITY;
#pragma unroll
      for (int i = 0; i < 32; ++i)
        if (v0 + 256 * i < V) offer(x[i] + add, t * V1 + v0 + 256 * i);
    }
  }
  if (tid == 0) offer(s_run[n], (n - 1) * V1 + V);        // blank: only as "jump out of the window"
  // ---- merge, level 1: K rounds over the heads of the wave's 64 lists; lane r keeps the r-th winner
  unsigned win_h = 0u, win_l = 0u;
  for (int r = 0; r < K; ++r) {
    unsigned h = lh[0], l = ll[0];
    const unsigned myh = h, myl = l;
    wave_max_pair(h, l);
    if (myh == h && myl == l && h != 0u) {   // this lane's head won: pop it
#pragma unroll
      for (int i = 0; i + 1 < KMAX; ++i) { lh[i] = lh[i + 1]; ll[i] = ll[i + 1]; }
      lh[KMAX - 1] = 0u; ll[KMAX - 1] = 0u;
    }
    if (lane == r) { win_h = h; win_l = l; }
  }
  if (lane < K) { s_hi[wave][lane] = win_h; s_lo[wave][lane] = win_l; }
  __syncthreads();
  // ---- level 2: wave 0 merges the four sorted lists of K (lanes 0..3 hold the heads)
  if (wave == 0) {
    int h2 = 0;
    for (int r = 0; r < K; ++r) {
      unsigned h = (lane < 4 && h2 < K) ? s_hi[lane][h2] : 0u, l = (lane < 4 && h2 < K) ? s_lo[lane][h2] : 0u;
      const unsigned myh = h, myl = l;
      wave_max_pair(h, l);
      if (lane < 4 && myh == h && myl == l && h != 0u) ++h2;
      if (lane == 0) {
        const size_t o = (size_t)blockIdx.x * K + r;
        const bool any = h != 0u;
        const int key = (int)~l;
        out_labels[o] = any ? key % V1 : -1;
        out_jumps[o] = any ? key / V1 : -1;
        out_scores[o] = any ? beam_score_of(h) : -INFINITY;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The same scoring step in two short kernels for vocabularies of at most 256 * 36 entries, where a
// row fits the registers of one workgroup: every row is read in one round trip.
//
// Kernel 1, one workgroup per row (b, t): log-sum-exp of the row, log P(blank | t), and the row's K
// largest label logits with their labels (ties: lower label first).  Adding the row's constant
// (blank prefix sum minus log-sum-exp) keeps their order, so these are the only entries of the row
// that can be among the hypothesis' K best.
template <int EPT>
__global__ __launch_bounds__(256) void beam_row_kernel(const float *logits, int V, int K, float *lse_out,
                                                       float *blank_lp, float *cand_logit, int *cand_label) {
  __shared__ float s_f[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, V1 = V + 1;
  const float *row = logits + (size_t)blockIdx.x * V1;
  float x[EPT];
#pragma unroll
  for (int i = 0; i < EPT; ++i) x[i] = tid + 256 * i < V1 ? row[tid + 256 * i] : -INFINITY;
  float mx = x[0];
#pragma unroll
  for (int i = 1; i < EPT; ++i) mx = fmaxf(mx, x[i]);
  mx = wave_max_f32(mx);
  if (lane == 0) s_f[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
  __syncthreads();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < EPT; ++i) sum += expf(x[i] - mx);
  sum = wave_sum(sum);
  if (lane == 0) s_f[wave] = sum;
  __syncthreads();
  const float lse = mx + logf((s_f[0] + s_f[1]) + (s_f[2] + s_f[3]));
  if (tid == 0) {
    lse_out[blockIdx.x] = lse;
    blank_lp[blockIdx.x] = row[V] - lse;
  }
  // The row's K largest label logits.  Level 1: every wave takes K rounds of "largest remaining entry of
  // my 64 lanes" (no workgroup barrier); level 2: wave 0 merges the four sorted lists.
  __shared__ unsigned s_wh[4][kBeamMaxK], s_wl[4][kBeamMaxK];
  unsigned hi[EPT];
#pragma unroll
  for (int i = 0; i < EPT; ++i) hi[i] = tid + 256 * i < V ? beam_order_bits(x[i]) : 0u;   // blank and padding never compete
  for (int r = 0; r < K; ++r) {
    unsigned bh = 0u, bl = 0u;
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const unsigned l = ~(unsigned)(tid + 256 * i);
      const bool better = hi[i] > bh || (hi[i] == bh && hi[i] != 0u && l > bl);
      bh = better ? hi[i] : bh;
      bl = better ? l : bl;
    }
    unsigned wh = bh, wl = bl;
    wave_max_pair(wh, wl);
    const int v = (int)~wl;
    if (wh != 0u && (v & 255) == tid) {   // the winner's owner retires it
#pragma unroll
      for (int i = 0; i < EPT; ++i)
        if (i == (v >> 8)) hi[i] = 0u;
    }
    if (lane == 0) { s_wh[wave][r] = wh; s_wl[wave][r] = wl; }
  }
  __syncthreads();
  if (wave == 0) {
    int h2 = 0;   // lanes 0..3: head of wave `lane`'s list
    unsigned res_h = 0u, res_l = 0u;   // lane r keeps the r-th winner; stored after the rounds
    for (int r = 0; r < K; ++r) {
      unsigned h = (lane < 4 && h2 < K) ? s_wh[lane][h2] : 0u, l = (lane < 4 && h2 < K) ? s_wl[lane][h2] : 0u;
      const unsigned myh = h, myl = l;
      wave_max_pair(h, l);
      if (lane < 4 && myh == h && myl == l && h != 0u) ++h2;
      if (lane == r) { res_h = h; res_l = l; }
    }
    if (lane < K) {
      cand_logit[(size_t)blockIdx.x * K + lane] = res_h != 0u ? beam_score_of(res_h) : -INFINITY;
      cand_label[(size_t)blockIdx.x * K + lane] = res_h != 0u ? (int)~res_l : -1;
    }
  }
}

// Kernel 2, one wave per hypothesis: running sum of the blank log-probabilities, then K rounds over
// the heads of the rows' candidate lists (lane t holds row t; the lists are sorted, and so are
// their scores) with the all-blank entry competing as one more candidate.
__global__ __launch_bounds__(64) void beam_merge_kernel(const float *lse, const float *blank_lp, const float *cand_logit,
                                                        const int *cand_label, int n, int V, int K, int *out_labels,
                                                        int *out_jumps, float *out_scores) {
  __shared__ float s_cl[kBeamMaxWindow * kBeamMaxK];
  __shared__ int s_cv[kBeamMaxWindow * kBeamMaxK];
  const int lane = threadIdx.x, b = blockIdx.x, V1 = V + 1;
  const bool has_row = lane < n;
  // the hypothesis' candidates in one round trip: the rounds below walk them with dependent reads
  for (int i = lane; i < n * K; i += 64) {
    s_cl[i] = cand_logit[(size_t)b * n * K + i];
    s_cv[i] = cand_label[(size_t)b * n * K + i];
  }
  __syncthreads();
  const float my_blank = has_row ? blank_lp[(size_t)b * n + lane] : 0.f;
  // exclusive prefix sum over the rows, in row order (fp32, the order the definition adds them in)
  float run = 0.f, total = 0.f;
  for (int t = 0; t < n; ++t) {
    const float v = readlane_f32(my_blank, t);
    if (lane == t) run = total;
    total += v;
  }
  const float add = has_row ? run - lse[(size_t)b * n + lane] : 0.f;
  const float *cl = s_cl + (has_row ? lane : 0) * K;
  const int *cv = s_cv + (has_row ? lane : 0) * K;
  unsigned blank_h = beam_order_bits(total), blank_l = ~(unsigned)((n - 1) * V1 + V);
  int head = 0;
  float cur = has_row ? cl[0] : -INFINITY;
  int curv = has_row ? cv[0] : -1;
  unsigned res_h = 0u, res_l = 0u;   // lane r keeps the r-th winner; label and jump are worked out after the rounds
  for (int r = 0; r < K; ++r) {
    unsigned h = 0u, l = 0u;
    if (has_row && head < K && curv >= 0) { h = beam_order_bits(cur + add); l = ~(unsigned)(lane * V1 + curv); }
    const unsigned myh = h, myl = l;
    wave_max_pair(h, l);
    const bool blank_wins = blank_h != 0u && (blank_h > h || (blank_h == h && blank_l > l));
    if (blank_wins) { h = blank_h; l = blank_l; blank_h = 0u; }
    else if (myh == h && myl == l && h != 0u) {   // this row's head won: move on to its next candidate
      ++head;
      cur = head < K ? cl[head] : -INFINITY;
      curv = head < K ? cv[head] : -1;
    }
    if (lane == r) { res_h = h; res_l = l; }
  }
  if (lane < K) {
    const size_t o = (size_t)b * K + lane;
    const int key = (int)~res_l;
    out_labels[o] = res_h != 0u ? key % V1 : -1;
    out_jumps[o] = res_h != 0u ? key / V1 : -1;
    out_scores[o] = res_h != 0u ? beam_score_of(res_h) : -INFINITY;
  }
}

}  // namespace wind
