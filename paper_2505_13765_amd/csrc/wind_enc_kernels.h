// Once-per-call kernels (state set-up, encoder projection) and the window gather of every iteration.
#pragma once
#include "wind_types.h"

namespace wind {

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_int_kernel(int *p, int n, int v) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) p[i] = v;
}

__global__ __launch_bounds__(256) void init_state_kernel(ModelDev m, CallDev c) {
  const int tid = threadIdx.x;
  // every workgroup zeroes its share of the prediction-network state; the first also builds the lists
  const size_t nstate = (size_t)m.L * c.B * m.Hp;
  for (size_t i = (size_t)blockIdx.x * 256 + tid; i < nstate; i += (size_t)gridDim.x * 256) {
    c.h[i] = 0.f; c.c[i] = 0.f; c.hn[i] = 0.f;
    c.hb_hi[i] = 0; c.hb_lo[i] = 0; c.hbn_hi[i] = 0; c.hbn_lo[i] = 0;
  }
  if (blockIdx.x != 0) return;
  for (int i = tid; i < kNumStats; i += 256) c.stats[i] = 0ull;
  for (int b = tid; b < c.B; b += 256) {
    int len = c.lengths[b];
    len = len < 0 ? 0 : (len > c.T ? c.T : len);
    c.len[b] = len;
    c.out_counts[b] = 0;
    c.emit_idx[b] = b;         // the first prediction-network step runs on every utterance
    c.emit_list_tok[b] = m.V;  // on the start token
  }
  __syncthreads();
  if (tid < 64) {              // slot table of parity 0: the non-empty utterances, in order
    int na = 0;
    for (int base = 0; base < c.B; base += 64) {
      const int b = base + tid;
      const int len = b < c.B ? c.len[b] : 0;
      const unsigned long long mk = __ballot(len > 0);
      if (len > 0) {
        const int pos = na + __popcll(mk & ((1ull << tid) - 1ull));
        c.slot_state[pos] = make_int4(b, 0, len, 0);
        c.slot_count[pos] = 0;
      }
      na += __popcll(mk);
    }
    if (tid == 0) {
      c.n_active[0] = na;
      c.n_active[1] = 0;
      *c.n_emit = c.B;
      c.ticket[0] = 0u;
      c.ticket[1] = 0u;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// e[b,t,:] = W_enc enc_out[b,t,:] + b_enc for t < len[b]: bf16 MFMA, fp32 accumulate, fp32 out.
template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) void enc_proj_mfma_kernel(ModelDev m, CallDev c, int tiles_per_utt) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);
  const int b = blockIdx.x / tiles_per_utt, t0 = (blockIdx.x % tiles_per_utt) * Cfg::BM;
  const int len = c.len[b];
  if (t0 >= len) return;
  const int n0 = blockIdx.y * Cfg::BN, D = m.D;
  const float *base = c.enc + (size_t)b * c.T * D;
  auto aload = [&](int, int row, int k) -> u32x4 {
    int t = t0 + row;
    t = t < len ? t : len - 1;
    const f32x4 *src = reinterpret_cast<const f32x4 *>(base + (size_t)t * D + k);
    const f32x4 x0 = src[0], x1 = src[1];
    u32x4 o;
    o.x = pack_bf16x2(x0.x, x0.y); o.y = pack_bf16x2(x0.z, x0.w);
    o.z = pack_bf16x2(x1.x, x1.y); o.w = pack_bf16x2(x1.z, x1.w);
    return o;
  };
  f32x16 acc[Cfg::MI][Cfg::NI];
  gemm_mainloop<Cfg>(aload, reinterpret_cast<const bf16_t *>(m.w_enc) + (size_t)n0 * D, D, smem, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
  for (int ni = 0; ni < Cfg::NI; ++ni) {
    const int col = n0 + wn * Cfg::WN + ni * 32 + (lane & 31);
    if (col >= m.Hj) continue;
    const float bias = m.b_enc[col];
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = t0 + wm * Cfg::WM + acc_row(mi, r, lane);
        if (t < len) c.e[((size_t)b * c.T + t) * m.Hj + col] = acc[mi][ni][r] + bias;
      }
  }
}

// Large calls: the encoder outputs are first rounded to bf16 rows (valid frames only), so that the
// projection can use the direct-to-LDS tile core at full tile size.
// (slab: in slabs of 32 inputs, [D / 32][B*T + 256][32], for enc_proj_wide_kernel)
__global__ __launch_bounds__(256) void enc_round_kernel(ModelDev m, CallDev c, int slab) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long row = (long long)blockIdx.x * 4 + wave;
  if (row >= (long long)c.B * c.T) return;
  const int b = (int)(row / c.T), t = (int)(row - (long long)b * c.T);
  if (t >= c.len[b]) return;
  const float *src = c.enc + (size_t)row * m.D;
  const size_t slab_elems = ((size_t)c.B * c.T + 256) * 32;
  bf16_t *dst = slab ? c.enc_b + (size_t)row * 32 : c.enc_b + (size_t)row * m.D;
  for (int k = lane * 4; k < m.D; k += 256) {
    const float4 x = *reinterpret_cast<const float4 *>(src + k);
    bf16_t *p = slab ? dst + (size_t)(k >> 5) * slab_elems + (k & 31) : dst + k;
    *reinterpret_cast<uint2 *>(p) = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
  }
}

// e = W_enc enc + b_enc on 256 x 256 tiles of the five-slot ring: a row tile is 256 consecutive
// frames of one utterance (rows past its length are computed and dropped).
template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) void enc_proj_ring5_kernel(ModelDev m, CallDev c, int tiles_per_utt) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int b = blockIdx.x / tiles_per_utt, t0 = (blockIdx.x % tiles_per_utt) * Cfg::BM;
  const int len = c.len[b];
  if (t0 >= len) return;
  const int n0 = blockIdx.y * Cfg::BN, D = m.D;
  f32x16 acc[Cfg::MI][Cfg::NI];
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
  gemm_mainloop_ring5<Cfg>(c.enc_b + ((size_t)b * c.T + t0) * D, reinterpret_cast<const bf16_t *>(m.w_enc) + (size_t)n0 * D, D,
                           smem_raw, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
#pragma unroll
  for (int ni = 0; ni < Cfg::NI; ++ni) {
    const int col = n0 + wn * Cfg::WN + ni * 32 + (lane & 31);
    if (col >= m.Hj) continue;
    const float bias = m.b_enc[col];
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = t0 + wm * Cfg::WM + acc_row(mi, r, lane);
        if (t < len) c.e[((size_t)b * c.T + t) * m.Hj + col] = acc[mi][ni][r] + bias;
      }
  }
}

// The same product on the 256-column tile core of wind_mfma_wide.h (four waves of up to 512 registers, operands
// in slabs of 32 inputs, five-stage ring).  A row tile is up to 256 consecutive frames of one utterance, as high
// as the frames left need (64 MI rows); the four column tiles of a row tile get launch ids that differ by
// multiples of 8, so that they run on one XCD and the frames come from memory once.  Every output is the same
// chain of MFMAs over D as in the other kernels.
template <int MI>
__device__ __forceinline__ void enc_proj_wide_tile(const ModelDev &m, const CallDev &c, int b, int t0, int len, int n0,
                                                   unsigned char *smem_raw) {
  using Cfg = WideCfg<MI>;
  const int KS = m.D / 32, hj_pad = (m.Hj + 255) / 256 * 256;
  const long long rows_total = (long long)c.B * c.T + 256;
  const uint32_t slab_a = (uint32_t)rows_total * 64u, slab_b = (uint32_t)hj_pad * 64u;
  const i32x4 rs_a = wide_rsrc(c.enc_b, slab_a * (uint32_t)KS), rs_b = wide_rsrc(m.w_enc_slab, slab_b * (uint32_t)KS);
  const int wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1, lane = threadIdx.x & 63;
  f32x16 acc[Cfg::MI][Cfg::NI];
  bf16x8 af[2][Cfg::MI], bfr[2][Cfg::NI];
  wide_head_b(rs_b, slab_b, n0, KS, smem_raw);
  auto zero = [&]() {
#pragma unroll
    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
  };
  wide_mainloop<Cfg>(rs_a, slab_a, rs_b, slab_b, KS, 0, 1, n0, (int)rows_total, smem_raw, acc, af, bfr, zero, b * c.T + t0);
  // Transposed blocks: a lane holds four runs of four consecutive columns of one row, 16 stores of 16 bytes per
  // block pair.  (Not transposed, a store would write 32 consecutive columns of a row, whole cache lines, but
  // four times as many store instructions: 0.88 against 0.67 ms on the 128 x 2000-frame batch.)
  wide_last_step<Cfg>(acc, af[1], bfr[1], [&](int mi, int p, const f32x16 &lo, const f32x16 &hi) {
    const int t = t0 + (2 * mi + wm) * 32 + (lane & 31);
    if (t >= len) return;
    float *out = c.e + ((size_t)b * c.T + t) * m.Hj;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 128 + 64 * p + 32 * h + 8 * g + 4 * (lane >> 5);
        if (col >= m.Hj) continue;   // Hj is a multiple of 64: whole groups of four
        const float4 bias = *reinterpret_cast<const float4 *>(m.b_enc + col);
        const f32x16 &v = h ? hi : lo;
        *reinterpret_cast<float4 *>(out + col) = make_float4(v[4 * g] + bias.x, v[4 * g + 1] + bias.y, v[4 * g + 2] + bias.z, v[4 * g + 3] + bias.w);
      }
  });
}

__global__ __launch_bounds__(256) void enc_proj_wide_kernel(ModelDev m, CallDev c, int tiles_per_utt, int n_row_tiles, int n_col_tiles) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int id = (int)blockIdx.x, q = id >> 3;
  const int rt = (q / n_col_tiles) * 8 + (id & 7), ct = q % n_col_tiles;
  if (rt >= n_row_tiles) return;
  const int b = rt / tiles_per_utt, t0 = (rt % tiles_per_utt) * 256;
  const int len = c.len[b];
  if (t0 >= len) return;
  const int mi = (min(len - t0, 256) + 63) / 64;
  switch (mi) {
    case 1: enc_proj_wide_tile<1>(m, c, b, t0, len, ct * 256, smem_raw); break;
    case 2: enc_proj_wide_tile<2>(m, c, b, t0, len, ct * 256, smem_raw); break;
    case 3: enc_proj_wide_tile<3>(m, c, b, t0, len, ct * 256, smem_raw); break;
    default: enc_proj_wide_tile<4>(m, c, b, t0, len, ct * 256, smem_raw); break;
  }
}

// fp32 models: out[row, j] = bias[j] + sum_k w[j,k] x[row,k] for the valid frames of each utterance.
__global__ __launch_bounds__(256) void enc_proj_f32_kernel(ModelDev m, CallDev c) {
  extern __shared__ float xs[];
  const int b = blockIdx.y, t = blockIdx.x;
  if (t >= c.len[b]) return;
  const float *x = c.enc + ((size_t)b * c.T + t) * m.D;
  for (int k = threadIdx.x; k < m.D; k += 256) xs[k] = x[k];
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float *w = reinterpret_cast<const float *>(m.w_enc);
  for (int j = wave; j < m.Hj; j += 4) {
    float a = 0.f;
    for (int k = lane; k < m.D; k += 64) a = fmaf(w[(size_t)j * m.D + k], xs[k], a);
    a = wave_sum(a);
    if (lane == 0) c.e[((size_t)b * c.T + t) * m.Hj + j] = a + m.b_enc[j];
  }
}

// ---------------------------------------------------------------------------------------------
// Window gather (Algorithm 2: the joiner on a window of frames against the current decoder output, its
// first half): one wave per window row.
// slab: z in slabs of 32 hidden units, [Hj / 32][Mpad][32], as joint_wide_kernel reads it, instead of dense rows.
// wide_rows > 0: iterations with more window rows than that are counted (ST_WIDE; the host's choice of the
// joint kernel for the next call of the same shape rests on it).
__global__ __launch_bounds__(256) void build_z_kernel(ModelDev m, CallDev c, int parity, int slab, int wide_rows) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  const int a = row / c.W, j = row - a * c.W;
  if (a >= c.B) return;
  const int na = c.n_active[parity];
  const int4 st = c.slot_state[parity * c.slot_stride + a];   // same round trip as the count
  // the counters that this iteration's decision kernel adds to: every reader of their old values is done
  if (c.lists_atomic && blockIdx.x == 0 && threadIdx.x == 0) { c.n_active[parity ^ 1] = 0; *c.n_emit = 0; }
  if (wide_rows > 0 && blockIdx.x == 0 && threadIdx.x == 0 && na * c.W > wide_rows) c.stats[ST_WIDE] += 1ull;   // one writer per iteration
  if (c.iter_rows && blockIdx.x == 0 && wave == 0 && na > 0) {
    // profile mode: rows the method evaluates in this iteration = sum of n over the windows; iterations
    // so far = the decision kernel's counter (complete: that kernel precedes this one in the stream)
    int rows = 0;
    for (int i = lane; i < na; i += 64) {
      const int4 s = c.slot_state[parity * c.slot_stride + i];
      rows += min(c.W, s.z - s.y);
    }
    rows = wave_sum_i32(rows);
    const unsigned long long it = c.stats[ST_ITER];
    if (lane == 0 && it < (unsigned long long)c.iter_rows_cap) c.iter_rows[it] = rows;
  }
  if (a >= na) return;
  const int b = st.x, tt = st.y + j;
  const bool valid = tt < st.z;
  const int Hj = m.Hj;
  const float *er = c.e + ((size_t)b * c.T + (valid ? tt : 0)) * Hj;
  const float *pr = c.p + (size_t)b * Hj;
  bf16_t *zr = slab ? c.z + (size_t)row * 32 : c.z + (size_t)row * Hj;
  const size_t slab_elems = (size_t)c.Mpad * 32;
  float dot = 0.f, nrm = 0.f;
  // 1024 hidden units per pass: the pass's twelve loads per lane go out together (one round trip)
  for (int k0 = lane * 4; k0 < Hj; k0 += 1024) {
    float4 ev[4], pv[4], wb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + 256 * i;
      ev[i] = pv[i] = wb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k < Hj) {
        wb[i] = *reinterpret_cast<const float4 *>(m.w_blank + k);
        if (valid) {
          ev[i] = *reinterpret_cast<const float4 *>(er + k);
          pv[i] = *reinterpret_cast<const float4 *>(pr + k);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + 256 * i;
      if (k >= Hj) continue;
      float4 x;   // invalid rows: e and p were left at zero
      x.x = fmaxf(ev[i].x + pv[i].x, 0.f); x.y = fmaxf(ev[i].y + pv[i].y, 0.f);
      x.z = fmaxf(ev[i].z + pv[i].z, 0.f); x.w = fmaxf(ev[i].w + pv[i].w, 0.f);
      dot = fmaf(x.x, wb[i].x, dot); dot = fmaf(x.y, wb[i].y, dot);
      dot = fmaf(x.z, wb[i].z, dot); dot = fmaf(x.w, wb[i].w, dot);
      nrm = fmaf(x.x, x.x, nrm); nrm = fmaf(x.y, x.y, nrm);
      nrm = fmaf(x.z, x.z, nrm); nrm = fmaf(x.w, x.w, nrm);
      bf16_t *zp = slab ? zr + (size_t)(k >> 5) * slab_elems + (k & 31) : zr + k;
      *reinterpret_cast<uint2 *>(zp) = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
    }
  }
  dot = wave_sum(dot);
  nrm = wave_sum(nrm);
  if (lane == 0) {
    c.blank_logit[row] = dot + m.b_out[m.V];
    c.znorm[row] = sqrtf(nrm);
  }
}

}  // namespace wind
