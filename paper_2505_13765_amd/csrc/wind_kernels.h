// Device kernels of the WIND greedy decoder (gfx950).  See include/wind.h for the model.
//
// One loop iteration (Method, Algorithm 2, all active utterances at once), bf16 models:
//   build_z        window gather: z[r,j,:] = relu(e[b, t_b + j, :] + p[b,:]) in bf16, plus the
//                  blank logit and the norm of every row in fp32
//   joint_ws       label logits of every window row on bf16 MFMA; per row and per 64-column part
//                  the two largest (logit, column) keys are kept, nothing else is stored.  Tiles of
//                  128 columns whose height (64 to 256 rows) and number per workgroup follow the
//                  iteration's row count; four waves of a workgroup multiply, four fetch
//   decide         per utterance: row argmax from the keys, near-ties re-decided with fp32 dot
//                  products, first non-blank row by wavefront ballot, pointer / hypothesis update,
//                  the utterance's place in the next iteration's slot table and in the emit list
//                  (claimed with atomic counters), and the first LSTM layer's step for the label
//                  (elementwise, on top of the recurrent gate sums kept in CallDev::rec)
//   lstm_layer     the layers above the first, for the utterances that emitted: their input half
//   pred_proj      p = W_pred h + b_pred for those utterances; the same launch renews the
//                  recurrent gate sums of every layer for them
// Optionally (CallDev::rec null, lists_atomic 0) the steps are whole LSTM steps after the decision
// and the last workgroup of decide compacts the lists in order.  The prediction network has three
// implementations: MFMA tiles with the hidden state split into bf16 hi + lo, low-latency
// wave-per-unit kernels (the start-token step of the resident loop kernel), generic FMA (fp32
// models).  fp32 models replace build_z + joint by joint_exact (fp32 FMA, argmax taken directly).
// One or two utterances of a one-layer model run the whole loop as one resident kernel
// (wind_loop_kernel).
#pragma once
#include "wind_mfma.h"
#include "wind_mfma_dma.h"
#include "wind_mfma_ws.h"

namespace wind {

constexpr int kMaxLayers = 4;
constexpr int kMaxWindow = 64;
constexpr int kTinyRows = 64;   // slots the resident loop kernel keeps in LDS (it runs far fewer)
constexpr int kStatJump0 = 8;  // index of jump_hist[0] in the device counter array
constexpr int kNumStats = kStatJump0 + kMaxWindow + 1;
enum { ST_ITER = 0, ST_WINDOWS, ST_ROWS, ST_USEFUL, ST_LABELS, ST_FORCED, ST_RECHECK, ST_OVERFLOW };

// Weights on the device.  WT-typed matrices are bf16 (bf16 models) or fp32 (fp32 models).
struct ModelDev {
  int D, E, Hp, L, Hj, V;
  int Vpad;                     // rows of w_out (>= V+1, zero filled past V)
  const void *emb;              // [V+1, E]
  // The first layer's input is an embedding row, so its input half of the gate sums is a table
  // lookup: emb_gates[v][4*j+g] = b_ih + b_hh + w_ih[gate g of unit j] . emb[v], built once at load.
  const float *emb_gates;       // [V+1, 4Hp] fp32
  // Recurrent weights.  Layer 0: [4Hp, Hp] = w_hh (in_0 = 0 below); layer l > 0: [4Hp, in_l + Hp] =
  // [w_ih | w_hh] with in_l = Hp.  Row 4*j+g = gate g (i,f,g,o) of unit j.
  const void *w_cat[kMaxLayers];
  const float *b_cat[kMaxLayers]; // [4Hp] same row order, b_ih + b_hh (layers > 0)
  const void *w_cat_t[kMaxLayers]; // bf16 models: the same rows grouped for MFMA tiles, see lstm_layer_dma_kernel
  const float *b_cat_t[kMaxLayers];
  const void *w_enc;            // [Hj_pad, D]
  const float *b_enc;           // [Hj]
  const void *w_pred;           // [Hj, Hp]
  const float *b_pred;          // [Hj]
  const void *w_out;            // [Vpad, Hj]; row V = blank
  const float *b_out;           // [V+1]
  const float *w_blank;         // [Hj] fp32 copy of row V
  float tau_scale;              // near-tie band = tau_scale * |z|_2 (+ key truncation)
};

// One decode call: caller buffers, sizes, and the library's state arrays.
struct CallDev {
  int B, T, W, S, cap;
  const float *enc;             // [B,T,D]
  const int *lengths;           // [B] as given
  int *out_tokens, *out_frames, *out_counts;
  float *e;                     // [B*T, Hj]
  bf16_t *enc_b;                // [B*T + 256, D] encoder outputs rounded to bf16 (large calls only, else null)
  int *len;                     // [B] clamped to [0,T]
  // Active utterances live in a slot table, ping-pong by iteration parity: slot a of the current
  // parity holds everything an iteration needs to know about its a-th active utterance, so that a
  // kernel reaches it with one load whose address does not depend on another load.
  int4 *slot_state;             // [2][slot_stride] (utterance, t, len, labels on the current frame)
  int *slot_count;              // [2][slot_stride] labels emitted so far
  int slot_stride;              // max(B, 64)
  int *n_active;                // [2]
  int4 *res_state;              // [B] per slot, this iteration's outcome: the new (utterance, t, len, sym)
  int4 *res_aux;                // [B] (count, flag, label, event): flag bit0 still active, bit1 emitted and
                                //     still active; event = the window's counters, packed (see decide_utterance)
  int *emit_idx;                // [B] utterances that emitted and are still active, in order
  int *emit_list_tok;           // [B] their labels, in the same order
  int *n_emit;                  // [1]
  unsigned *ticket;             // [2] workgroups done (decide_kernel)
  int lists_atomic;             // 1: decide_kernel's workgroups claim their places in the next slot table and the
                                //    emit list with atomic counters (order varies, results do not); 0: the last
                                //    workgroup to finish compacts res_state / res_aux in slot order
  float *h, *c, *hn;            // [L][B][Hp]
  bf16_t *hb_hi, *hb_lo, *hbn_hi, *hbn_lo;  // [L][B][Hp] large-batch path: h and new h as bf16 hi + lo
  const bf16_t *hb_zero;        // [max(E,Hp)] zeros (the lo part of an embedding row)
  // Large batches: the recurrent half of every layer's gate sums, w_hh . h, for the hidden vectors as
  // they stand (row order 4*unit + gate, no bias).  It changes only when its utterance emits, and it is
  // renewed beside the projection of that step, so the next step, once its label is known, has only
  // the input half left to do.  Null where this is not used (the full products are then formed per step).
  float *rec;                   // [L][B][4Hp]
  float *p;                     // [B][Hj]
  bf16_t *z;                    // [Mpad][Hj]
  float *blank_logit;           // [Mpad]
  float *znorm;                 // [Mpad]
  // Keys: per window row and column part the largest (logit, column) keys of the part.  The joint kernel
  // writes three per entry (four words, the last unused); the resident loop kernel keeps two (two words).
  float *parts;                 // [Mpad][nparts][4] (joint kernel) or [rows][nparts_tiny][2] (loop kernel)
  int nparts;                   // parts per row and label columns per part, as written by the joint kernel
  int part_width;
  int nparts_tiny;              // parts per row of the resident loop kernel (32 columns each)
  int *row_label;               // [Mpad] (fp32 models)
  unsigned long long *stats;    // [kNumStats]
  long long *dbg;               // optional [8] phase time stamps of the few-rows kernel's deciding workgroup (100 MHz clock)
  int *iter_rows;               // optional [iter_rows_cap] window rows of every loop iteration, in order (profile mode)
  int iter_rows_cap;
};

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
__global__ __launch_bounds__(256) void enc_round_kernel(ModelDev m, CallDev c) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long row = (long long)blockIdx.x * 4 + wave;
  if (row >= (long long)c.B * c.T) return;
  const int b = (int)(row / c.T), t = (int)(row - (long long)b * c.T);
  if (t >= c.len[b]) return;
  const float *src = c.enc + (size_t)row * m.D;
  bf16_t *dst = c.enc_b + (size_t)row * m.D;
  for (int k = lane * 4; k < m.D; k += 256) {
    const float4 x = *reinterpret_cast<const float4 *>(src + k);
    *reinterpret_cast<uint2 *>(dst + k) = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
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
__global__ __launch_bounds__(256) void build_z_kernel(ModelDev m, CallDev c, int parity) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  const int a = row / c.W, j = row - a * c.W;
  if (a >= c.B) return;
  const int na = c.n_active[parity];
  const int4 st = c.slot_state[parity * c.slot_stride + a];   // same round trip as the count
  // the counters that this iteration's decision kernel adds to: every reader of their old values is done
  if (c.lists_atomic && blockIdx.x == 0 && threadIdx.x == 0) { c.n_active[parity ^ 1] = 0; *c.n_emit = 0; }
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
  bf16_t *zr = c.z + (size_t)row * Hj;
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
      *reinterpret_cast<uint2 *>(zr + k) = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
    }
  }
  dot = wave_sum(dot);
  nrm = wave_sum(nrm);
  if (lane == 0) {
    c.blank_logit[row] = dot + m.b_out[m.V];
    c.znorm[row] = sqrtf(nrm);
  }
}

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
#pragma unroll
  for (int mi = 0; mi < Cfg::MI; ++mi) {
    float k1 = kKeyNone, k2 = kKeyNone, k3 = kKeyNone;
#pragma unroll
    for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) push_top3(k1, k2, k3, make_key(acc[mi][ni][r], ni * 32 + 8 * (r >> 2) + (r & 3)));
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

// ---------------------------------------------------------------------------------------------
// Running argmax (ties to the lowest id) over the fp32 logits of nc candidate labels, lane i
// holding the i-th candidate's column, for the hidden vector the wave holds (zr[i] = z[2*lane +
// 128*i .. +1]).  Four weight rows are requested together, so that a near-tie costs one memory
// round trip for up to four candidates.
template <class WT, int NZ>
__device__ __forceinline__ void evaluate_candidates_wide(const ModelDev &m, const float2 (&zr)[NZ], int mycol, int nc,
                                                    int lane, float &bestv, int &besti) {
  const WT *w = reinterpret_cast<const WT *>(m.w_out);
  for (int c0 = 0; c0 < nc; c0 += 4) {
    const int col0 = __shfl(mycol, c0, kWave), col1 = __shfl(mycol, min(c0 + 1, nc - 1), kWave);
    const int col2 = __shfl(mycol, min(c0 + 2, nc - 1), kWave), col3 = __shfl(mycol, min(c0 + 3, nc - 1), kWave);
    const WT *w0 = w + (size_t)col0 * m.Hj, *w1 = w + (size_t)col1 * m.Hj;
    const WT *w2 = w + (size_t)col2 * m.Hj, *w3 = w + (size_t)col3 * m.Hj;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
    for (int i = 0; i < NZ; ++i) {
      const int k = 2 * lane + 128 * i;
      if (k < m.Hj) {
        const float2 x0 = ldw2(w0, k), x1 = ldw2(w1, k), x2 = ldw2(w2, k), x3 = ldw2(w3, k);
        a0 = fmaf(x0.x, zr[i].x, a0); a0 = fmaf(x0.y, zr[i].y, a0);
        a1 = fmaf(x1.x, zr[i].x, a1); a1 = fmaf(x1.y, zr[i].y, a1);
        a2 = fmaf(x2.x, zr[i].x, a2); a2 = fmaf(x2.y, zr[i].y, a2);
        a3 = fmaf(x3.x, zr[i].x, a3); a3 = fmaf(x3.y, zr[i].y, a3);
      }
    }
    const float v0 = wave_sum(a0) + m.b_out[col0], v1 = wave_sum(a1) + m.b_out[col1];
    const float v2 = wave_sum(a2) + m.b_out[col2], v3 = wave_sum(a3) + m.b_out[col3];
    if (v0 > bestv || (v0 == bestv && col0 < besti)) { bestv = v0; besti = col0; }
    if (v1 > bestv || (v1 == bestv && col1 < besti)) { bestv = v1; besti = col1; }
    if (v2 > bestv || (v2 == bestv && col2 < besti)) { bestv = v2; besti = col2; }
    if (v3 > bestv || (v3 == bestv && col3 < besti)) { bestv = v3; besti = col3; }
  }
}

template <int NZ>
__device__ __forceinline__ void evaluate_candidates(const ModelDev &m, const float2 (&ev)[NZ], const float2 (&pv)[NZ],
                                                    int mycol, int nc, int lane, float &bestv, int &besti) {
  // ev holds the row's encoder projections e and pv its prediction projections p, as requested by
  // the caller and not yet looked at; they are combined into z = relu(e + p) only behind the
  // round's weight requests, so that both requests are in flight together: a near-tie then costs
  // one trip to memory, not two.  Weights stay packed (two bf16 per register) until used.
  const bf16_t *w = reinterpret_cast<const bf16_t *>(m.w_out);
  for (int c0 = 0; c0 < nc; c0 += 4) {
    const int col0 = __shfl(mycol, c0, kWave), col1 = __shfl(mycol, min(c0 + 1, nc - 1), kWave);
    const int col2 = __shfl(mycol, min(c0 + 2, nc - 1), kWave), col3 = __shfl(mycol, min(c0 + 3, nc - 1), kWave);
    const bf16_t *w0 = w + (size_t)col0 * m.Hj, *w1 = w + (size_t)col1 * m.Hj;
    const bf16_t *w2 = w + (size_t)col2 * m.Hj, *w3 = w + (size_t)col3 * m.Hj;
    const float o0 = m.b_out[col0], o1 = m.b_out[col1], o2 = m.b_out[col2], o3 = m.b_out[col3];
    uint32_t x0[NZ], x1[NZ], x2[NZ], x3[NZ];
#pragma unroll
    for (int i = 0; i < NZ; ++i) {
      const int k = 2 * lane + 128 * i;
      x0[i] = x1[i] = x2[i] = x3[i] = 0u;
      if (k < m.Hj) {
        x0[i] = *reinterpret_cast<const uint32_t *>(w0 + k); x1[i] = *reinterpret_cast<const uint32_t *>(w1 + k);
        x2[i] = *reinterpret_cast<const uint32_t *>(w2 + k); x3[i] = *reinterpret_cast<const uint32_t *>(w3 + k);
      }
    }
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
    for (int i = 0; i < NZ; ++i) {
      const float zx = fmaxf(ev[i].x + pv[i].x, 0.f), zy = fmaxf(ev[i].y + pv[i].y, 0.f);
      a0 = fmaf(__uint_as_float(x0[i] << 16), zx, a0); a0 = fmaf(__uint_as_float(x0[i] & 0xFFFF0000u), zy, a0);
      a1 = fmaf(__uint_as_float(x1[i] << 16), zx, a1); a1 = fmaf(__uint_as_float(x1[i] & 0xFFFF0000u), zy, a1);
      a2 = fmaf(__uint_as_float(x2[i] << 16), zx, a2); a2 = fmaf(__uint_as_float(x2[i] & 0xFFFF0000u), zy, a2);
      a3 = fmaf(__uint_as_float(x3[i] << 16), zx, a3); a3 = fmaf(__uint_as_float(x3[i] & 0xFFFF0000u), zy, a3);
    }
    const float v0 = wave_sum(a0) + o0, v1 = wave_sum(a1) + o1;
    const float v2 = wave_sum(a2) + o2, v3 = wave_sum(a3) + o3;
    if (v0 > bestv || (v0 == bestv && col0 < besti)) { bestv = v0; besti = col0; }
    if (v1 > bestv || (v1 == bestv && col1 < besti)) { bestv = v1; besti = col1; }
    if (v2 > bestv || (v2 == bestv && col2 < besti)) { bestv = v2; besti = col2; }
    if (v3 > bestv || (v3 == bestv && col3 < besti)) { bestv = v3; besti = col3; }
  }
}

constexpr int kDecideMaxHj = 2048;  // exact_logit keeps Hj/128 float2 per lane

// An fp32 value as two bf16: hi = RNE(v), lo = RNE(v - hi) (see the large-batch prediction network)
__device__ __forceinline__ void store_hi_lo(bf16_t *hi, bf16_t *lo, size_t idx, float v) {
  const uint32_t h = f32_to_bf16_bits(v);
  hi[idx] = (bf16_t)h;
  lo[idx] = (bf16_t)f32_to_bf16_bits(v - bf16_bits_to_f32(h));
}

struct DecideShared {
  int label[kMaxWindow];
  unsigned hist[kMaxWindow + 1];
  int recheck;
  int is_last;
  int step_tok;                // the label whose prediction-network step follows (emitted and still active), else -1
  // a row whose near-tie path met a column part to be re-evaluated whole leaves that part to the whole
  // workgroup: the part (-1: none) and the best fp32 logit found so far (its label is in label[])
  int pend_part[kMaxWindow];
  float pend_v[kMaxWindow];
  int n_pend;                  // rows with such a part in this window
  float coop_v[16];            // per wave: best fp32 logit and label among its share of the part's columns
  int coop_i[16];
  // LOCAL mode (fused few-rows kernel): per-slot state and per-row scalars kept in LDS, so that the
  // deciding workgroup does not go back to memory for them
  int4 slot[kTinyRows];        // utterance id, t, len, sym
  int cnt[kTinyRows];
  int flag[kTinyRows];
  int tok[kTinyRows];
  unsigned event[kTinyRows];
  float blank[kTinyRows], znorm[kTinyRows];
};

// The near-tie path of decide_row: every label key at or above `thresh` is re-evaluated in fp32 (bf16
// weight row times the hidden vector rebuilt from fp32 e and p) and the argmax over those values and
// the fp32 blank logit is returned.  A part whose SECOND key is at or above `thresh` is re-evaluated
// whole, since the two keys it kept may hide further labels inside the band.
// NZ = Hj / 128 rounded up: the lanes hold two hidden units per step.
// With `defer`, the first such part is not evaluated here: it is returned in `deferred` with the best
// logit of everything else in `best_out`, for the workgroup to evaluate together (see decide_utterance).
template <int NZ, int KW>
__device__ __forceinline__ int recheck_row(const ModelDev &m, const CallDev &c, int row, int b, int frame, int nparts,
                                           int stride, int part_width, float vblank, float thresh, float4 kk0,
                                           bool defer, int &deferred, float &best_out) {
  const int lane = threadIdx.x & 63, V = m.V;
  const size_t prow = (size_t)row * stride;
  float2 ev[NZ], pv[NZ];   // requested here, first looked at behind the weight rows' requests
  const float *er = c.e + ((size_t)b * c.T + frame) * m.Hj;
  const float *pr = c.p + (size_t)b * m.Hj;
#pragma unroll
  for (int i = 0; i < NZ; ++i) {
    const int k = 2 * lane + 128 * i;
    ev[i] = make_float2(0.f, 0.f);
    pv[i] = make_float2(0.f, 0.f);
    if (k < m.Hj) {
      ev[i] = *reinterpret_cast<const float2 *>(er + k);
      pv[i] = *reinterpret_cast<const float2 *>(pr + k);
    }
  }
  float bestv = vblank;     // blank has the highest id: it wins only if strictly larger
  int besti = V;
  // candidate columns, one per lane (lane i holds the i-th), evaluated four at a time
  int mycol = 0, nc = 0;
  for (int p0 = 0; p0 < nparts; p0 += 64) {
    const int pi = p0 + lane;
    float4 kk = no_keys();
    if (p0 == 0) kk = kk0;
    else if (pi < nparts) kk = load_keys<KW>(c.parts, prow + pi);
    // A part keeps only its largest keys (three from the joint kernel, two in the resident loop kernel).
    // If the last of them is inside the band, a further label of that part may be too, unseen: every
    // column of such a part becomes a candidate.
    const bool in1 = key_val(kk.x) >= thresh, in2 = key_val(kk.y) >= thresh;
    const bool all_in = KW == 4 ? key_val(kk.z) >= thresh : in2;
    unsigned long long whole = __ballot(all_in), mask = __ballot(in1 && !all_in), mask2 = __ballot(in2 && !all_in);
    while (whole) {
      const int src = __ffsll((long long)whole) - 1;
      whole &= whole - 1;
      if (defer && deferred < 0) { deferred = p0 + src; continue; }
      const int col0 = (p0 + src) * part_width;
      for (int i = 0; i < part_width && col0 + i < V; ++i) {
        if (lane == nc) mycol = col0 + i;
        if (++nc == 64) {
          evaluate_candidates<NZ>(m, ev, pv, mycol, nc, lane, bestv, besti);
          nc = 0;
        }
      }
    }
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      unsigned long long todo = which ? mask2 : mask;
      while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const float skey = __shfl(which ? kk.y : kk.x, src, kWave);
        const int col = (p0 + src) * part_width + key_col(skey);
        if (lane == nc) mycol = col;
        if (++nc == 64) {
          evaluate_candidates<NZ>(m, ev, pv, mycol, nc, lane, bestv, besti);
          nc = 0;
        }
      }
    }
  }
  evaluate_candidates<NZ>(m, ev, pv, mycol, nc, lane, bestv, besti);
  best_out = bestv;
  return besti;
}

// The same for joint hidden sizes above 1024 (up to kDecideMaxHj): the hidden vector is combined
// first and the weight rows are requested afterwards, which keeps the live registers within a
// 1024-thread workgroup's share.
template <int KW>
__device__ __forceinline__ int recheck_row_wide(const ModelDev &m, const CallDev &c, int row, int b, int frame, int nparts,
                                                int stride, int part_width, float vblank, float thresh, float4 kk0,
                                                bool defer, int &deferred, float &best_out) {
  const int lane = threadIdx.x & 63, V = m.V;
  const size_t prow = (size_t)row * stride;
  constexpr int NZ = kDecideMaxHj / 128;
  float2 zr[NZ];
  const float *er = c.e + ((size_t)b * c.T + frame) * m.Hj;
  const float *pr = c.p + (size_t)b * m.Hj;
#pragma unroll
  for (int i = 0; i < NZ; ++i) {
    const int k = 2 * lane + 128 * i;
    zr[i] = make_float2(0.f, 0.f);
    if (k < m.Hj) {
      const float2 ev = *reinterpret_cast<const float2 *>(er + k);
      const float2 pv = *reinterpret_cast<const float2 *>(pr + k);
      zr[i] = make_float2(fmaxf(ev.x + pv.x, 0.f), fmaxf(ev.y + pv.y, 0.f));
    }
  }
  float bestv = vblank;     // blank has the highest id: it wins only if strictly larger
  int besti = V;
  // candidate columns, one per lane (lane i holds the i-th), evaluated four at a time
  int mycol = 0, nc = 0;
  for (int p0 = 0; p0 < nparts; p0 += 64) {
    const int pi = p0 + lane;
    float4 kk = no_keys();
    if (p0 == 0) kk = kk0;
    else if (pi < nparts) kk = load_keys<KW>(c.parts, prow + pi);
    // A part keeps only its largest keys (three from the joint kernel, two in the resident loop kernel).
    // If the last of them is inside the band, a further label of that part may be too, unseen: every
    // column of such a part becomes a candidate.
    const bool in1 = key_val(kk.x) >= thresh, in2 = key_val(kk.y) >= thresh;
    const bool all_in = KW == 4 ? key_val(kk.z) >= thresh : in2;
    unsigned long long whole = __ballot(all_in), mask = __ballot(in1 && !all_in), mask2 = __ballot(in2 && !all_in);
    while (whole) {
      const int src = __ffsll((long long)whole) - 1;
      whole &= whole - 1;
      if (defer && deferred < 0) { deferred = p0 + src; continue; }
      const int col0 = (p0 + src) * part_width;
      for (int i = 0; i < part_width && col0 + i < V; ++i) {
        if (lane == nc) mycol = col0 + i;
        if (++nc == 64) {
          evaluate_candidates_wide<bf16_t, NZ>(m, zr, mycol, nc, lane, bestv, besti);
          nc = 0;
        }
      }
    }
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      unsigned long long todo = which ? mask2 : mask;
      while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const float skey = __shfl(which ? kk.y : kk.x, src, kWave);
        const int col = (p0 + src) * part_width + key_col(skey);
        if (lane == nc) mycol = col;
        if (++nc == 64) {
          evaluate_candidates_wide<bf16_t, NZ>(m, zr, mycol, nc, lane, bestv, besti);
          nc = 0;
        }
      }
    }
  }
  evaluate_candidates_wide<bf16_t, NZ>(m, zr, mycol, nc, lane, bestv, besti);
  best_out = bestv;
  return besti;
}

// Label of one window row, decided by a whole wave: argmax over the row's keys, with every key
// inside the near-tie band re-evaluated in fp32 (see the header comment of this file).
// kk0 = this lane's keys of the row for part `lane` (the caller loads them, possibly for several
// rows at once so that the loads overlap); parts 64 and up are read here.
template <class WT, bool WIDE, int KW>
__device__ __forceinline__ int decide_row(const ModelDev &m, const CallDev &c, int row, int b, int frame,
                                          int nparts, int stride, int part_width, float vblank, float znorm,
                                          float4 kk0, int &n_recheck, bool defer, int &deferred, float &best_out) {
  const int lane = threadIdx.x & 63, V = m.V;
  const size_t prow = (size_t)row * stride;
  float k1 = kk0.x;
  for (int pi = lane + 64; pi < nparts; pi += 64) k1 = fmaxf(k1, load_keys<KW>(c.parts, prow + pi).x);
  const float kbest = wave_max_f32(k1);
  const float vbest = key_val(kbest);
  const float top = fmaxf(vbest, vblank);
  const float tau = m.tau_scale * znorm + 6.2e-5f * fabsf(top);
  const float thresh = top - tau;
  if (vbest < thresh) return V;                  // blank clear of every label
  // how many label keys are inside the band?
  int cnt = (key_val(kk0.x) >= thresh) + (key_val(kk0.y) >= thresh) + (key_val(kk0.z) >= thresh);
  for (int pi = lane + 64; pi < nparts; pi += 64) {
    const float4 kk = load_keys<KW>(c.parts, prow + pi);
    cnt += (key_val(kk.x) >= thresh) + (key_val(kk.y) >= thresh) + (key_val(kk.z) >= thresh);
  }
  cnt = wave_sum_i32(cnt);
  if (cnt == 1 && vblank < thresh) {
    // a single label clear of blank and of every other label: find its part
    int col = kk0.x == kbest ? lane * part_width + key_col(kbest) : -1;
    for (int pi = lane + 64; pi < nparts; pi += 64)
      if (load_keys<KW>(c.parts, prow + pi).x == kbest) col = pi * part_width + key_col(kbest);
    return wave_max_i32(col);
  }
  // near tie: fp32 logits of every candidate, hidden vector rebuilt from fp32 e and p
  ++n_recheck;
  if constexpr (WIDE)
    return recheck_row_wide<KW>(m, c, row, b, frame, nparts, stride, part_width, vblank, thresh, kk0, defer, deferred, best_out);
  else
    return recheck_row<8, KW>(m, c, row, b, frame, nparts, stride, part_width, vblank, thresh, kk0, defer, deferred, best_out);
}

// Four window rows per wave at once, 16 lanes per row, for rows of at most 32 parts: lane 16 q + s holds
// the keys of parts s and s + 16 (kA, kB) and the blank logit and norm of row j = the q-th row of this
// wave; the reductions of decide_row then run inside the rows of 16 lanes, for all four rows in the same
// instructions.  A row inside the near-tie band goes through decide_row itself, keys re-read by the whole
// wave through `reload` (part index -> keys).  Writes sh.label[j] for j < W; returns the rows re-decided.
template <class WT, class Reload>
__device__ __forceinline__ int decide_rows_quad(const ModelDev &m, const CallDev &c, int a, int4 st, int nparts, int part_width,
                                                float2 kA, float2 kB, float vblank, float znorm, int j,
                                                const Reload &reload, DecideShared &sh) {
  const int lane = threadIdx.x & 63, s = lane & 15, V = m.V;
  const int n = min(c.W, st.z - st.y);
  const float kbest = row16_max_f32(fmaxf(kA.x, kB.x));
  const float vbest = key_val(kbest);
  const float top = fmaxf(vbest, vblank);
  const float thresh = top - (m.tau_scale * znorm + 6.2e-5f * fabsf(top));
  const int cnt = row16_sum_i32((key_val(kA.x) >= thresh) + (key_val(kA.y) >= thresh) + (key_val(kB.x) >= thresh) +
                                (key_val(kB.y) >= thresh));
  int col = -1;
  if (kA.x == kbest) col = s * part_width + key_col(kbest);
  if (kB.x == kbest) col = (s + 16) * part_width + key_col(kbest);
  col = row16_max_i32(col);
  int label = V;
  bool slow = false;
  if (j < n && !(vbest < thresh)) {
    if (cnt == 1 && vblank < thresh) label = col;
    else slow = true;
  }
  int n_recheck = 0;
  unsigned long long todo = __ballot(slow && s == 0);
  while (todo) {   // wave-uniform
    const int q = (__ffsll((long long)todo) - 1) >> 4;
    todo &= todo - 1;
    const int jq = __builtin_amdgcn_readlane(j, 16 * q), row = a * c.W + jq;
    float4 kk0 = no_keys();
    if (lane < nparts) { const float2 k2 = reload(row, lane); kk0.x = k2.x; kk0.y = k2.y; }
    int none = -1;
    float unused = 0.f;
    const int l = decide_row<WT, false, 2>(m, c, row, st.x, st.y + jq, nparts, nparts, part_width, readlane_f32(vblank, 16 * q),
                                        readlane_f32(znorm, 16 * q), kk0, n_recheck, false, none, unused);
    if ((lane >> 4) == q) label = l;
  }
  if (s == 0 && j < c.W) sh.label[j] = label;
  return n_recheck;
}

// Keys and row scalars of the first rows a wave decides, requested before anything else is known
// about the utterance so that they share the round trip of the slot table.
constexpr int kRowsAhead = 4;
struct RowsAhead {
  float4 kk0[kRowsAhead];
  float vb[kRowsAhead], zn[kRowsAhead];
};

// One utterance (slot a of the active list, state st = (utterance, t, len, sym), cnt labels so
// far), handled by the whole calling workgroup: one wave per window row (rows round-robin over the
// waves), then the first non-blank row by ballot and the pointer / hypothesis update of
// Algorithm 2.  nparts key pairs per row are valid, rows are `stride` pairs apart.  Ends with a
// workgroup barrier.
template <class WT, bool LOCAL, bool WIDE = false>
__device__ __forceinline__ void decide_utterance(const ModelDev &m, const CallDev &c, int a, int4 st, int cnt,
                                                 int exact_mode, int nparts, int stride, int part_width,
                                                 const RowsAhead &ahead, DecideShared &sh, bool write_out = true,
                                                 bool rows_done = false, int pre_recheck = 0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int b = st.x, t = st.y, len = st.z, V = m.V;
  const int n = min(c.W, len - t);
  int n_recheck = pre_recheck;   // rows_done: the caller has filled sh.label (see decide_rows_quad)
  if (threadIdx.x == 0) { sh.recheck = 0; sh.n_pend = 0; }
  __syncthreads();
  constexpr int KW = LOCAL ? 2 : 4;   // the resident loop kernel keeps two keys per part, the joint kernel three
  auto one_row = [&](int j, float4 k0, float vb, float zn) {
    int label = V, deferred = -1;
    float best = 0.f;
    if (j < n) {
      const int row = a * c.W + j;
      if constexpr (sizeof(WT) == 4) {   // fp32 models take the argmax in joint_exact_kernel
        label = c.row_label[row];
      } else {
        if (exact_mode) label = c.row_label[row];
        else label = decide_row<WT, WIDE, KW>(m, c, row, b, t + j, nparts, stride, part_width, vb, zn,
                                        lane < nparts ? k0 : no_keys(), n_recheck, !LOCAL, deferred, best);
      }
    }
    if (lane == 0) {
      sh.label[j] = label; sh.pend_part[j] = deferred; sh.pend_v[j] = best;
      if (deferred >= 0) atomicAdd(&sh.n_pend, 1);
    }
  };
#pragma unroll
  for (int q = 0; q < kRowsAhead; ++q) {
    const int j = wave + q * nwaves;
    if (!rows_done && j < c.W) one_row(j, ahead.kk0[q], ahead.vb[q], ahead.zn[q]);
  }
  for (int j = wave + kRowsAhead * nwaves; !rows_done && j < c.W; j += nwaves) {
    float4 k0 = no_keys();
    float vb = 0.f, zn = 0.f;
    if (!exact_mode && j < n) {
      const int row = a * c.W + j;
      if (lane < nparts) k0 = load_keys<KW>(c.parts, (size_t)row * stride + lane);
      vb = LOCAL ? sh.blank[row] : c.blank_logit[row];
      zn = LOCAL ? sh.znorm[row] : c.znorm[row];
    }
    one_row(j, k0, vb, zn);
  }
  if (lane == 0 && n_recheck) atomicAdd(&sh.recheck, n_recheck);
  __syncthreads();
  if constexpr (!LOCAL && sizeof(WT) == 2) {
    // Column parts left to the workgroup (a part's second key inside the near-tie band: all of its
    // columns are candidates).  Every wave takes four of the part's columns per round, so a part of 64
    // costs a 16-wave workgroup one trip to memory where the row's own wave would need sixteen.
    for (int j = 0; !rows_done && sh.n_pend > 0 && j < n; ++j) {
      const int part = sh.pend_part[j];   // the same for every thread
      if (part < 0) continue;
      const int col0 = part * part_width, ncol = min(part_width, V - col0);
      float bv = -INFINITY;
      int bi = 0x7FFFFFFF;
      if (4 * wave < ncol) {
        const float *er = c.e + ((size_t)b * c.T + t + j) * m.Hj, *pr = c.p + (size_t)b * m.Hj;
        constexpr int NZ = WIDE ? kDecideMaxHj / 128 : 8;
        float2 ev[NZ], pv[WIDE ? 1 : NZ];   // WIDE: the hidden vector is combined at once (fewer live registers)
#pragma unroll
        for (int i = 0; i < NZ; ++i) {
          const int k = 2 * lane + 128 * i;
          float2 e2 = make_float2(0.f, 0.f), p2 = make_float2(0.f, 0.f);
          if (k < m.Hj) {
            e2 = *reinterpret_cast<const float2 *>(er + k);
            p2 = *reinterpret_cast<const float2 *>(pr + k);
          }
          if constexpr (WIDE) {
            ev[i] = make_float2(fmaxf(e2.x + p2.x, 0.f), fmaxf(e2.y + p2.y, 0.f));
          } else {
            ev[i] = e2;
            pv[i] = p2;
          }
        }
        for (int c0 = 4 * wave; c0 < ncol; c0 += 4 * nwaves) {
          const int nc = min(4, ncol - c0), mycol = col0 + c0 + min(lane, nc - 1);
          if constexpr (WIDE) evaluate_candidates_wide<bf16_t, NZ>(m, ev, mycol, nc, lane, bv, bi);
          else evaluate_candidates<NZ>(m, ev, pv, mycol, nc, lane, bv, bi);
        }
      }
      if (lane == 0 && wave < 16) { sh.coop_v[wave] = bv; sh.coop_i[wave] = bi; }
      __syncthreads();
      if (threadIdx.x == 0) {
        float best = sh.pend_v[j];
        int label = sh.label[j];
        for (int w2 = 0; w2 < min(nwaves, 16); ++w2) {
          const float v = sh.coop_v[w2];
          const int i = sh.coop_i[w2];
          if (v > best || (v == best && i < label)) { best = v; label = i; }
        }
        sh.label[j] = label;
      }
      __syncthreads();
    }
  }
  if (wave == 0) {
    const bool nb = lane < n && sh.label[lane] != V;
    const unsigned long long mask = __ballot(nb);
    if (lane == 0) {
      const int i = mask ? __ffsll((long long)mask) - 1 : -1;   // smallest i with labels[i] != blank
      int tn = t, sym = st.w;
      int jump, emitted = 0, forced = 0, tok = V, overflow = 0;
      if (i < 0) {
        tn += n; sym = 0; jump = n;
      } else {
        tok = sh.label[i];
        if (cnt < c.cap) {
          if (write_out) {
            c.out_tokens[(size_t)b * c.cap + cnt] = tok;
            c.out_frames[(size_t)b * c.cap + cnt] = t + i;
          }
          ++cnt;
        } else {
          overflow = 1;
        }
        tn += i;
        sym = (i == 0) ? sym + 1 : 1;
        jump = i;
        emitted = 1;
        if (sym >= c.S) { tn += 1; sym = 0; jump += 1; forced = 1; }
      }
      if (emitted && write_out) c.out_counts[b] = cnt;
      const int active = tn < len;
      const int flag = active | ((emitted & active) << 1);
      // counters of this window, summed by the compacting wave: n (7 bits), useful rows (7), jump (7),
      // rechecks (7), emitted, forced, overflow
      const int useful = i < 0 ? n : i + 1;
      const unsigned ev = (unsigned)n | ((unsigned)useful << 7) | ((unsigned)jump << 14) |
                          ((unsigned)min(sh.recheck, 127) << 21) | ((unsigned)emitted << 28) |
                          ((unsigned)forced << 29) | ((unsigned)overflow << 30);
      if (LOCAL) {
        sh.flag[a] = flag; sh.tok[a] = tok; sh.event[a] = ev;
        sh.slot[a] = make_int4(b, tn, len, sym); sh.cnt[a] = cnt;
      } else {
        if (c.lists_atomic) {   // the calling kernel takes it from here
          sh.slot[0] = make_int4(b, tn, len, sym); sh.cnt[0] = cnt; sh.flag[0] = flag; sh.tok[0] = tok; sh.event[0] = ev;
        } else {
          c.res_state[a] = make_int4(b, tn, len, sym);
          c.res_aux[a] = make_int4(cnt, flag, tok, (int)ev);
        }
        sh.step_tok = (flag & 2) ? tok : -1;
      }
    }
  }
  __syncthreads();
}

// Builds the next iteration's slot table (other parity) and the emit list from the slots' outcomes,
// and adds the iteration's counters to the statistics.  Called by wave 0 of one workgroup per
// iteration, after every utterance has been decided and those writes have been fenced.
template <bool LOCAL>
__device__ __forceinline__ void compact_lists(const CallDev &c, int parity, int na, DecideShared &sh) {
  const int lane = threadIdx.x & 63;
  int4 *dst_state = c.slot_state + (parity ^ 1) * c.slot_stride;
  int *dst_count = c.slot_count + (parity ^ 1) * c.slot_stride;
  int n_act = 0, n_em = 0;
  unsigned sum_rows = 0, sum_useful = 0, sum_recheck = 0, sum_labels = 0, sum_forced = 0, sum_over = 0;
  // The slots' outcomes were written by other workgroups and come from the memory side: the reads of
  // two rounds of 64 slots go out together, so that they share one round trip.
  for (int base = 0; base < na; base += 128) {
    const int idx0 = base + lane, idx1 = base + 64 + lane;
    int4 st0 = make_int4(0, 0, 0, 0), st1 = st0, aux0 = st0, aux1 = st0;
    if (!LOCAL) {
      if (idx0 < na) { st0 = c.res_state[idx0]; aux0 = c.res_aux[idx0]; }
      if (idx1 < na) { st1 = c.res_state[idx1]; aux1 = c.res_aux[idx1]; }
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int idx = q ? idx1 : idx0;
      int4 st = q ? st1 : st0;
      const int4 aux = q ? aux1 : aux0;
      int f = 0, cnt = 0, tok = 0;
      if (idx < na) {
        unsigned ev;
        if (LOCAL) {
          st = sh.slot[idx]; cnt = sh.cnt[idx]; f = sh.flag[idx]; tok = sh.tok[idx]; ev = sh.event[idx];
        } else {
          cnt = aux.x; f = aux.y; tok = aux.z; ev = (unsigned)aux.w;
        }
        sum_rows += ev & 127u; sum_useful += (ev >> 7) & 127u; sum_recheck += (ev >> 21) & 127u;
        sum_labels += (ev >> 28) & 1u; sum_forced += (ev >> 29) & 1u; sum_over += (ev >> 30) & 1u;
        atomicAdd(&sh.hist[(ev >> 14) & 127u], 1u);
      }
      const unsigned long long ma = __ballot(f & 1), me = __ballot((f >> 1) & 1);
      const unsigned long long below = (1ull << lane) - 1ull;
      if (f & 1) {
        const int pos = n_act + __popcll(ma & below);
        dst_state[pos] = st;
        dst_count[pos] = cnt;
      }
      if (f & 2) {
        const int pos = n_em + __popcll(me & below);
        c.emit_idx[pos] = st.x;
        c.emit_list_tok[pos] = tok;
      }
      n_act += __popcll(ma);
      n_em += __popcll(me);
    }
  }
  sum_rows = (unsigned)wave_sum_i32((int)sum_rows); sum_useful = (unsigned)wave_sum_i32((int)sum_useful);
  sum_recheck = (unsigned)wave_sum_i32((int)sum_recheck); sum_labels = (unsigned)wave_sum_i32((int)sum_labels);
  sum_forced = (unsigned)wave_sum_i32((int)sum_forced); sum_over = (unsigned)wave_sum_i32((int)sum_over);
  // counters: additions that return nothing, so that the kernel's end does not wait for a read first
  for (int j = lane; j <= kMaxWindow; j += 64)
    if (sh.hist[j]) atomicAdd(&c.stats[kStatJump0 + j], (unsigned long long)sh.hist[j]);
  if (lane == 0) {
    c.n_active[parity ^ 1] = n_act;
    *c.n_emit = n_em;
    *c.ticket = 0u;
    atomicAdd(&c.stats[ST_ITER], 1ull); atomicAdd(&c.stats[ST_WINDOWS], (unsigned long long)na);
    atomicAdd(&c.stats[ST_ROWS], (unsigned long long)sum_rows); atomicAdd(&c.stats[ST_USEFUL], (unsigned long long)sum_useful);
    if (sum_recheck) atomicAdd(&c.stats[ST_RECHECK], (unsigned long long)sum_recheck);
    if (sum_labels) atomicAdd(&c.stats[ST_LABELS], (unsigned long long)sum_labels);
    if (sum_forced) atomicAdd(&c.stats[ST_FORCED], (unsigned long long)sum_forced);
    if (sum_over) atomicAdd(&c.stats[ST_OVERFLOW], (unsigned long long)sum_over);
  }
}

// Row argmax, first non-blank by ballot, pointer and hypothesis update, list compaction.
// One workgroup per active utterance; the last workgroup to finish rebuilds the lists.
// WIDE: joint hidden sizes above 1024 (the near-tie path then keeps the hidden vector in more registers).
template <class WT, bool WIDE>
__global__ __launch_bounds__(1024) void decide_kernel(ModelDev m, CallDev c, int parity, int exact_mode) {
  __shared__ DecideShared sh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int a = blockIdx.x;
  const long long ts0 = c.dbg ? wall_clock64() : 0;   // option "debug_stamps": where a launch's time goes
  // one round trip: the active count, this slot's state, and the keys / blank logit / norm of the
  // rows this wave decides (their addresses depend on the slot number only)
  const int na = c.n_active[parity];
  const int4 st = c.slot_state[parity * c.slot_stride + a];
  const int cnt = c.slot_count[parity * c.slot_stride + a];
  RowsAhead ahead;
#pragma unroll
  for (int q = 0; q < kRowsAhead; ++q) {
    const int j = wave + q * nwaves;
    ahead.kk0[q] = no_keys();
    ahead.vb[q] = 0.f; ahead.zn[q] = 0.f;
    if (!exact_mode && j < c.W) {
      const int row = a * c.W + j;
      if (lane < c.nparts) ahead.kk0[q] = load_keys<4>(c.parts, (size_t)row * c.nparts + lane);
      ahead.vb[q] = c.blank_logit[row];
      ahead.zn[q] = c.znorm[row];
    }
  }
  for (int j = threadIdx.x; j <= kMaxWindow; j += blockDim.x) sh.hist[j] = 0u;
  if (na == 0 && a == 0 && threadIdx.x == 0) c.n_active[parity ^ 1] = 0;  // keep both slots at "done"
  if (a >= na) return;
  decide_utterance<WT, false, WIDE>(m, c, a, st, cnt, exact_mode, c.nparts, c.nparts, c.part_width, ahead, sh);
  const long long ts1 = c.dbg ? wall_clock64() : 0;
  if (c.dbg && threadIdx.x == 0) {   // rows phase of workgroups with / without a near-tie
    atomicAdd((unsigned long long *)&c.dbg[sh.recheck ? 4 : 6], (unsigned long long)(ts1 - ts0));
    atomicAdd((unsigned long long *)&c.dbg[sh.recheck ? 5 : 7], 1ull);
  }
  // With the recurrent sums at hand, the first LSTM layer's step for this utterance's label is
  // elementwise: the label's row of input gate sums plus the recurrent sums, the gates, the new cell
  // and hidden vector (written in place: nothing reads the old ones any more).  Where the
  // last workgroup compacts the lists, it runs beside that, on the waves other than the compacting one.
  auto first_layer_step = [&](int first, int nthreads) {
    const int tok = sh.step_tok;
    if (c.rec == nullptr || tok < 0 || threadIdx.x < first) return;
    const int b = st.x, Hp = m.Hp;
    const float *xg = m.emb_gates + (size_t)tok * 4 * Hp, *rg = c.rec + (size_t)b * 4 * Hp;
    // up to four units per thread and pass, their loads requested together (one round trip per pass)
    for (int u0 = threadIdx.x - first; u0 < Hp; u0 += 4 * nthreads) {
      float4 x[4], r[4];
      float cp[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int u = u0 + i * nthreads;
        if (u < Hp) {
          x[i] = *reinterpret_cast<const float4 *>(xg + 4 * u);
          r[i] = *reinterpret_cast<const float4 *>(rg + 4 * u);
          cp[i] = c.c[(size_t)b * Hp + u];
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int u = u0 + i * nthreads;
        if (u >= Hp) continue;
        const size_t si = (size_t)b * Hp + u;
        const float ig = 1.f / (1.f + expf(-(r[i].x + x[i].x))), fg = 1.f / (1.f + expf(-(r[i].y + x[i].y)));
        const float og = 1.f / (1.f + expf(-(r[i].w + x[i].w)));
        const float cn = fg * cp[i] + ig * tanhf(r[i].z + x[i].z);
        c.c[si] = cn;
        store_hi_lo(c.hb_hi, c.hb_lo, si, og * tanhf(cn));
      }
    }
  };
  if (c.lists_atomic) {
    // No workgroup waits for the others: each claims its utterance's place in the next slot table and,
    // with a label, in the emit list, and adds its window's counters.  The order of the lists varies
    // from run to run; what is computed per utterance does not depend on it.
    if (threadIdx.x < 16) {
      const int4 ns = sh.slot[0];
      const int flag = sh.flag[0];
      const unsigned ev = sh.event[0];
      const int k = threadIdx.x;
      if (k == 0 && (flag & 1)) {
        const int pos = atomicAdd(&c.n_active[parity ^ 1], 1);
        c.slot_state[(parity ^ 1) * c.slot_stride + pos] = ns;
        c.slot_count[(parity ^ 1) * c.slot_stride + pos] = sh.cnt[0];
      }
      if (k == 1 && (flag & 2)) {
        const int pos = atomicAdd(c.n_emit, 1);
        c.emit_idx[pos] = ns.x;
        c.emit_list_tok[pos] = sh.tok[0];
      }
      unsigned long long add = 0ull;
      int which = -1;
      switch (k) {
        case 2: which = ST_WINDOWS; add = 1ull; break;
        case 3: which = ST_ROWS; add = ev & 127u; break;
        case 4: which = ST_USEFUL; add = (ev >> 7) & 127u; break;
        case 5: which = ST_RECHECK; add = (ev >> 21) & 127u; break;
        case 6: which = ST_LABELS; add = (ev >> 28) & 1u; break;
        case 7: which = ST_FORCED; add = (ev >> 29) & 1u; break;
        case 8: which = ST_OVERFLOW; add = (ev >> 30) & 1u; break;
        case 9: which = kStatJump0 + (int)((ev >> 14) & 127u); add = 1ull; break;
        case 10: which = ST_ITER; add = a == 0 ? 1ull : 0ull; break;
        default: break;
      }
      if (which >= 0 && add) atomicAdd(&c.stats[which], add);
    }
    // with enough waves, the one that waits for its claims' answers takes no part in the layer step
    if (nwaves >= 8) first_layer_step(64, blockDim.x - 64);
    else first_layer_step(0, blockDim.x);
    return;
  }
  if (threadIdx.x == 0) {
    __threadfence();
    const unsigned tk = atomicAdd(c.ticket, 1u);
    sh.is_last = (tk == (unsigned)(na - 1));
  }
  __syncthreads();
  if (!sh.is_last) {
    first_layer_step(0, blockDim.x);
    return;
  }
  const long long ts2 = c.dbg ? wall_clock64() : 0;
  if (nwaves > 1) first_layer_step(64, blockDim.x - 64);
  __threadfence();
  if (threadIdx.x < 64) compact_lists<false>(c, parity, na, sh);
  if (nwaves == 1) first_layer_step(0, blockDim.x);
  if (c.dbg && threadIdx.x == 0) {
    const long long ts3 = wall_clock64();
    c.dbg[0] += ts1 - ts0; c.dbg[1] += ts2 - ts1; c.dbg[2] += ts3 - ts2; c.dbg[3] += 1;
  }
}

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
template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) void lstm_layer_dma_kernel(ModelDev m, CallDev c, int layer, int pre) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
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
  float4 add_e[EPI];
#pragma unroll
  for (int q = 0; q < EPI; ++q) {
    const int idx = tid + q * Cfg::NT, r = min(idx / UB, R - 1), u = idx % UB;
    c_prev[q] = c.c[lofs + (size_t)ub_e[q] * Hp + (n0 >> 2) + u];
    add_e[q] = make_float4(bias[u], bias[UB + u], bias[2 * UB + u], bias[3 * UB + u]);
    if (layer == 0) add_e[q] = *reinterpret_cast<const float4 *>(m.emb_gates + (size_t)tok_e[q] * 4 * Hp + n0 + 4 * u);
    if (pre) {
      const float4 rs = *reinterpret_cast<const float4 *>(c.rec + ((size_t)layer * c.B + ub_e[q]) * 4 * Hp + n0 + 4 * u);
      add_e[q].x += rs.x; add_e[q].y += rs.y; add_e[q].z += rs.z; add_e[q].w += rs.w;
    }
    (void)r;
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
    const float gi = hi[0] + lo[0] + add_e[q].x;
    const float gf = hi[UB] + lo[UB] + add_e[q].y;
    const float gg = hi[2 * UB] + lo[2 * UB] + add_e[q].z;
    const float go = hi[3 * UB] + lo[3 * UB] + add_e[q].w;
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
struct LoopDev {
  unsigned *bar;       // word 0: abort; word (1 + g) * 32: barriers workgroup g has reached; all zero at launch
  float *h_x;          // [B][Hp] new hidden vectors
  float *p_x;          // [B][Hj] new projections
  float2 *parts_x;     // [2][32][nparts_tiny] keys, by iteration parity
  int G, upw, ppw;     // workgroups; LSTM units and W_pred rows per workgroup (multiples of 4)
  int max_iters;       // more iterations than any decode of this call can take
  unsigned spin_limit;
};
constexpr int kLoopMaxB = 2;
constexpr int kLoopRows = 32;

struct LoopShared {
  int4 nslot[kLoopMaxB];
  int ncnt[kLoopMaxB];
  int emit_ub[kLoopMaxB], emit_tok[kLoopMaxB];
  int n_act, n_emit, ok;
};

// LDS: [wl: upw*4 rows of Hp bf16][wp: ppw rows of Hp bf16][zs: 32 rows of Hj+8 bf16, at least 16 KB][hhi, hlo: B*Hp bf16 each]
//      [pfull: B*Hj f32][cst: B*upw f32]
// bf16 elements of the window-row region zs.  The region also takes the K-split partial sums of the MFMA
// phase (4 waves x 16 registers x 64 lanes of fp32 = 16 KB), which is the larger of the two for Hj < 248.
__host__ __device__ inline size_t loop_z_elems(int Hj) {
  const size_t z = (size_t)kLoopRows * (Hj + 8);
  return z > 8192 ? z : 8192;
}
__host__ __device__ inline size_t loop_smem_bytes(int Hp, int Hj, int B, int upw, int ppw) {
  return (size_t)upw * 4 * Hp * 2 + (size_t)ppw * Hp * 2 + loop_z_elems(Hj) * 2 + (size_t)B * Hp * 4 +
         (size_t)B * Hj * 4 + (size_t)B * upw * 4;
}

// Values that another workgroup of the running kernel wrote are read and written with agent-scope
// atomics (they go past the caches that are private to a CU or an XCD), so that the barrier needs
// no cache invalidation and the read-only operands stay in L2 from iteration to iteration.
__device__ __forceinline__ float ld_shared_f32(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_shared_f32(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_shared_f32x2(const float2 *p) {
  const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}
__device__ __forceinline__ void st_shared_f32x2(float2 *p, float2 v) {
  const unsigned long long u = (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kLoopFlagStride = 32;   // one 128-byte line per workgroup's arrival word
// The barrier in two halves, so that work that needs nothing from the other workgroups can fill the
// time the arrivals take to travel: loop_arrive publishes this workgroup's arrival, loop_wait waits
// for everybody's.  Between the two a workgroup must not write anything the others read before
// the barrier, nor read what they write.
__device__ __forceinline__ void loop_arrive(const LoopDev &lp, unsigned passed) {
  __syncthreads();   // this workgroup's stores of the phase have been issued and acknowledged
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // ... and are visible to the agent before the arrival is
    __hip_atomic_store(&lp.bar[(1 + blockIdx.x) * kLoopFlagStride], passed + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ __forceinline__ bool loop_wait(const LoopDev &lp, unsigned &passed, LoopShared &ls) {
  const unsigned epoch = ++passed;
  if (threadIdx.x < 64) {
    // every workgroup publishes the number of barriers it has reached; wave 0 watches all of them,
    // one lane per workgroup (no read-modify-write on a shared word: the arrivals do not queue up)
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
      const unsigned ab = __hip_atomic_load(lp.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (++spins > lp.spin_limit || ab) { good = 0; break; }
    }
    if (threadIdx.x == 0) {
      if (!good) __hip_atomic_store(lp.bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ls.ok = good;
    }
  }
  __syncthreads();
  asm volatile("" ::: "memory");   // the exchange reads that follow stay behind the wait
  return ls.ok != 0;
}
__device__ __forceinline__ bool loop_barrier(const LoopDev &lp, unsigned &passed, LoopShared &ls) {
  loop_arrive(lp, passed);
  return loop_wait(lp, passed, ls);
}

// Sums of 16 / 8 / 4 per-lane values over the wave with a halving exchange: each step a lane keeps
// half of its values and adds the partner's copies of them, until one value is left, which the
// last steps sum over the lanes that still hold parts of it.  The steps that carry the most values
// pair lanes inside a row of 16 with DPP permutations (row mirror, half mirror); the lane bit that
// decides which half is kept gives the value's index one bit per step:
//   16 values: index = b3 b2 b4 b5 (lane bits), i.e. value v ends up, complete, in the four lanes
//              32*(v&1) + 16*((v>>1)&1) + 4*(v>>2) + 0..3
//    8 values: index = b3 b2 b4; lanes 16*(v&1) + 4*(v>>1) + 0..3 and the same + 32
//    4 values: index = b3 b2; lanes 4*v + 0..3 of every row
__device__ __forceinline__ float wave_sum16_scatter(const float (&v)[16], int lane) {
  float a[8], b[4], c2[2];
  const bool u3 = (lane & 8) != 0, u2 = (lane & 4) != 0, u4 = (lane & 16) != 0, u5 = (lane & 32) != 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (u3 ? v[i + 8] : v[i]) + dpp_f32<kDppRowMirror>(u3 ? v[i] : v[i + 8]);
#pragma unroll
  for (int i = 0; i < 4; ++i) b[i] = (u2 ? a[i + 4] : a[i]) + dpp_f32<kDppRowHalfMirror>(u2 ? a[i] : a[i + 4]);
#pragma unroll
  for (int i = 0; i < 2; ++i) c2[i] = (u4 ? b[i + 2] : b[i]) + __shfl_xor(u4 ? b[i] : b[i + 2], 16, kWave);
  float d = (u5 ? c2[1] : c2[0]) + __shfl_xor(u5 ? c2[0] : c2[1], 32, kWave);
  d += dpp_f32<kDppQuadXor2>(d);
  d += dpp_f32<kDppQuadXor1>(d);
  return d;
}
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
__device__ __forceinline__ float wave_sum4_scatter(const float (&v)[4], int lane) {
  float a[2];
  const bool u3 = (lane & 8) != 0, u2 = (lane & 4) != 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) a[i] = (u3 ? v[i + 2] : v[i]) + dpp_f32<kDppRowMirror>(u3 ? v[i] : v[i + 2]);
  float d = (u2 ? a[1] : a[0]) + dpp_f32<kDppRowHalfMirror>(u2 ? a[0] : a[1]);
  d += __shfl_xor(d, 16, kWave);
  d += __shfl_xor(d, 32, kWave);
  d += dpp_f32<kDppQuadXor2>(d);
  d += dpp_f32<kDppQuadXor1>(d);
  return d;
}

__global__ __launch_bounds__(256) void wind_loop_kernel(ModelDev m, CallDev c, LoopDev lp) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  __shared__ DecideShared sh;
  __shared__ LoopShared ls;
  __shared__ unsigned long long lstats[kNumStats];   // workgroup 0: the call's counters, written out at the end
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = blockIdx.x;
  const int Hj = m.Hj, Hp = m.Hp, W = c.W, B = c.B;
  const int zstride = Hj + 8;
  bf16_t *wl = reinterpret_cast<bf16_t *>(smem_raw);
  bf16_t *wp = wl + (size_t)lp.upw * 4 * Hp;
  bf16_t *zs = wp + (size_t)lp.ppw * Hp;
  // the hidden vectors as bf16 hi + lo (hi = RNE(h), lo = RNE(h - hi), 16 mantissa bits together): the dot
  // products with the bf16 weights then take one packed instruction per pair and part, with nothing to unpack
  bf16_t *hhi = zs + loop_z_elems(Hj), *hlo = hhi + (size_t)B * Hp;
  float *pfull = reinterpret_cast<float *>(hlo + (size_t)B * Hp);
  auto put_h2 = [&](int i, float2 v) {   // elements i (even) and i + 1
    const uint32_t hb = pack_bf16x2(v.x, v.y);
    *reinterpret_cast<uint32_t *>(hhi + i) = hb;
    *reinterpret_cast<uint32_t *>(hlo + i) = pack_bf16x2(v.x - __uint_as_float(hb << 16), v.y - __uint_as_float(hb & 0xFFFF0000u));
  };
  // sum over this lane's eight k of w[k] * (hi[k] + lo[k]), on top of acc
  auto dot8 = [&](const bf16_t *wrow, int hofs, float acc) {
    const u32x4 wv = *reinterpret_cast<const u32x4 *>(wrow);
    const u32x4 a = *reinterpret_cast<const u32x4 *>(hhi + hofs), b = *reinterpret_cast<const u32x4 *>(hlo + hofs);
    acc = dot2_bf16(wv.x, a.x, acc); acc = dot2_bf16(wv.y, a.y, acc); acc = dot2_bf16(wv.z, a.z, acc); acc = dot2_bf16(wv.w, a.w, acc);
    acc = dot2_bf16(wv.x, b.x, acc); acc = dot2_bf16(wv.y, b.y, acc); acc = dot2_bf16(wv.z, b.z, acc); acc = dot2_bf16(wv.w, b.w, acc);
    return acc;
  };
  float *cst = pfull + (size_t)B * Hj;

  // ---- once: this workgroup's weights, the state after the start-token step, the slot table
  const int unit0 = g * lp.upw, prow0 = g * lp.ppw;
  for (int i = tid * 8; i < lp.upw * 4 * Hp; i += 256 * 8) {
    const int row = i / Hp, k = i - row * Hp;           // row = 4 * local unit + gate
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (unit0 + (row >> 2) < Hp)
      v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const bf16_t *>(m.w_cat[0]) + ((size_t)unit0 * 4 + row) * Hp + k);
    *reinterpret_cast<u32x4 *>(wl + i) = v;
  }
  for (int i = tid * 8; i < lp.ppw * Hp; i += 256 * 8) {
    const int row = i / Hp, k = i - row * Hp;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (prow0 + row < Hj) v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const bf16_t *>(m.w_pred) + (size_t)(prow0 + row) * Hp + k);
    *reinterpret_cast<u32x4 *>(wp + i) = v;
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
  float warm = 0.f, pend[2] = {0.f, 0.f};
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
  const bf16_t *wrow = reinterpret_cast<const bf16_t *>(m.w_out) + (size_t)(n0 + (lane & 31)) * Hj + k0 + (lane >> 5) * 8;
  bf16x8 bfrag[kTinyPrefetch];
#pragma unroll
  for (int i = 0; i < kTinyPrefetch; ++i)
    if (i < nk) bfrag[i] = *reinterpret_cast<const bf16x8 *>(wrow + i * 16);
  const int cip = lane & 31, col = n0 + cip;
  const bool col_ok = has_cols && col < m.V;
  const float col_bias = col_ok ? m.b_out[col_ok ? col : 0] : kKeyNone;
  const float b_blank = m.b_out[m.V];
  CallDev cl = c;   // the decision code reads the keys through parts and, for near-ties, the current projections through p
  cl.p = pfull;
  cl.parts = reinterpret_cast<float *>(zs);   // the iteration's keys are copied over the window rows once those are used up
  constexpr int KI = kTinyMaxHj / 256;
  float4 wblank[KI];
#pragma unroll
  for (int i = 0; i < KI; ++i) {
    const int k = lane * 4 + 256 * i;
    wblank[i] = k < Hj ? *reinterpret_cast<const float4 *>(m.w_blank + k) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  unsigned passed = 0;
  __syncthreads();
  // The recurrent half of the gate sums, W_hh h, depends on the hidden vector only, which changes
  // when its utterance emits: it is formed as soon as the new vector is here (while the arrivals of
  // the projection exchange travel), so that a step, once the label is known, only adds the
  // label's row of input sums.  rec[b]: this wave's 16 (unit, gate) sums for utterance b, value
  // 4q + gate in lanes 4q + 16*(gate>>1) + 32*(gate&1) + 0..3.
  auto recurrent_sums = [&](int ub) {
    float part[16];   // [unit q][gate]
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int u = wave + 4 * q;
#pragma unroll
      for (int gate = 0; gate < 4; ++gate) part[4 * q + gate] = 0.f;
      if (u >= lp.upw) continue;
      for (int k = lane * 8; k < Hp; k += 512) {
#pragma unroll
        for (int gate = 0; gate < 4; ++gate)
          part[4 * q + gate] = dot8(wl + ((size_t)u * 4 + gate) * Hp + k, ub * Hp + k, part[4 * q + gate]);
      }
    }
    return wave_sum16_scatter(part, lane);
  };
  float rec[kLoopMaxB];
#pragma unroll
  for (int b = 0; b < kLoopMaxB; ++b) rec[b] = b < B ? recurrent_sums(b) : 0.f;

  const bool dbg = c.dbg != nullptr && g == 0 && tid == 0;
  long long tsum[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, n_it = 0, n_em_it = 0;
  for (int it = 0; it < lp.max_iters && na > 0; ++it) {
    const int par = it & 1;
    const long long t0 = dbg ? wall_clock64() : 0;
    const int n_rows = na * W;
    float2 *parts = lp.parts_x + (size_t)par * kLoopRows * c.nparts_tiny;
    for (int j = tid; j <= kMaxWindow; j += 256) sh.hist[j] = 0u;
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
          er = c.e + ((size_t)st.x * c.T + (valid[q] ? st.y + j : 0)) * Hj;
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
    // Touch the lines of the window after this one (every XCD's L2 wants its own copy).  The values
    // are consumed one iteration later, so that no wave ever waits for these loads.
    {
      warm += pend[0] + pend[1];
      pend[0] = 0.f; pend[1] = 0.f;
      const int lines_per_row = (Hj * 4 + 127) / 128;   // at most 32: eight rows per step, 32 lanes each
      for (int a = 0; a < na; ++a) {
        const int4 st = sh.slot[a];
        const int t_first = st.y + W, t_end = min(st.y + 2 * W, st.z);
        const int l = tid & 31;
        for (int tr = t_first + (tid >> 5), i2 = 0; tr < t_end; tr += 8, ++i2)
          if (l < lines_per_row) pend[i2 & 1] += c.e[((size_t)st.x * c.T + tr) * Hj + l * 32];
      }
    }
    __syncthreads();
    const long long t1 = dbg ? wall_clock64() : 0;
    // ---- this workgroup's 32 columns: K split over the four waves, W_out from registers
    if (has_cols) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      const bf16_t *zrow = zs + (size_t)(lane & 31) * zstride + k0 + (lane >> 5) * 8;
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
        st_shared_f32x2(&parts[(size_t)acc_row(0, s0, lane) * c.nparts_tiny + g], make_float2(o1[0], o2[0]));
      }
    }
    const long long t2 = dbg ? wall_clock64() : 0;
    if (!loop_barrier(lp, passed, ls)) return;            // exchange 1: every row's keys are in memory
    const long long t3 = dbg ? wall_clock64() : 0;
    // ---- the decisions, taken alike by every workgroup; workgroup 0 writes the outputs
    // With at most 64 parts per row and 4 rows per wave the decision only looks at the keys its
    // caller hands it, which are read here straight from the exchange buffer; otherwise the keys
    // are copied to LDS first.
    float2 *lparts = reinterpret_cast<float2 *>(zs);
    const bool direct = c.nparts_tiny <= 64 && W <= 4 * kRowsAhead;
    if (!direct) {
      for (int i = tid; i < n_rows * c.nparts_tiny; i += 256) lparts[i] = ld_shared_f32x2(parts + i);
      __syncthreads();
    }
    const bool quad = direct && c.nparts_tiny <= 32;   // four rows per wave decided at once
    for (int a = 0; a < na; ++a) {
      RowsAhead ahead;
      if (quad) {
        const int s = lane & 15, j = wave + (lane >> 4) * 4, row = a * W + j;
        float2 kA = make_float2(kKeyNone, kKeyNone), kB = kA;
        float vb = 0.f, zn = 0.f;
        if (j < W) {
          if (s < c.nparts_tiny) kA = ld_shared_f32x2(parts + (size_t)row * c.nparts_tiny + s);
          if (s + 16 < c.nparts_tiny) kB = ld_shared_f32x2(parts + (size_t)row * c.nparts_tiny + s + 16);
          vb = sh.blank[row];
          zn = sh.znorm[row];
        }
        auto reload = [&](int r, int part) { return ld_shared_f32x2(parts + (size_t)r * c.nparts_tiny + part); };
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
    const int n_emit = ls.n_emit;
    if (tid < na) { sh.slot[tid] = ls.nslot[tid]; sh.cnt[tid] = ls.ncnt[tid]; }
    __syncthreads();
    const long long t4 = dbg ? wall_clock64() : 0;
    if (dbg) { tsum[0] += t1 - t0; tsum[1] += t2 - t1; tsum[2] += t3 - t2; tsum[3] += t4 - t3; ++n_it; }
    if (n_emit == 0 || na == 0) continue;
    // ---- one LSTM step for the utterances that emitted: this workgroup's units, weights from LDS
    for (int r = 0; r < n_emit; ++r) {
      const int ub = ls.emit_ub[r], tok = ls.emit_tok[r];
      // the label's input gate sums of this wave's (at most four) units: one round trip for all
      float4 addq[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int unit = unit0 + wave + 4 * q;
        addq[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (wave + 4 * q < lp.upw && unit < Hp) addq[q] = *reinterpret_cast<const float4 *>(m.emb_gates + (size_t)tok * 4 * Hp + unit * 4);
      }
      // the recurrent sums were formed when this utterance's hidden vector last changed: every gate's
      // nonlinearity runs on its own lanes, then lane 4q gathers its unit's four
      float tot = rec[0];
#pragma unroll
      for (int b = 1; b < kLoopMaxB; ++b) tot = ub == b ? rec[b] : tot;
      const int q = (lane >> 2) & 3, gate = ((lane >> 4) & 1) * 2 + (lane >> 5);
      float4 aq = addq[0];
      if (q == 1) aq = addq[1];
      if (q == 2) aq = addq[2];
      if (q == 3) aq = addq[3];
      const float pre = tot + (gate == 0 ? aq.x : gate == 1 ? aq.y : gate == 2 ? aq.z : aq.w);
      const float act = gate == 2 ? tanhf(pre) : 1.f / (1.f + expf(-pre));
      const int base = lane & 12;
      const float ig = __shfl(act, base, kWave), fg = __shfl(act, base + 32, kWave);
      const float gg = __shfl(act, base + 16, kWave), og = __shfl(act, base + 48, kWave);
      const int u = wave + 4 * q, unit = unit0 + u;
      if ((lane & 0x33) == 0 && u < lp.upw && unit < Hp) {
        const float cn = fg * cst[ub * lp.upw + u] + ig * gg;
        cst[ub * lp.upw + u] = cn;
        st_shared_f32(&lp.h_x[(size_t)ub * Hp + unit], og * tanhf(cn));
      }
    }
    const long long t5 = dbg ? wall_clock64() : 0;
    if (!loop_barrier(lp, passed, ls)) return;            // exchange 2: the new hidden vectors
    const long long t6 = dbg ? wall_clock64() : 0;
    for (int r = 0; r < n_emit; ++r) {
      const int ub = ls.emit_ub[r];
      for (int k = tid * 2; k < Hp; k += 512) put_h2(ub * Hp + k, ld_shared_f32x2(reinterpret_cast<const float2 *>(&lp.h_x[(size_t)ub * Hp + k])));
    }
    __syncthreads();
    // ---- this workgroup's rows of the prediction projection
    for (int r = 0; r < n_emit; ++r) {
      const int ub = ls.emit_ub[r];
      // this wave's rows jl = wave + 4q, q < ppw / 4, four at a time
      for (int q0 = 0; q0 * 4 < lp.ppw; q0 += 4) {
        float part[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int jl = wave + 4 * (q0 + q);
          part[q] = 0.f;
          if (jl >= lp.ppw) continue;
          for (int k = lane * 8; k < Hp; k += 512) part[q] = dot8(wp + (size_t)jl * Hp + k, ub * Hp + k, part[q]);
        }
        const float tot = wave_sum4_scatter(part, lane);   // lanes 4q .. 4q+3 of every row of 16 hold row q's sum
        const int jl = wave + 4 * (q0 + ((lane >> 2) & 3)), j = prow0 + jl;
        if ((lane & 0x33) == 0 && jl < lp.ppw && j < Hj) st_shared_f32(&lp.p_x[(size_t)ub * Hj + j], tot + m.b_pred[j]);
      }
    }
    const long long t7 = dbg ? wall_clock64() : 0;
    loop_arrive(lp, passed);                              // exchange 3: the new projections ...
    for (int r = 0; r < n_emit; ++r) {                    // ... and, while the arrivals travel, the next step's recurrent sums
      const int ub = ls.emit_ub[r];
      const float v = recurrent_sums(ub);
#pragma unroll
      for (int b = 0; b < kLoopMaxB; ++b) rec[b] = ub == b ? v : rec[b];
    }
    if (!loop_wait(lp, passed, ls)) return;
    const long long t8 = dbg ? wall_clock64() : 0;
    for (int r = 0; r < n_emit; ++r) {
      const int ub = ls.emit_ub[r];
      for (int k = tid; k < Hj; k += 256) pfull[(size_t)ub * Hj + k] = ld_shared_f32(&lp.p_x[(size_t)ub * Hj + k]);
    }
    __syncthreads();
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
    for (int i = tid; i < kNumStats; i += 256) c.stats[i] = lstats[i];
    if (tid == 0) {
      c.n_active[0] = na;   // zero unless max_iters ran out
      c.n_active[1] = na;
    }
  }
  if (warm == 1.2345e-30f && lp.spin_limit == 0u) lp.h_x[0] = warm;   // keeps the warming loads alive; never true
}

}  // namespace wind
