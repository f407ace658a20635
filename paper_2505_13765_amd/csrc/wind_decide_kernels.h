// The decision: row argmax from the keys with near-ties re-decided in fp32, first non-blank row, pointer and
// hypothesis update, the lists of the next iteration, and the first LSTM layer's step.
#pragma once
#include "wind_types.h"

namespace wind {

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
                                           int stride, int part_width, float vblank, float thresh, float4 kk0, bool have1, float4 kk1,
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
    else if (have1 && p0 == 64) kk = kk1;
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
                                                int stride, int part_width, float vblank, float thresh, float4 kk0, bool have1, float4 kk1,
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
    else if (have1 && p0 == 64) kk = kk1;
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
// rows at once so that the loads overlap); parts 64 and up are read here, except that with have1 the
// caller also brings kk1, the keys of part lane + 64 (all there is to read for up to 128 parts: the
// row then costs no second trip to memory).
template <class WT, bool WIDE, int KW>
__device__ __forceinline__ int decide_row(const ModelDev &m, const CallDev &c, int row, int b, int frame,
                                          int nparts, int stride, int part_width, float vblank, float znorm,
                                          float4 kk0, bool have1, float4 kk1, int &n_recheck, bool defer, int &deferred,
                                          float &best_out) {
  const int lane = threadIdx.x & 63, V = m.V;
  const size_t prow = (size_t)row * stride;
  auto keys_at = [&](int pi) -> float4 { return have1 && pi == lane + 64 ? kk1 : load_keys<KW>(c.parts, prow + pi); };
  float k1 = kk0.x;
  for (int pi = lane + 64; pi < nparts; pi += 64) k1 = fmaxf(k1, keys_at(pi).x);
  const float kbest = wave_max_f32(k1);
  const float vbest = key_val(kbest);
  const float top = fmaxf(vbest, vblank);
  const float tau = m.tau_scale * znorm + 6.2e-5f * fabsf(top);
  const float thresh = top - tau;
  if (vbest < thresh) return V;                  // blank clear of every label
  // how many label keys are inside the band?
  int cnt = (key_val(kk0.x) >= thresh) + (key_val(kk0.y) >= thresh) + (key_val(kk0.z) >= thresh);
  for (int pi = lane + 64; pi < nparts; pi += 64) {
    const float4 kk = keys_at(pi);
    cnt += (key_val(kk.x) >= thresh) + (key_val(kk.y) >= thresh) + (key_val(kk.z) >= thresh);
  }
  cnt = wave_sum_i32(cnt);
  if (cnt == 1 && vblank < thresh) {
    // a single label clear of blank and of every other label: find its part
    int col = kk0.x == kbest ? lane * part_width + key_col(kbest) : -1;
    for (int pi = lane + 64; pi < nparts; pi += 64)
      if (keys_at(pi).x == kbest) col = pi * part_width + key_col(kbest);
    return wave_max_i32(col);
  }
  // near tie: fp32 logits of every candidate, hidden vector rebuilt from fp32 e and p
  ++n_recheck;
  if constexpr (WIDE)
    return recheck_row_wide<KW>(m, c, row, b, frame, nparts, stride, part_width, vblank, thresh, kk0, have1, kk1, defer, deferred,
                                best_out);
  else
    return recheck_row<8, KW>(m, c, row, b, frame, nparts, stride, part_width, vblank, thresh, kk0, have1, kk1, defer, deferred,
                              best_out);
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
                                        readlane_f32(znorm, 16 * q), kk0, false, no_keys(), n_recheck, false, none, unused);
    if ((lane >> 4) == q) label = l;
  }
  if (s == 0 && j < c.W) sh.label[j] = label;
  return n_recheck;
}

// Keys and row scalars of the first rows a wave decides, requested before anything else is known
// about the utterance so that they share the round trip of the slot table.
// TWO: also the keys of part lane + 64 (rows of 65 .. 128 parts), for a wave that decides a single row.
constexpr int kRowsAhead = 4;
template <int N, bool TWO>
struct RowsAheadT {
  static constexpr int kRows = N;
  static constexpr bool kTwo = TWO;
  float4 kk0[N];
  float4 kk1[TWO ? N : 1];
  float vb[N], zn[N];
};
using RowsAhead = RowsAheadT<kRowsAhead, false>;

// What a decided window does to its utterance (Algorithm 2's update, with the cap on labels per frame):
// i = the smallest row whose label is not blank (label_i), or -1; n = rows of the window.  Writes the
// label and its frame to the outputs if write_out.  Returns the new state (utterance, t, len, labels
// on the frame), the label count, flag (bit 0: the utterance goes on, bit 1: it goes on and emitted),
// the label, and the window's counters packed into one word: n (7 bits), useful rows (7), jump (7),
// rechecks (7), emitted, forced on, overflow.
struct WindowOutcome {
  int4 slot;
  int cnt, flag, tok;
  unsigned ev;
};
__device__ __forceinline__ WindowOutcome window_outcome(const CallDev &c, int4 st, int cnt, int n, int i, int label_i, int V,
                                                        int recheck, bool write_out) {
  const int b = st.x, t = st.y, len = st.z;
  int tn = t, sym = st.w;
  int jump, emitted = 0, forced = 0, tok = V, overflow = 0;
  if (i < 0) {
    tn += n; sym = 0; jump = n;
  } else {
    tok = label_i;
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
  WindowOutcome wo;
  wo.slot = make_int4(b, tn, len, sym);
  wo.cnt = cnt;
  wo.flag = active | ((emitted & active) << 1);
  wo.tok = tok;
  const int useful = i < 0 ? n : i + 1;
  wo.ev = (unsigned)n | ((unsigned)useful << 7) | ((unsigned)jump << 14) | ((unsigned)min(recheck, 127) << 21) |
          ((unsigned)emitted << 28) | ((unsigned)forced << 29) | ((unsigned)overflow << 30);
  return wo;
}

// One utterance (slot a of the active list, state st = (utterance, t, len, sym), cnt labels so
// far), handled by the whole calling workgroup: one wave per window row (rows round-robin over the
// waves), then the first non-blank row by ballot and the pointer / hypothesis update of
// Algorithm 2.  nparts key pairs per row are valid, rows are `stride` pairs apart.  Ends with a
// workgroup barrier.
template <class WT, bool LOCAL, bool WIDE = false, class RA = RowsAhead>
__device__ __forceinline__ void decide_utterance(const ModelDev &m, const CallDev &c, int a, int4 st, int cnt,
                                                 int exact_mode, int nparts, int stride, int part_width,
                                                 const RA &ahead, DecideShared &sh, bool write_out = true,
                                                 bool rows_done = false, int pre_recheck = 0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int b = st.x, t = st.y, len = st.z, V = m.V;
  const int n = min(c.W, len - t);
  int n_recheck = pre_recheck;   // rows_done: the caller has filled sh.label (see decide_rows_quad)
  if (threadIdx.x == 0) { sh.recheck = 0; sh.n_pend = 0; }
  __syncthreads();
  constexpr int KW = LOCAL ? 2 : 4;   // the resident loop kernel keeps two keys per part, the joint kernel three
  auto one_row = [&](int j, float4 k0, bool have1, float4 k1, float vb, float zn) {
    int label = V, deferred = -1;
    float best = 0.f;
    if (j < n) {
      const int row = a * c.W + j;
      if constexpr (sizeof(WT) == 4) {   // fp32 models take the argmax in joint_exact_kernel
        label = c.row_label[row];
      } else {
        if (exact_mode) label = c.row_label[row];
        else label = decide_row<WT, WIDE, KW>(m, c, row, b, t + j, nparts, stride, part_width, vb, zn,
                                        lane < nparts ? k0 : no_keys(), have1, k1, n_recheck, !LOCAL, deferred, best);
      }
    }
    if (lane == 0) {
      sh.label[j] = label; sh.pend_part[j] = deferred; sh.pend_v[j] = best;
      if (deferred >= 0) atomicAdd(&sh.n_pend, 1);
    }
  };
#pragma unroll
  for (int q = 0; q < RA::kRows; ++q) {
    const int j = wave + q * nwaves;
    float4 k1 = no_keys();
    if constexpr (RA::kTwo) k1 = ahead.kk1[q];
    if (!rows_done && j < c.W) one_row(j, ahead.kk0[q], RA::kTwo, k1, ahead.vb[q], ahead.zn[q]);
  }
  for (int j = wave + RA::kRows * nwaves; !rows_done && j < c.W; j += nwaves) {
    float4 k0 = no_keys();
    float vb = 0.f, zn = 0.f;
    if (!exact_mode && j < n) {
      const int row = a * c.W + j;
      if (lane < nparts) k0 = load_keys<KW>(c.parts, (size_t)row * stride + lane);
      vb = LOCAL ? sh.blank[row] : c.blank_logit[row];
      zn = LOCAL ? sh.znorm[row] : c.znorm[row];
    }
    one_row(j, k0, false, no_keys(), vb, zn);
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
      const WindowOutcome wo = window_outcome(c, st, cnt, n, i, i < 0 ? V : sh.label[i], V, sh.recheck, write_out);
      const int tn = wo.slot.y, sym = wo.slot.w, flag = wo.flag, tok = wo.tok;
      const unsigned ev = wo.ev;
      cnt = wo.cnt;
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
// TWO: rows of 65 .. 128 column parts in windows of at most one row per wave: each wave asks for both halves
// of its row's keys in the first round trip (and for no rows beyond its first, which it does not have).
template <class WT, bool WIDE, bool TWO = false>
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
  using RA = RowsAheadT<TWO ? 1 : kRowsAhead, TWO>;
  RA ahead;
#pragma unroll
  for (int q = 0; q < RA::kRows; ++q) {
    const int j = wave + q * nwaves;
    ahead.kk0[q] = no_keys();
    if (TWO) ahead.kk1[q] = no_keys();
    ahead.vb[q] = 0.f; ahead.zn[q] = 0.f;
    if (!exact_mode && j < c.W) {
      const int row = a * c.W + j;
      if (lane < c.nparts) ahead.kk0[q] = load_keys<4>(c.parts, (size_t)row * c.nparts + lane);
      if (TWO && lane + 64 < c.nparts) ahead.kk1[q] = load_keys<4>(c.parts, (size_t)row * c.nparts + lane + 64);
      ahead.vb[q] = c.blank_logit[row];
      ahead.zn[q] = c.znorm[row];
    }
  }
  for (int j = threadIdx.x; j <= kMaxWindow; j += blockDim.x) sh.hist[j] = 0u;
  if (na == 0 && a == 0 && threadIdx.x == 0) c.n_active[parity ^ 1] = 0;  // keep both slots at "done"
  if (a >= na) return;
  decide_utterance<WT, false, WIDE, RA>(m, c, a, st, cnt, exact_mode, c.nparts, c.nparts, c.part_width, ahead, sh);
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
        const float hv = og * tanhf(cn);
        store_hi_lo(c.hb_hi, c.hb_lo, si, hv);
        if (c.slot_rows) store_hi_lo(c.hbn_hi, c.hbn_lo, (size_t)a * Hp + u, hv);   // the layer's row of this SLOT
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
    // what the prediction-network launches need to know about this slot's row
    if (c.slot_rows && threadIdx.x == 32) reinterpret_cast<int *>(c.res_aux)[a] = sh.step_tok >= 0 ? st.x : -1;
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

}  // namespace wind
