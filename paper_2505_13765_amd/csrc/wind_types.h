// Constants, the model as it sits on the device (ModelDev) and the arrays of one decode call (CallDev).
#pragma once
#include "wind_mfma.h"
#include "wind_mfma_dma.h"
#include "wind_mfma_ws.h"
#include "wind_mfma_wide.h"

namespace wind {

constexpr int kMaxLayers = 4;
constexpr int kMaxWindow = 64;
constexpr int kTinyRows = 64;   // slots the resident loop kernel keeps in LDS (it runs far fewer)
constexpr int kStatJump0 = 9;  // index of jump_hist[0] in the device counter array
constexpr int kNumStats = kStatJump0 + kMaxWindow + 1;
enum { ST_ITER = 0, ST_WINDOWS, ST_ROWS, ST_USEFUL, ST_LABELS, ST_FORCED, ST_RECHECK, ST_OVERFLOW, ST_WIDE };   // ST_WIDE: iterations with more window rows than the gather kernel was told

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
  const void *w_enc_slab;       // bf16 models: the same matrix in slabs of 32 inputs, [D / 32][Hj_pad][32] (wide tiles), or null
  const float *b_enc;           // [Hj]
  const void *w_pred;           // [Hj, Hp]
  const float *b_pred;          // [Hj]
  const void *w_out;            // [Vpad, Hj]; row V = blank
  const void *w_out_slab;       // bf16 models: the same matrix in slabs of 32 K values, [Hj / 32][Vpad][32] (wide joint tiles)
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
  bf16_t *enc_b;                // [B*T + 256, D] encoder outputs rounded to bf16 (large calls only, else null); for
                                //   enc_proj_wide_kernel in slabs of 32 inputs, [D / 32][B*T + 256][32]
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
  int slot_rows;                // 1 (large batches of models with more than one layer, with rec and lists_atomic): the LSTM
                                //    launches of the layers above the first take their rows by SLOT: row a = the a-th active
                                //    utterance of the iteration, whether it emitted or not.  Its new hidden vectors sit in
                                //    hbn_*[layer][a], and word a of res_aux (as ints) is the utterance if it steps, else -1:
                                //    a launch can ask for its operand rows before it knows anything about the iteration
  float *h, *c, *hn;            // [L][B][Hp]
  bf16_t *hb_hi, *hb_lo, *hbn_hi, *hbn_lo;  // [L][B][Hp] large-batch path: h and new h as bf16 hi + lo
  const bf16_t *hb_zero;        // [max(E,Hp)] zeros (the lo part of an embedding row)
  // Large batches: the recurrent half of every layer's gate sums, w_hh . h, for the hidden vectors as
  // they stand (row order 4*unit + gate, no bias).  It changes only when its utterance emits, and it is
  // renewed beside the projection of that step, so the next step, once its label is known, has only
  // the input half left to do.  Null where this is not used (the full products are then formed per step).
  float *rec;                   // [L][B][4Hp]
  float *p;                     // [B][Hj]
  bf16_t *z;                    // [Mpad][Hj]; in iterations that run joint_wide_kernel, slabs of 32 K values: [Hj / 32][Mpad][32]
  float *blank_logit;           // [Mpad]
  float *znorm;                 // [Mpad]
  // Keys: per window row and column part the largest (logit, column) keys of the part.  The joint kernel
  // writes three per entry (four words, the last unused); the resident loop kernel keeps two (two words).
  float *parts;                 // [Mpad][nparts][4] (joint kernel) or [rows][nparts_tiny][2] (loop kernel)
  int nparts;                   // parts per row and label columns per part, as written by the joint kernel
  int part_width;
  int nparts_tiny;              // parts per row of the resident loop kernel (32 columns each)
  int Mpad;                     // rows of z, blank_logit, znorm, parts
  int *row_label;               // [Mpad] (fp32 models)
  unsigned long long *stats;    // [kNumStats]
  long long *dbg;               // optional [8] phase time stamps of the few-rows kernel's deciding workgroup (100 MHz clock)
  int *iter_rows;               // optional [iter_rows_cap] window rows of every loop iteration, in order (profile mode)
  int iter_rows_cap;
};

}  // namespace wind
