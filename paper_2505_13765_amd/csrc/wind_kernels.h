// Device kernels of the WIND greedy decoder (gfx950).  See include/wind.h for the model.
//
// One loop iteration (Method, Algorithm 2, all active utterances at once), bf16 models:
//   build_z        window gather: z[r,j,:] = relu(e[b, t_b + j, :] + p[b,:]) in bf16, plus the
//                  blank logit and the norm of every row in fp32
//   joint_ws /     label logits of every window row on bf16 MFMA; per row and per 64-column part
//   joint_wide     the three largest (logit, column) keys are kept, nothing else is stored.  Tiles
//                  whose height (64 to 256 rows) and number per workgroup follow the iteration's
//                  row count: 128 columns wide, four waves of a workgroup multiplying and four
//                  fetching (joint_ws), or, in iterations with many rows, 256 columns wide on four
//                  waves of up to 512 registers that do both (joint_wide; build_z then writes z in
//                  slabs of 32 hidden units)
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
#include "wind_types.h"
#include "wind_enc_kernels.h"
#include "wind_joint_kernels.h"
#include "wind_decide_kernels.h"
#include "wind_pred_kernels.h"
#include "wind_loop_kernel.h"
