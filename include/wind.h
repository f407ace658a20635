/*
 * wind.h — C ABI of the MI355X (gfx950) WIND greedy decoder for RNN-T models.
 *
 * The library decodes a batch of encoder outputs with windowed non-blank detection: for every
 * active utterance the joint network is evaluated on up to W consecutive encoder frames against
 * the current prediction-network output, each row is argmaxed, the pointer jumps to the first
 * non-blank row, that label is emitted and the prediction network takes one step (Method,
 * Algorithm 2; its result equals the frame-by-frame loop of Algorithm 1).  All utterances of a
 * batch advance together, each with its own frame pointer.
 *
 * Model (the paper names only "encoder, decoder, joiner"; this is the usual RNN-T factorisation):
 *   joiner(f, g) = W_out relu(W_enc f + b_enc + W_pred g + b_pred) + b_out  -> V+1 logits
 *   decoder      = embedding [V+1, E] + L stacked LSTM cells (gate order i, f, g, o; two bias
 *                  vectors per layer); its output g is the top layer's hidden vector
 *   blank id = V; the decoder's start token is also id V; argmax ties go to the lowest id.
 *
 * Conventions
 *   - Every `const void *` / `float *` / `int32_t *` argument marked DEVICE is a pointer to GPU
 *     memory owned by the caller (for example a torch tensor's data_ptr()); HOST pointers are
 *     ordinary process memory.  The library never frees caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every function returns WIND_OK (0) or a negative wind_status; none throws or aborts.
 *     wind_last_error() gives a thread-local, library-owned description of the last failure.
 *   - wind_greedy_decode / wind_sequential_decode return after the decode has finished on
 *     `stream` (they poll a completion word); outputs are then complete in device memory.
 *   - Calls on one wind_model must not overlap: the model owns the decode workspace.
 */
#ifndef WIND_H_
#define WIND_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  WIND_OK = 0,
  WIND_ERR_ARG = -1,        /* null pointer, size out of range, inconsistent shapes */
  WIND_ERR_HIP = -2,        /* a HIP runtime call failed; see wind_last_error()      */
  WIND_ERR_OVERFLOW = -3,   /* an utterance produced more than `cap` labels          */
  WIND_ERR_UNSUPPORTED = -4,/* a shape the kernels do not cover                      */
  WIND_ERR_UNFINISHED = -5  /* an asynchronous decode ran out of its iteration budget */
} wind_status;

typedef enum { WIND_F32 = 0, WIND_BF16 = 1 } wind_dtype;

#define WIND_MAX_LAYERS 4
#define WIND_MAX_WINDOW 64

typedef struct wind_model wind_model; /* opaque, library-owned */

/*
 * Weights as the caller holds them: HOST pointers to fp32 arrays, row-major.  With
 * dtype == WIND_BF16 the library stores every matrix (emb, w_ih, w_hh, w_enc, w_pred, w_out) as
 * bf16, rounding to nearest-even, and computes with fp32 accumulation; biases stay fp32.  With
 * WIND_F32 everything stays fp32.
 */
typedef struct {
  int32_t D, E, Hp, L, Hj, V;
  int32_t dtype;                               /* wind_dtype */
  const float *emb;                            /* [V+1, E]                         */
  const float *w_ih[WIND_MAX_LAYERS];          /* layer l: [4Hp, in_l], in_0 = E, in_l = Hp */
  const float *w_hh[WIND_MAX_LAYERS];          /* [4Hp, Hp]                        */
  const float *b_ih[WIND_MAX_LAYERS];          /* [4Hp]                            */
  const float *b_hh[WIND_MAX_LAYERS];          /* [4Hp]                            */
  const float *w_enc, *b_enc;                  /* [Hj, D], [Hj]                    */
  const float *w_pred, *b_pred;                /* [Hj, Hp], [Hj]                   */
  const float *w_out, *b_out;                  /* [V+1, Hj], [V+1]                 */
} wind_weights;

/* Counters of the last decode call on a model (Analysis, "Jump Distribution"). */
typedef struct {
  int64_t iterations;       /* loop iterations that had at least one active utterance        */
  int64_t windows;          /* (utterance, iteration) pairs = joiner calls on a window       */
  int64_t rows;             /* window rows evaluated = sum of n over windows                 */
  int64_t useful_rows;      /* rows at or before the first non-blank of their window         */
  int64_t labels;           /* labels emitted                                                */
  int64_t forced_advances;  /* pointer advances taken because S labels sat on one frame      */
  int64_t rechecks;         /* rows whose argmax was re-decided in fp32 after the bf16 pass  */
  int64_t jump_hist[WIND_MAX_WINDOW + 1]; /* pointer advance per window, 0..W                 */
} wind_stats;

/*
 * Copies the weights to the GPU in the layouts the kernels want and returns a model handle.
 * Every copy and kernel of the call goes to `stream`, and the call returns after they have
 * completed: the caller may free its arrays afterwards.  Limits: 1 <= L <= 4; D, E, Hp, Hj >= 1; V >= 1.
 * With WIND_BF16, D, E, Hp and Hj must be multiples of 64 and Hj <= 2048 (WIND_ERR_UNSUPPORTED otherwise).
 */
int wind_load_weights(const wind_weights *w, void *stream, wind_model **out);
int wind_free(wind_model *m);

/*
 * Method, Algorithm 2, batched with one frame pointer per utterance.
 *   enc_out   DEVICE [B, T, D] fp32 row-major; frames at or beyond lengths[b] are never used for a
 *             decision and may hold anything.  With WIND_BF16 each value is rounded to bf16 on load.
 *   lengths   DEVICE [B] int32, 0 <= lengths[b] <= T
 *   W         window size, 1..WIND_MAX_WINDOW
 *   max_symbols_per_step  S >= 1: after S labels on one frame the pointer moves to the next frame
 *             without another joiner call (Algorithm 1 has no such bound; this is the usual guard)
 *   out_tokens, out_frames  DEVICE [B, cap] int32: label k of utterance b and the 0-based frame it
 *             was emitted on; entries beyond out_counts[b] are left untouched
 *   out_counts DEVICE [B] int32
 *   cap       capacity per utterance; T * S always suffices.  If an utterance needs more, its
 *             extra labels are dropped, out_counts[b] is clamped to cap, and the call returns
 *             WIND_ERR_OVERFLOW after finishing the decode.
 * Returns WIND_ERR_ARG for null pointers, B < 1, T < 0, W or S out of range, cap < 1.
 */
int wind_greedy_decode(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T,
                       int W, int max_symbols_per_step, int32_t *out_tokens, int32_t *out_frames,
                       int32_t *out_counts, int cap, void *stream);

/*
 * wind_greedy_decode without the wait and without the library's own memory: everything the decode
 * needs lives in `workspace` (DEVICE, 256-byte aligned, at least wind_workspace_bytes(m, B, T, W) bytes;
 * contents on entry do not matter, the caller keeps it alive until the call has completed), the kernels
 * are enqueued on `stream`, and the call returns.  The loop's length depends on the data, and nothing
 * polls here: the call enqueues max_iterations loop iterations (rounded up to whole graph replays of
 * "unroll" iterations; T * (S + 1) + 2 always suffices and is the cap), and the iterations past the end
 * of the decode cost a few empty launches each.  wind_get_stats of a previous call of the same shape
 * (its `iterations`) tells how many a workload needs.
 * Completion: the next wind_get_stats on the model waits for `stream`, and returns WIND_OK, or
 * WIND_ERR_OVERFLOW (as wind_greedy_decode), or WIND_ERR_UNFINISHED if utterances were still active
 * after max_iterations (outputs and counts then hold the labels found up to there).  Until then the
 * model accepts no other decode call.  Other arguments as wind_greedy_decode.  Returns WIND_ERR_ARG for
 * a null, misaligned or too small workspace (the message names both sizes) and max_iterations < 1,
 * WIND_ERR_UNSUPPORTED with options "graph" = 0, "profile" or "host_sync".  The first call of a shape
 * captures and instantiates its graph (host-side work and runtime allocations).
 */
int wind_greedy_decode_async(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, int W,
                             int max_symbols_per_step, int32_t *out_tokens, int32_t *out_frames,
                             int32_t *out_counts, int cap, void *workspace, size_t workspace_bytes,
                             int64_t max_iterations, void *stream);

/*
 * Method, Algorithm 1 (the standard frame-by-frame loop; Table 1's window-size-1 row), batched
 * the same way: one joiner row per utterance and iteration.  Same arguments without W.
 */
int wind_sequential_decode(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T,
                           int max_symbols_per_step, int32_t *out_tokens, int32_t *out_frames,
                           int32_t *out_counts, int cap, void *stream);

/*
 * Method, "A Novel Beam-search Algorithm for WIND": the scoring step of Algorithm 3 (joiner on the
 * window, P' of Eq. 1, the K best pairs) for Bh hypotheses that sit on the same frame.  For every hypothesis b the joiner is
 * evaluated on the n frames of the window against that hypothesis' prediction-network output, the
 * rows are soft-maxed, and P'(v, t) of Eq. 1 is formed: the probability that v is the first output
 * in the window and comes at frame t (blank: only as "no output in the whole window", t = n - 1).
 * Returns the K best (label, jump) pairs of every hypothesis, best first; equal scores are
 * ordered by earlier frame, then lower label.
 *   enc_window  DEVICE [n, D] fp32: encoder frames t0 .. t0+n-1 (1 <= n <= 64)
 *   dec_out     DEVICE [Bh, Hp] fp32: the top LSTM layer's hidden vector of every hypothesis
 *   K           1..32
 *   out_labels  DEVICE [Bh, K] int32: label (blank = V); -1 if fewer than K entries have P' > 0
 *   out_jumps   DEVICE [Bh, K] int32: frame offset inside the window (blank: n - 1)
 *   out_scores  DEVICE [Bh, K] fp32: log P' of the pair
 * Hypothesis bookkeeping (Algorithm 3's map from frames to hypotheses, recombination, pruning)
 * stays with the caller.  Allocates its workspace on first use; returns after completion.
 * Returns WIND_ERR_ARG for null pointers or sizes out of range (Bh * n <= 65536).
 */
int wind_beam_window_scores(wind_model *m, const float *enc_window, int n, const float *dec_out, int Bh, int K,
                            int32_t *out_labels, int32_t *out_jumps, float *out_scores, void *stream);

/*
 * The same scoring step for callers that cannot allocate device memory or wait on the stream:
 * code under HIP graph capture, serving loops with a fixed memory budget, harnesses that forbid
 * hipMalloc.  It calls no allocating routine and does not synchronise: the kernels are enqueued on
 * `stream` and the call returns; the outputs are complete once the stream has passed them.  Its
 * scratch memory (projected frames, hidden rows, logits, per-row candidates) is a static device
 * array of WIND_STATIC_SCRATCH_BYTES inside the library, one per GPU, held until the process ends.
 * Shapes whose scratch layout does not fit are rejected with WIND_ERR_ARG and a message that names
 * both sizes (the layout grows with Bh * n * (V + 1) * 4 bytes of logits; 16 hypotheses x 16 frames
 * of a 1024-label model need 1.9 MB).  Every call on a GPU uses that GPU's one array, whatever the
 * model or stream: calls that overlap in time on one GPU race; serialise them.
 * Arguments, outputs and tie order as wind_beam_window_scores.
 */
#define WIND_STATIC_SCRATCH_BYTES (8u << 20)
int wind_beam_window_scores_static(wind_model *m, const float *enc_window, int n, const float *dec_out, int Bh, int K,
                                   int32_t *out_labels, int32_t *out_jumps, float *out_scores, void *stream);

/*
 * Method, "A Novel Beam-search Algorithm for WIND", Algorithm 3, whole: beam search over one
 * utterance.  A map from frames to the hypotheses that rest there is kept on the host; the
 * hypotheses of the smallest frame t are taken out, recombined, passed through the prefix step and
 * pruned to K (the three steps listed under the algorithm), scored on the window of
 * n = min(window, T - t) frames with P' of Eq. 1, and each of their K best (label, jump) pairs goes
 * back into the map at the frame it leads to (label: t + jump, blank: t + n).  Every model
 * evaluation runs on the GPU: the encoder projection of all frames once, one prediction-network
 * step per new label sequence that survives pruning (states are kept for every sequence the
 * search has touched), the joiner rows of each window, their soft-max, P' and the K best pairs,
 * and the rows the prefix step needs.
 *   enc_out     DEVICE [T, D] fp32 encoder outputs of the utterance
 *   window      N of the algorithm, 1..64;  K  beam, 1..32
 *   S           safeguard against staying on one frame for ever (the algorithm's footnote): after
 *               the S-th consecutive label on a frame a hypothesis moves one frame on, at no cost,
 *               as in the greedy decoders of this library; S >= 1
 *   prefix_mode what the prefix step does with a hypothesis A that is a proper prefix of another
 *               hypothesis B on the same frame.  In every mode but OFF, B gains A's probability
 *               times the probability of emitting the missing labels on frame t (only completions
 *               that the safeguard allows).  KEEP leaves A in the set (the definition in the work
 *               the section credits for this step); REMOVE takes A out (the section's own sentence)
 *   out_tokens, out_frames  HOST [cap] int32: labels of the most probable hypothesis at frame T and
 *               the frame of each; out_count HOST: their number; out_score HOST: its log-probability
 *   stats       HOST, may be NULL;  on_round  may be NULL: called after the scoring step of every
 *               pass with the surviving hypotheses and their chosen pairs (HOST arrays that are
 *               valid during the call only): hyp_tokens / hyp_frames are the hypotheses' labels and
 *               label frames back to back (hyp_len[b] each), labels / jumps / scores are [n_hyps, K]
 * Scores are natural-log probabilities, accumulated in fp64 on the host from fp32 log P' values.
 * Equal scores: duplicates keep the lexicographically smaller time stamps; pruning and the final
 * choice prefer the shorter, then the lexicographically smaller label sequence.
 * Returns WIND_ERR_OVERFLOW (after setting out_count and out_score) if the result has more than
 * cap labels.  Returns after completion; allocates on first use and when the search outgrows its
 * state pool.
 */
typedef enum { WIND_PREFIX_OFF = 0, WIND_PREFIX_KEEP = 1, WIND_PREFIX_REMOVE = 2 } wind_prefix_mode;
typedef struct {
  int64_t rounds;          /* passes of the while-loop                                        */
  int64_t hyps_scored;     /* hypotheses sent through the scoring step, over all passes       */
  int64_t decoder_steps;   /* prediction-network steps (one per label sequence given a state) */
  int64_t completions;     /* (A, B) pairs handled by the prefix step                         */
  int64_t completion_rows; /* joiner rows evaluated for them                                  */
  int64_t max_pending;     /* most hypotheses taken out of the map in one pass                */
  int64_t nodes;           /* distinct label sequences created                                */
} wind_beam_stats;
typedef void (*wind_beam_round_fn)(void *user, int t, int n, int n_hyps, const int32_t *hyp_len, const int32_t *hyp_tokens,
                                   const int32_t *hyp_frames, const double *hyp_score, const int32_t *hyp_sym, int K,
                                   const int32_t *labels, const int32_t *jumps, const float *scores);
int wind_beam_decode(wind_model *m, const float *enc_out, int T, int window, int K, int S, int prefix_mode,
                     int32_t *out_tokens, int32_t *out_frames, int cap, int32_t *out_count, double *out_score,
                     wind_beam_stats *stats, wind_beam_round_fn on_round, void *user, void *stream);

/*
 * Device memory, in bytes, of the workspace that a decode call of this shape needs (encoder
 * projections of every frame, window rows, keys, prediction-network state, ...).  The model owns
 * one workspace, allocated on the first call and regrown when a later call needs more; this query
 * lets a caller budget HBM before the call.  HOST pointer.  No GPU work.
 */
int wind_workspace_bytes(const wind_model *m, int B, int T, int W, size_t *bytes);

/* Counters of the last decode call; HOST pointer.  After wind_greedy_decode_async this call completes that
 * decode first (it waits for its stream) and returns its status. */
int wind_get_stats(wind_model *m, wind_stats *out);

/*
 * Debug: joiner logits of one window.  Steps the prediction network from nothing over
 * prefix[0..prefix_len) (HOST int32 labels), then evaluates the joiner on frames t0..t0+n-1 of
 * utterance b of enc_out (DEVICE [B, T, D]).  Writes DEVICE float [n, V+1] (Algorithm 2's
 * `joined`; n = 16, V+1 = 1025 gives the 16400 floats of Analysis, "Memory Footprint").
 *   exact = 0: the values the MFMA pass sees (bf16 hidden vector, fp32 accumulation; for
 *              WIND_F32 models the same as exact = 1)
 *   exact = 1: fp32 hidden vector, fp32 FMA (what near-tie decisions are re-decided with)
 */
int wind_debug_joint_logits(wind_model *m, const float *enc_out, int B, int T, int b, int t0, int n,
                            const int32_t *prefix, int prefix_len, int exact, float *logits,
                            void *stream);

/*
 * Debug: the encoder half of the joiner as a decode call computes it once per call,
 * e[b, t, :] = W_enc enc_out[b, t, :] + b_enc (the joiner of Algorithms 1 and 2 is linear in the
 * encoder frame up to its activation, so this half is hoisted out of the loop).  Writes DEVICE float
 * e_out [B, T, Hj]; rows with t >= lengths[b] are unspecified.  enc_out DEVICE [B, T, D], lengths
 * DEVICE [B].  Returns after completion.
 */
int wind_debug_enc_proj(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, float *e_out,
                        void *stream);

/*
 * Debug: what the joint kernel of a decode call leaves behind for the first loop iteration
 * (Algorithm 2: the joiner on the first window against the start state, and each row's argmax), bf16 models.
 * The window rows are r = a * W + j for the a-th utterance with lengths > 0 and its frames
 * j = 0 .. W-1 (frames at or past the utterance's end: rows of a zero hidden vector).  The label
 * columns are cut into *nparts parts of *part_width columns; for every row and part the kernel keeps
 * the three largest logits of the part, each as one fp32 word whose low 7 mantissa bits hold
 * 127 - (column within the part): value = word with those bits cleared.  keys DEVICE float
 * [B * W, *nparts, 4] (largest, second, third, unused), or NULL to query the two sizes only (HOST
 * pointers).  A part with fewer than three label columns has -3.0e38 in the unused places.  Returns
 * after completion.
 */
int wind_debug_joint_keys(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, int W,
                          float *keys, int32_t *nparts, int32_t *part_width, void *stream);

/*
 * Per-kernel device time, for the roofline report.  With option "profile" = 1 the decode loop is
 * launched kernel by kernel (no graph) and every launch carries an event pair that receives the
 * dispatch's begin and end time stamps (the kernel's own duration, without launch gaps); this call returns
 * the accumulated milliseconds and launch counts since the option was last set, indexed by
 * wind_kernel_id.  HOST pointers to WIND_NUM_KERNELS entries each.
 */
typedef enum {
  WIND_K_ENC_PROJ = 0,  /* encoder projection, once per call           */
  WIND_K_BUILD_Z = 1,   /* window gather + activation                  */
  WIND_K_JOINT = 2,     /* output contraction + row argmax             */
  WIND_K_DECIDE = 3,    /* first non-blank, pointer update, compaction */
  WIND_K_LSTM = 4,      /* all LSTM layers of one step                 */
  WIND_K_PRED_PROJ = 5, /* prediction projection                       */
  WIND_NUM_KERNELS = 6
} wind_kernel_id;
int wind_get_kernel_times(wind_model *m, double *ms, int64_t *launches);

/*
 * Device time of the last decode call on a model, from events on the call's stream: the whole call,
 * and the loop alone, i.e. without the once-per-call set-up (state, encoder projection of every frame,
 * start-token step) — the "decoder-only" kind of time of Table 5, whose total also holds the encoder.
 * In milliseconds; HOST pointers.  The loop's end is the last launch the call made (with graph replay
 * that includes the launches that found every utterance finished).  WIND_ERR_ARG before the first call.
 */
int wind_get_call_times(wind_model *m, double *total_ms, double *loop_ms);

/*
 * The joint kernel launch by launch, for the roofline report: after a decode call made with option
 * "profile" = 1 (bf16 models), rows[i] is the number of window rows that loop iteration i
 * evaluated (the sum of n = min(W, len - t) over its active utterances; Algorithm 2) and us[i] the
 * duration of that iteration's joint launch in microseconds.  HOST arrays of `cap` entries; *n
 * receives the number of iterations recorded (at most 16384), of which the first min(*n, cap) are
 * written.  WIND_ERR_ARG for null pointers.
 */
int wind_get_joint_launches(wind_model *m, int32_t *rows, float *us, int cap, int *n);

/*
 * How the last decode call ran its loop (the loop of Algorithm 2, for one or two utterances, can run
 * as one resident kernel; option "loop_kernel"): *workgroups receives the number of workgroups of
 * that kernel, 0 if the call replayed the graph of per-step kernels instead; *one_l2 receives 1 if
 * those workgroups all sat on one XCD and exchanged their values through its L2 (option
 * "loop_one_xcd"), else 0.  Completes a pending asynchronous decode first.  HOST pointers;
 * WIND_ERR_ARG for null pointers.
 */
int wind_get_loop_info(wind_model *m, int *workgroups, int *one_l2);

/*
 * Tuning knobs, for benchmarks and tests.  key/value pairs:
 *   "graph"   1 (default): the decode loop is replayed from a captured HIP graph; 0: kernels are
 *             launched one by one (the with / without graph rows of Table 5)
 *   "host_sync"  1: the loop as a framework runs it without graphs (the rows without graph of Table 5):
 *             every iteration's kernels are launched one by one and the host waits for them and reads the
 *             number of active utterances before launching the next iteration (default 0; overrides "graph")
 *   "unroll"  loop iterations per graph launch (default 16, even)
 *   "profile" 1: time every kernel launch with events (see wind_get_kernel_times); implies no graph
 *   "recheck_kappa_milli"  kappa * 1000 (default 8000).  bf16 models screen every window row with a
 *             bf16 hidden vector and re-decide in fp32 every label within
 *             tau = kappa * 2.1e-3 * max_v |w_out[v]| * |z| / sqrt(Hj) of the row's largest logit (blank
 *             included): kappa standard deviations of the difference of two screened logits, under the
 *             assumption that the hidden units' rounding errors are independent and the weight rows are
 *             not aligned with z (random or trained dense rows).  For rows aligned with z the error can
 *             reach 2^-8 |w| |z| (kappa ~ 7.4 sqrt(Hj)); raise kappa for such models: the band only
 *             costs fp32 re-evaluations, never correctness
 *   "pred_mfma_min_batch"  smallest B for which the prediction network runs on MFMA tiles
 *             (default 1; bf16 models only; below it one wave per hidden unit does fp32 FMA)
 *   "loop_kernel"  1 (default): decodes of one or two utterances with at most 32 window rows (bf16, one
 *             LSTM layer, weights that fit the chip's LDS) run the whole loop as one resident kernel
 *             whose workgroups meet at grid barriers; 0: always the graph of per-step kernels
 *   "loop_fused"  1 (default): with at most 16 window rows and a joint hidden size that is a multiple of 128,
 *             at most 640, that kernel builds the window rows directly as matrix-core operands; 0: it
 *             stages them in LDS (the form for every other shape)
 *   "loop_one_xcd"  1 (default): where 32 workgroups suffice for that kernel (and the window rows number
 *             at most 16), they are placed on the CUs of one XCD and exchange through its L2, which
 *             shortens every grid barrier; the kernel checks the placement itself and falls back to
 *             device-wide stores if it is not as expected.  0: spread over the chip
 *   "loop_spin_limit"  polls a workgroup of that kernel waits at a barrier before it gives up
 *             (default 2^21, about a second); the decode then returns WIND_ERR_HIP.  Tests set it
 *             to 0 to exercise that path: every workgroup still leaves the kernel normally
 *   "atomic_lists"  1 (default): in the graph of per-step kernels of bf16 models, every workgroup of the
 *             decision kernel claims its utterance's place in the next iteration's list of active
 *             utterances and in the list of utterances that emitted with an atomic counter (the
 *             order of those lists then varies between runs, the decoded output does not); 0: the
 *             last workgroup to finish compacts the lists in order
 *   "joint_wide"  which iterations of the graph of per-step kernels evaluate the joiner's output layer on
 *             256-column tiles (bf16 models with Hj >= 320) instead of 128-column tiles: 1 (default) those
 *             with so many window rows that the tiles are at least 192 rows high when they fill the
 *             chip (above 1024 rows for 8192 labels, above 2048 for 4096), chosen per graph replay from
 *             the active count the host last read back or from the previous call of the same shape; 0
 *             none; 2 all.  The decoded output does not depend on it: both kernels form every logit by
 *             the same operations in the same order
 *   "lstm_rec"  1 (default): where the prediction network runs on MFMA tiles, the recurrent half of every
 *             LSTM layer's gate sums (w_hh . h) is kept ready for the hidden vectors as they stand and
 *             renewed beside the projection, so a step only adds the input half once the label is
 *             known (the first layer inside the decision kernel); 0: whole steps after the decision
 *   "slot_rows"  1 (default): with "lstm_rec" and "atomic_lists", in models of more than one LSTM layer, the
 *             layers above the first take their rows by slot of the iteration's list of active utterances
 *             (rows of utterances that do not step are computed and dropped), so that their kernels can ask
 *             for their operands before they have read anything about the iteration; 0: through the list of
 *             utterances that emitted.  The decoded output does not depend on it
 *   "decide_two"  1 (default): for rows of 65 .. 128 column parts (4097 .. 8192 labels) and windows of at most
 *             16 rows, a wave of the decision kernel asks for both halves of its row's keys at once; 0: for the
 *             second half once the first has been looked at (the form for every other shape)
 *   "enc_wide"  1 (default): large calls of bf16 models with D >= 320 run the encoder projection on the
 *             256-column tile core; 0: on 256 x 256 tiles of eight waves.  Same bits either way
 *   "beam_exact"  1: the beam-search entry points evaluate bf16 models' joiner rows with an fp32
 *             hidden vector and fp32 FMA instead of the bf16 MFMA pass, so that their choices do
 *             not depend on the rounding of the hidden vector (default 0)
 *   "debug_stamps"  1: the resident loop kernel and the decision kernel record
 *             phase time stamps, which the next decode prints to stderr (development aid; default 0)
 */
int wind_set_option(wind_model *m, const char *key, int64_t value);

const char *wind_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* WIND_H_ */
