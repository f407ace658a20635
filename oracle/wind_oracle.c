/*
 * CPU oracle for RNN-T greedy decoding.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product path never does and shares no code with it.
 *
 * What it computes
 *   oracle_greedy      the standard frame-by-frame RNN-T inference loop (Method, Algorithm 1, with
 *                      the two rules listed in "Background: RNN-T": a non-blank label is appended
 *                      and fed to the decoder while the frame pointer stays; a blank leaves the
 *                      decoder alone and moves to the next frame).  This is the definition every
 *                      other decoder is held to: the windowed method reaches exactly this output
 *                      (Method, remark after Algorithm 2; Table 1's identical WER column).
 *   oracle_wind        the windowed loop (Method, Algorithm 2), written a second time from the
 *                      algorithm's own steps.  It exists to pin oracle_greedy, not to be compared
 *                      with the GPU.
 *   oracle_joiner, oracle_decoder_step, oracle_decoder_from_scratch, oracle_encoder_projection
 *                      the model pieces, exported so tests can pin them to library routines and
 *                      enumerate tiny lattices by brute force.
 *
 * Readings where the paper is silent (the paper only says the joiner "combines" the two streams
 * and calls the prediction network "decoder"):
 *   joiner(f, g) = W_out * relu(W_enc f + b_enc + W_pred g + b_pred) + b_out, logits over V+1 ids;
 *   blank id = V; decoder([]) = one LSTM step from zero state on the embedding of id V;
 *   decoder = embedding + L stacked LSTM cells, gate order i,f,g,o, two bias vectors,
 *     c' = sigm(f) c + sigm(i) tanh(g), h' = sigm(o) tanh(c'); its output is the top layer's h;
 *   argmax ties go to the lowest id;
 *   at most S labels per frame: after the S-th consecutive label on one frame the pointer moves on
 *     without another joiner call (Algorithm 1 has no such bound; S >= 1).
 *
 * Arithmetic: inputs are float (bf16-representable where the configuration says bf16); every sum,
 * product and transcendental is fp64, accumulated in index order, with no intermediate rounding.
 *
 * Pins (tests/test_oracle_pins.py): Algorithm 2 == Algorithm 1 for every window size, window 1
 * makes the same joiner calls, brute-force lattice walk with from-scratch decoder states on tiny
 * vocabularies, torch.nn.LSTM / linear in fp64, closed forms for always-blank / never-blank /
 * decoder-blind models, output invariants, and the window-count closed form.  The absolute token
 * values on the five workloads are not printed anywhere in the paper: "parity unpinned" for those,
 * beyond the cross-checks above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t D, E, Hp, L, Hj, V;
  const float *emb;                 /* [V+1, E] */
  const float *w_ih[4], *w_hh[4];   /* layer l: [4Hp, in_l], [4Hp, Hp]; in_0 = E, in_l = Hp */
  const float *b_ih[4], *b_hh[4];   /* [4Hp] */
  const float *w_enc, *b_enc;       /* [Hj, D], [Hj] */
  const float *w_pred, *b_pred;     /* [Hj, Hp], [Hj] */
  const float *w_out, *b_out;       /* [V+1, Hj], [V+1] */
} oracle_model;

/* one joiner evaluation of the sequential decoder, kept for the comparison protocol */
typedef struct {
  int32_t t;        /* frame */
  int32_t u;        /* labels emitted before this evaluation */
  int32_t label;    /* decision taken (the forced one if a forced choice applied) */
  int32_t top1;     /* argmax id */
  int32_t top2;     /* runner-up id */
  double v1, v2;    /* their logits */
  double vlabel;    /* logit of the decision taken */
} oracle_eval;

static double sigm(double x) { return 1.0 / (1.0 + exp(-x)); }

/* One step of the prediction network on `token`; h, c are [L*Hp], updated in place. */
void oracle_decoder_step(const oracle_model *m, int token, double *h, double *c) {
  const int Hp = m->Hp;
  double *x = (double *)malloc(sizeof(double) * (size_t)(m->E > Hp ? m->E : Hp));
  double *gates = (double *)malloc(sizeof(double) * 4 * (size_t)Hp);
  int in = m->E;
  for (int k = 0; k < in; ++k) x[k] = (double)m->emb[(size_t)token * m->E + k];
  for (int l = 0; l < m->L; ++l) {
    double *hl = h + (size_t)l * Hp, *cl = c + (size_t)l * Hp;
    for (int r = 0; r < 4 * Hp; ++r) {
      double a = (double)m->b_ih[l][r];
      for (int k = 0; k < in; ++k) a += (double)m->w_ih[l][(size_t)r * in + k] * x[k];
      double b = (double)m->b_hh[l][r];
      for (int k = 0; k < Hp; ++k) b += (double)m->w_hh[l][(size_t)r * Hp + k] * hl[k];
      gates[r] = a + b;
    }
    for (int j = 0; j < Hp; ++j) {
      double ig = sigm(gates[j]), fg = sigm(gates[Hp + j]);
      double gg = tanh(gates[2 * Hp + j]), og = sigm(gates[3 * Hp + j]);
      cl[j] = fg * cl[j] + ig * gg;
      hl[j] = og * tanh(cl[j]);
    }
    in = Hp;
    for (int k = 0; k < Hp; ++k) x[k] = hl[k];
  }
  free(x);
  free(gates);
}

/* The decoder output for a label sequence hyp, computed from nothing: zero state, the start id V, then every label of hyp.
   g receives the top layer's h ([Hp]). */
void oracle_decoder_from_scratch(const oracle_model *m, const int32_t *hyp, int n, double *g) {
  size_t sz = (size_t)m->L * m->Hp;
  double *h = (double *)calloc(sz, sizeof(double)), *c = (double *)calloc(sz, sizeof(double));
  oracle_decoder_step(m, m->V, h, c);
  for (int i = 0; i < n; ++i) oracle_decoder_step(m, hyp[i], h, c);
  memcpy(g, h + (size_t)(m->L - 1) * m->Hp, sizeof(double) * m->Hp);
  free(h);
  free(c);
}

/* The encoder half of the joiner's hidden vector, W_enc f + b_enc ([Hj]), written out as the same sums
   oracle_joiner forms (the joiner's first term; the reading of "combines" stated in the header).
   Exported so that a decoder which forms this half once per frame can be checked on it. */
void oracle_encoder_projection(const oracle_model *m, const float *f, double *out) {
  for (int j = 0; j < m->Hj; ++j) {
    double a = (double)m->b_enc[j];
    for (int d = 0; d < m->D; ++d) a += (double)m->w_enc[(size_t)j * m->D + d] * (double)f[d];
    out[j] = a;
  }
}

/* The joiner on one encoder frame f and one decoder output g -> logits[V+1] */
void oracle_joiner(const oracle_model *m, const float *f, const double *g, double *logits) {
  double *z = (double *)malloc(sizeof(double) * (size_t)m->Hj);
  for (int j = 0; j < m->Hj; ++j) {
    double a = (double)m->b_enc[j];
    for (int d = 0; d < m->D; ++d) a += (double)m->w_enc[(size_t)j * m->D + d] * (double)f[d];
    double b = (double)m->b_pred[j];
    for (int k = 0; k < m->Hp; ++k) b += (double)m->w_pred[(size_t)j * m->Hp + k] * g[k];
    double s = a + b;
    z[j] = s > 0.0 ? s : 0.0;
  }
  for (int v = 0; v <= m->V; ++v) {
    double a = (double)m->b_out[v];
    for (int j = 0; j < m->Hj; ++j) a += (double)m->w_out[(size_t)v * m->Hj + j] * z[j];
    logits[v] = a;
  }
  free(z);
}

/* argmax with ties to the lowest id; also the runner-up */
static void top2(const double *x, int n, int *i1, int *i2) {
  int a = 0, b = -1;
  for (int v = 1; v < n; ++v) {
    if (x[v] > x[a]) { b = a; a = v; }
    else if (b < 0 || x[v] > x[b]) b = v;
  }
  *i1 = a;
  *i2 = b;
}

/*
 * Algorithm 1 on one utterance.  forced[k] = {t, u, label}: at the evaluation of frame t with u
 * labels already emitted take `label` instead of the argmax (used by the comparison protocol to
 * follow a legitimate near-tie divergence).  Returns 0, or -1 if an output or log capacity is hit.
 */
int oracle_greedy(const oracle_model *m, const float *enc, int len, int S,
                  const int32_t *forced, int n_forced,
                  int32_t *tokens, int32_t *frames, int cap, int32_t *count,
                  oracle_eval *log, int log_cap, int32_t *n_log) {
  const int blank = m->V;
  size_t sz = (size_t)m->L * m->Hp;
  double *h = (double *)calloc(sz, sizeof(double)), *c = (double *)calloc(sz, sizeof(double));
  double *logits = (double *)malloc(sizeof(double) * (size_t)(m->V + 1));
  int t = 0, u = 0, sym = 0, nl = 0, rc = 0;
  oracle_decoder_step(m, blank, h, c);                       /* decoder output before any label */
  while (t < len) {
    const double *g = h + (size_t)(m->L - 1) * m->Hp;        /* the top layer's hidden vector */
    oracle_joiner(m, enc + (size_t)t * m->D, g, logits);
    int i1, i2;
    top2(logits, m->V + 1, &i1, &i2);
    int label = i1;
    for (int k = 0; k < n_forced; ++k)
      if (forced[3 * k] == t && forced[3 * k + 1] == u) label = forced[3 * k + 2];
    if (log) {
      if (nl >= log_cap) { rc = -1; break; }
      oracle_eval *e = &log[nl++];
      e->t = t; e->u = u; e->label = label; e->top1 = i1; e->top2 = i2;
      e->v1 = logits[i1]; e->v2 = i2 >= 0 ? logits[i2] : -INFINITY; e->vlabel = logits[label];
    }
    if (label != blank) {
      if (u >= cap) { rc = -1; break; }
      tokens[u] = label; frames[u] = t; ++u;                 /* the label joins the hypothesis ... */
      oracle_decoder_step(m, label, h, c);                   /* ... and is fed to the decoder; the frame stays */
      if (++sym == S) { t += 1; sym = 0; }
    } else {
      t += 1; sym = 0;
    }
  }
  *count = u;
  if (n_log) *n_log = nl;
  free(h); free(c); free(logits);
  return rc;
}

/*
 * Algorithm 2 on one utterance, window size W.  calls[k] = {t, n} for every joiner call on a
 * window; jump_hist[0..W] counts the pointer advance of every window step.  S is applied as in
 * oracle_greedy: the per-frame label counter carries over when the label is found at the head of
 * the window, restarts at 1 when it is found further in, and clears on an all-blank window.
 */
int oracle_wind(const oracle_model *m, const float *enc, int len, int W, int S,
                int32_t *tokens, int32_t *frames, int cap, int32_t *count,
                int32_t *calls, int calls_cap, int32_t *n_calls, int64_t *jump_hist) {
  const int blank = m->V, V1 = m->V + 1;
  size_t sz = (size_t)m->L * m->Hp;
  double *h = (double *)calloc(sz, sizeof(double)), *c = (double *)calloc(sz, sizeof(double));
  double *joined = (double *)malloc(sizeof(double) * (size_t)V1 * (size_t)W);
  int *labels = (int *)malloc(sizeof(int) * (size_t)W);
  int t = 0, u = 0, sym = 0, nc = 0, rc = 0;
  oracle_decoder_step(m, blank, h, c);
  while (t < len) {
    const double *g = h + (size_t)(m->L - 1) * m->Hp;
    int n = W < len - t ? W : len - t;
    for (int j = 0; j < n; ++j) {                            /* the joiner on the window's n frames, one decoder output */
      oracle_joiner(m, enc + (size_t)(t + j) * m->D, g, joined + (size_t)j * V1);
      int i2;
      top2(joined + (size_t)j * V1, V1, &labels[j], &i2);    /* each row's most probable id */
    }
    if (calls) {
      if (nc >= calls_cap) { rc = -1; break; }
      calls[2 * nc] = t; calls[2 * nc + 1] = n;
    }
    ++nc;
    int i = -1;
    for (int j = 0; j < n; ++j) if (labels[j] != blank) { i = j; break; }
    if (i < 0) {
      t += n; sym = 0;
      if (jump_hist) jump_hist[n]++;
    } else {
      if (u >= cap) { rc = -1; break; }
      tokens[u] = labels[i]; frames[u] = t + i; ++u;
      oracle_decoder_step(m, labels[i], h, c);
      t += i;
      sym = (i == 0) ? sym + 1 : 1;
      int jump = i;
      if (sym == S) { t += 1; sym = 0; jump += 1; }
      if (jump_hist) jump_hist[jump > W ? W : jump]++;
    }
  }
  *count = u;
  if (n_calls) *n_calls = nc;
  free(h); free(c); free(joined); free(labels);
  return rc;
}

/*
 * Algorithm 1 on each utterance of a batch, utterances in parallel (the only parallelism).
 * enc [B,T,D]; forced[k] = {b, t, u, label}; tokens/frames [B,cap]; log [B,log_cap] or NULL.
 * Returns the number of utterances that hit a capacity.
 */
int oracle_greedy_batch(const oracle_model *m, const float *enc, const int32_t *lengths, int B, int T,
                        int S, const int32_t *forced, int n_forced,
                        int32_t *tokens, int32_t *frames, int cap, int32_t *counts,
                        oracle_eval *log, int log_cap, int32_t *n_log, int threads) {
  int bad = 0;
#ifdef _OPENMP
  if (threads > 0) omp_set_num_threads(threads);
#endif
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad)
  for (int b = 0; b < B; ++b) {
    int nf = 0;
    for (int k = 0; k < n_forced; ++k) nf += forced[4 * k] == b;
    int32_t *fb = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)(nf ? nf : 1));
    for (int k = 0, q = 0; k < n_forced; ++k)
      if (forced[4 * k] == b) {
        fb[3 * q] = forced[4 * k + 1]; fb[3 * q + 1] = forced[4 * k + 2]; fb[3 * q + 2] = forced[4 * k + 3];
        ++q;
      }
    int rc = oracle_greedy(m, enc + (size_t)b * T * m->D, lengths[b], S, fb, nf,
                           tokens + (size_t)b * cap, frames + (size_t)b * cap, cap, &counts[b],
                           log ? log + (size_t)b * log_cap : NULL, log_cap, n_log ? &n_log[b] : NULL);
    bad += rc != 0;
    free(fb);
  }
  return bad;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
