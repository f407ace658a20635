// Host side of WIND beam search (section "A Novel Beam-search Algorithm for WIND", Algorithm 3):
// the map from frames to hypotheses, recombination, the prefix step, pruning and the expansion
// loop run on the host; every model evaluation (encoder projection, prediction-network steps for
// new label sequences, joiner rows, soft-max, P' of Eq. 1 and the K best pairs) runs in kernels of
// wind_beam.h.  Included by wind_api.hip after wind_model and its helpers.
//
// Label sequences are nodes of a trie (parent, label), so that "same sequence" is "same node" and
// "A is a prefix of B" is "A is an ancestor of B".  A node gets a state slot (LSTM h and c of every
// layer, projected output) the first time a hypothesis with that sequence survives pruning; its
// parent always has one by then, because hypotheses are only ever expanded after that point.
#pragma once

namespace {

struct BeamWs {
  float *e, *p, *logits, *lse, *blp, *cl;
  int *cv;
  bf16_t *z, *z_lo;
};

BeamIndex beam_identity() { return BeamIndex{nullptr, 0, {0}}; }
BeamIndex beam_list(const int *device_list) { return BeamIndex{device_list, 0, {0}}; }
BeamIndex beam_inline(const int *host_values, int n) {
  BeamIndex ix{nullptr, n, {0}};
  for (int i = 0; i < n; ++i) ix.inl[i] = host_values[i];
  return ix;
}

// Lays the scoring workspace for up to n frames, Bh hypotheses and `rows` joiner rows out from `base`
// (null: sizes only) and returns its size in bytes.
size_t beam_carve(const wind_model *m, size_t n, size_t Bh, size_t rows, char *base, BeamWs *ws) {
  const ModelDev &d = m->dev;
  const size_t rows_pad = round_up(rows, JointCfg::BM), V1 = (size_t)d.V + 1;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
  const size_t o_e = take(n * d.Hj * 4), o_p = take(Bh * d.Hj * 4);
  const size_t o_z = take(rows_pad * d.Hj * 2), o_zlo = take(rows_pad * d.Hj * 2), o_lg = take(rows * V1 * 4);
  const size_t o_lse = take(rows * 4), o_blp = take(rows * 4), o_cl = take(rows * kBeamMaxK * 4), o_cv = take(rows * kBeamMaxK * 4);
  if (base && ws) {
    ws->e = (float *)(base + o_e); ws->p = (float *)(base + o_p); ws->logits = (float *)(base + o_lg);
    ws->z = (bf16_t *)(base + o_z);
    ws->z_lo = (bf16_t *)(base + o_zlo);
    ws->lse = (float *)(base + o_lse); ws->blp = (float *)(base + o_blp); ws->cl = (float *)(base + o_cl);
    ws->cv = (int *)(base + o_cv);
  }
  return off;
}

// The model's own scoring workspace, allocated on first use and regrown on demand.
int beam_workspace(wind_model *m, size_t n, size_t Bh, size_t rows, BeamWs *ws) {
  const size_t off = beam_carve(m, n, Bh, rows, nullptr, nullptr);
  if (off > m->beam_ws_bytes) {
    HIP_TRY(hipDeviceSynchronize());
    if (m->beam_ws) HIP_TRY(hipFree(m->beam_ws));
    m->beam_ws = nullptr;
    m->beam_ws_bytes = 0;
    HIP_TRY(hipMalloc(&m->beam_ws, off));
    m->beam_ws_bytes = off;
    HIP_TRY(hipMemset(m->beam_ws, 0, off));   // the MFMA pass reads whole row tiles
  }
  beam_carve(m, n, Bh, rows, (char *)m->beam_ws, ws);
  return WIND_OK;
}

// logits[(b, t), :] = joiner row of frame t of e_win ([n, Hj] projected frames) and hypothesis b (row
// pi(b) of p).  bf16 models: the MFMA pass on the hidden vector rounded to bf16, or, with option
// "beam_exact", on its split into two bf16 vectors (close to fp32 accuracy).  fp32 models: fp32 FMA.
void beam_enqueue_logits(wind_model *m, const BeamWs &ws, const float *e_win, int n, const float *p, const BeamIndex &pi,
                         int Bh, hipStream_t s) {
  const ModelDev &d = m->dev;
  const size_t rows = (size_t)Bh * n, rows_pad = round_up(rows, JointCfg::BM), V1 = (size_t)d.V + 1;
  if (m->dtype == WIND_BF16 && d.Hj <= kBeamTinyMaxHj && rows <= (size_t)kBeamTinyMaxRows) {
    const int split = m->opt_beam_exact ? 1 : 0;
    const size_t smem = std::max<size_t>((size_t)(split + 1) * 32 * (d.Hj + 8) * 2, 16384);
    dim3 grid((unsigned)((V1 + 31) / 32), (unsigned)((rows + 31) / 32));
    beam_logits_tiny_kernel<<<grid, 256, smem, s>>>(d, e_win, p, pi, n, (int)rows, split, ws.logits);
  } else if (m->dtype == WIND_BF16) {
    bf16_t *z_lo = m->opt_beam_exact ? ws.z_lo : nullptr;
    beam_hidden_kernel<<<(unsigned)rows, 256, 0, s>>>(e_win, p, pi, ws.z, z_lo, n, d.Hj);
    dim3 grid((unsigned)(rows_pad / JointCfg::BM), (unsigned)((V1 + JointCfg::BN - 1) / JointCfg::BN));
    joint_mfma_store_kernel<JointCfg><<<grid, JointCfg::NT, JointCfg::SMEM_BYTES, s>>>(d, ws.z, z_lo, (int)rows, ws.logits);
  } else {
    beam_logits_kernel<float><<<(unsigned)rows, 256, (size_t)d.Hj * 4, s>>>(d, e_win, p, pi, n, ws.logits);
  }
}

// The K best (label, jump) pairs of every hypothesis from its n rows of logits.
void beam_enqueue_topk(wind_model *m, const BeamWs &ws, int n, int Bh, int K, int32_t *out_labels, int32_t *out_jumps,
                       float *out_scores, hipStream_t s) {
  const ModelDev &d = m->dev;
  const size_t rows = (size_t)Bh * n, V1 = (size_t)d.V + 1;
  if (V1 <= 256 * 36) {
    // one workgroup per row, then one wave per hypothesis
    if (V1 <= 256 * 8) beam_row_kernel<8><<<(unsigned)rows, 256, 0, s>>>(ws.logits, d.V, K, ws.lse, ws.blp, ws.cl, ws.cv);
    else beam_row_kernel<36><<<(unsigned)rows, 256, 0, s>>>(ws.logits, d.V, K, ws.lse, ws.blp, ws.cl, ws.cv);
    beam_merge_kernel<<<(unsigned)Bh, 64, 0, s>>>(ws.lse, ws.blp, ws.cl, ws.cv, n, d.V, K, out_labels, out_jumps, out_scores);
  } else if (K <= 8) {
    beam_score_kernel<8><<<(unsigned)Bh, 256, 0, s>>>(ws.logits, n, d.V, K, out_labels, out_jumps, out_scores);
  } else if (K <= 16) {
    beam_score_kernel<16><<<(unsigned)Bh, 256, 0, s>>>(ws.logits, n, d.V, K, out_labels, out_jumps, out_scores);
  } else {
    beam_score_kernel<32><<<(unsigned)Bh, 256, 0, s>>>(ws.logits, n, d.V, K, out_labels, out_jumps, out_scores);
  }
}

// out[r, :] = w x[r] + bias for fp32 rows x, weights in the model's storage type.
void beam_enqueue_linear(wind_model *m, const void *w, const float *bias, const float *x, float *out, int rows, int n_out,
                         int K, bool round_x, hipStream_t s) {
  constexpr int kR = 8;   // rows that share one pass over a weight row
  const dim3 grid((unsigned)((n_out + 3) / 4), (unsigned)((rows + kR - 1) / kR));
  if (m->dtype == WIND_BF16 && round_x)
    beam_linear_kernel<bf16_t, true, kR><<<grid, 256, 0, s>>>((const bf16_t *)w, bias, x, out, rows, n_out, K);
  else if (m->dtype == WIND_BF16)
    beam_linear_kernel<bf16_t, false, kR><<<grid, 256, 0, s>>>((const bf16_t *)w, bias, x, out, rows, n_out, K);
  else
    beam_linear_kernel<float, false, kR><<<grid, 256, 0, s>>>((const float *)w, bias, x, out, rows, n_out, K);
}

// ---- state pool and staging ---------------------------------------------------------------------
constexpr int kBeamCompRows = 1024;   // completion rows (prefix step) evaluated per batch
constexpr int kBeamStageInts = 2 * kBeamCompRows;   // device lists of a large completion batch: slots, labels
constexpr int kBeamResScores = 0, kBeamResLabels = kBeamMaxK * kBeamMaxK, kBeamResJumps = 2 * kBeamMaxK * kBeamMaxK,
              kBeamResComp = 3 * kBeamMaxK * kBeamMaxK, kBeamResWords = 3 * kBeamMaxK * kBeamMaxK + kBeamCompRows;

int beam_pool_reserve(wind_model *m, int slots, hipStream_t s) {
  BeamPool &bp = m->beam_pool;
  const ModelDev &d = m->dev;
  if (!bp.h_stage) {
    // results land in pinned host memory that the kernels write directly: a pass ends with a stream
    // synchronisation and no copy
    HIP_TRY(hipHostMalloc((void **)&bp.h_stage, sizeof(int) * kBeamStageInts, hipHostMallocDefault));
    HIP_TRY(hipHostMalloc((void **)&bp.h_res, 4 * kBeamResWords, hipHostMallocDefault));
    HIP_TRY(hipMalloc((void **)&bp.d_stage, sizeof(int) * kBeamStageInts));
    HIP_TRY(hipHostGetDevicePointer(&bp.d_res, bp.h_res, 0));
  }
  if (slots <= bp.cap) return WIND_OK;
  int cap = bp.cap ? bp.cap : 1024;
  while (cap < slots) cap *= 2;
  const size_t st = (size_t)d.L * d.Hp;
  float *h = nullptr, *c = nullptr, *p = nullptr;
  HIP_TRY(hipMalloc((void **)&h, (size_t)cap * st * 4));
  HIP_TRY(hipMalloc((void **)&c, (size_t)cap * st * 4));
  HIP_TRY(hipMalloc((void **)&p, (size_t)cap * d.Hj * 4));
  if (bp.cap) {
    HIP_TRY(hipMemcpyAsync(h, bp.h, (size_t)bp.cap * st * 4, hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipMemcpyAsync(c, bp.c, (size_t)bp.cap * st * 4, hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipMemcpyAsync(p, bp.p, (size_t)bp.cap * d.Hj * 4, hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    (void)hipFree(bp.h); (void)hipFree(bp.c); (void)hipFree(bp.p);
  }
  bp.h = h; bp.c = c; bp.p = p; bp.cap = cap;
  return WIND_OK;
}

void beam_pool_free(wind_model *m) {
  BeamPool &bp = m->beam_pool;
  if (bp.h) (void)hipFree(bp.h);
  if (bp.c) (void)hipFree(bp.c);
  if (bp.p) (void)hipFree(bp.p);
  if (bp.e_all) (void)hipFree(bp.e_all);
  if (bp.d_stage) (void)hipFree(bp.d_stage);
  if (bp.h_stage) (void)hipHostFree(bp.h_stage);
  if (bp.h_res) (void)hipHostFree(bp.h_res);
  bp = BeamPool{};
}

// One prediction-network step for `rows` (at most 32) new label sequences.
void beam_enqueue_decoder_step(wind_model *m, int rows, const int *parent, const int *child, const int *tok, hipStream_t s) {
  const ModelDev &d = m->dev;
  BeamPool &bp = m->beam_pool;
  const BeamIndex pa = beam_inline(parent, rows), ch = beam_inline(child, rows), tk = beam_inline(tok, rows);
  constexpr int R = 4;
  const unsigned lb = (unsigned)((d.Hp + 3) / 4), pb = (unsigned)((d.Hj + 3) / 4);
  for (int l = 0; l < d.L; ++l) {
    if (m->dtype == WIND_BF16) beam_lstm_layer_kernel<bf16_t, R><<<lb, 256, 0, s>>>(d, bp.h, bp.c, l, rows, pa, ch, tk);
    else beam_lstm_layer_kernel<float, R><<<lb, 256, 0, s>>>(d, bp.h, bp.c, l, rows, pa, ch, tk);
  }
  if (m->dtype == WIND_BF16) beam_pred_kernel<bf16_t, R><<<pb, 256, 0, s>>>(d, bp.h, bp.p, rows, ch);
  else beam_pred_kernel<float, R><<<pb, 256, 0, s>>>(d, bp.h, bp.p, rows, ch);
}

struct BeamNode {
  int parent, token, depth, slot;
};
struct BeamHyp {
  int node;
  double score;
  int sym;                   // labels already placed on the frame the hypothesis rests on
  std::vector<int> frames;   // frame of every label
};

double beam_logaddexp(double a, double b) {
  if (a == -INFINITY) return b;
  if (b == -INFINITY) return a;
  const double mx = a > b ? a : b;
  return mx + std::log(std::exp(a - mx) + std::exp(b - mx));
}

int beam_decode(wind_model *m, const float *enc_out, int T, int window, int K, int S, int prefix_mode, int32_t *out_tokens,
                int32_t *out_frames, int cap, int32_t *out_count, double *out_score, wind_beam_stats *stats,
                wind_beam_round_fn on_round, void *user, void *stream) {
  if (!m || (!enc_out && T > 0) || !out_tokens || !out_frames || !out_count || !out_score)
    return fail(WIND_ERR_ARG, "null argument");
  if (T < 0 || cap < 0) return fail(WIND_ERR_ARG, "T and cap must not be negative");
  if (window < 1 || window > kBeamMaxWindow) return fail(WIND_ERR_ARG, "window must have 1..64 frames");
  if (K < 1 || K > kBeamMaxK) return fail(WIND_ERR_ARG, "K must be in 1..32");
  if (S < 1) return fail(WIND_ERR_ARG, "S must be at least 1");
  if (prefix_mode < WIND_PREFIX_OFF || prefix_mode > WIND_PREFIX_REMOVE) return fail(WIND_ERR_ARG, "unknown prefix mode");
  wind_beam_stats st{};
  *out_count = 0;
  *out_score = 0.0;
  if (stats) *stats = st;
  if (T == 0) return WIND_OK;

  const ModelDev &d = m->dev;
  hipStream_t s = (hipStream_t)stream;
  BeamPool &bp = m->beam_pool;
  const int V = d.V, V1 = V + 1;
  BeamWs ws;
  int rc = beam_workspace(m, (size_t)window, (size_t)kBeamMaxK, (size_t)std::max(kBeamMaxK * window, kBeamCompRows), &ws);
  if (rc) return rc;
  rc = beam_pool_reserve(m, 1024, s);
  if (rc) return rc;
  // every frame through the encoder projection, once
  if ((size_t)T * d.Hj * 4 > bp.e_bytes) {
    HIP_TRY(hipStreamSynchronize(s));
    if (bp.e_all) (void)hipFree(bp.e_all);
    bp.e_all = nullptr; bp.e_bytes = 0;
    HIP_TRY(hipMalloc((void **)&bp.e_all, (size_t)T * d.Hj * 4));
    bp.e_bytes = (size_t)T * d.Hj * 4;
  }
  beam_enqueue_linear(m, d.w_enc, d.b_enc, enc_out, bp.e_all, T, d.Hj, d.D, true, s);

  // trie of label sequences; slot 0 holds the zero state, the empty sequence is one step from it on the start id
  std::vector<BeamNode> nodes;
  std::unordered_map<unsigned long long, int> child_of;
  int next_slot = 2;
  nodes.push_back(BeamNode{-1, V, 0, 1});
  const size_t slot_sz = (size_t)d.L * d.Hp;
  HIP_TRY(hipMemsetAsync(bp.h, 0, slot_sz * 4, s));
  HIP_TRY(hipMemsetAsync(bp.c, 0, slot_sz * 4, s));
  {
    const int zero_slot = 0, root_slot = 1, start_id = V;
    beam_enqueue_decoder_step(m, 1, &zero_slot, &root_slot, &start_id, s);
  }
  rc = check_launch("beam search set-up");
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(s));
  st.decoder_steps = 1;

  auto tokens_of = [&](int node) {
    std::vector<int> t((size_t)nodes[node].depth);
    for (int q = node; nodes[q].parent >= 0; q = nodes[q].parent) t[(size_t)nodes[q].depth - 1] = nodes[q].token;
    return t;
  };
  auto child_node = [&](int parent, int token) {
    const unsigned long long key = ((unsigned long long)(unsigned)parent << 32) | (unsigned)token;
    auto it = child_of.find(key);
    if (it != child_of.end()) return it->second;
    nodes.push_back(BeamNode{parent, token, nodes[parent].depth + 1, -1});
    child_of.emplace(key, (int)nodes.size() - 1);
    return (int)nodes.size() - 1;
  };
  // step 1: one entry per label sequence, probabilities added in list order; the time stamps and
  // label count of the most probable duplicate are kept (ties: smaller time stamps, then count)
  auto recombine = [&](std::vector<BeamHyp> &hyps) {
    std::vector<BeamHyp> out;
    std::unordered_map<int, size_t> at;
    std::vector<double> best_single;
    for (BeamHyp &h : hyps) {
      auto it = at.find(h.node);
      if (it == at.end()) {
        at.emplace(h.node, out.size());
        best_single.push_back(h.score);
        out.push_back(std::move(h));
        continue;
      }
      BeamHyp &g = out[it->second];
      double &bs = best_single[it->second];
      const double total = beam_logaddexp(g.score, h.score);
      const bool take = h.score > bs || (h.score == bs && (h.frames < g.frames || (h.frames == g.frames && h.sym < g.sym)));
      if (take) { g.frames = std::move(h.frames); g.sym = h.sym; bs = h.score; }
      g.score = total;
    }
    hyps.swap(out);
  };

  std::map<int, std::vector<BeamHyp>> resting;
  resting[0].push_back(BeamHyp{0, 0.0, 0, {}});
  std::vector<int> cb_len, cb_tok, cb_fr, cb_sym;
  std::vector<double> cb_score;
  while (!resting.empty()) {
    const int t = resting.begin()->first;
    if (t == T) break;
    std::vector<BeamHyp> hyps = std::move(resting.begin()->second);
    resting.erase(resting.begin());
    ++st.rounds;
    st.max_pending = std::max<int64_t>(st.max_pending, (int64_t)hyps.size());
    recombine(hyps);

    // step 2: every B receives, from each proper prefix A in the set, A's probability (as it was
    // before this step) times the probability of emitting the missing labels on frame t
    if (prefix_mode != WIND_PREFIX_OFF && hyps.size() > 1) {
      struct Pair { size_t a, b; };
      std::vector<Pair> pairs;
      std::unordered_map<int, int> row_of;   // child node X -> row holding log P(label(X) | t, decoder(parent(X)))
      std::vector<int> row_node;
      std::unordered_map<int, size_t> hyp_of;
      for (size_t i = 0; i < hyps.size(); ++i) hyp_of.emplace(hyps[i].node, i);
      for (size_t b = 0; b < hyps.size(); ++b) {
        int q = hyps[b].node;
        for (int up = 1; up < S && nodes[q].parent >= 0; ++up) {
          q = nodes[q].parent;
          auto it = hyp_of.find(q);
          if (it == hyp_of.end() || hyps[it->second].sym + up >= S) continue;
          pairs.push_back(Pair{it->second, b});
          for (int x = hyps[b].node; x != q; x = nodes[x].parent)
            if (row_of.emplace(x, (int)row_node.size()).second) row_node.push_back(x);
        }
      }
      if (!pairs.empty()) {
        std::vector<float> lp(row_node.size());
        for (size_t r0 = 0; r0 < row_node.size(); r0 += kBeamCompRows) {
          const int rows = (int)std::min<size_t>(kBeamCompRows, row_node.size() - r0);
          int *slot = bp.h_stage, *tok = slot + kBeamCompRows;
          for (int r = 0; r < rows; ++r) {
            const BeamNode &x = nodes[row_node[r0 + r]];
            slot[r] = nodes[x.parent].slot;
            tok[r] = x.token;
          }
          BeamIndex si, ti;
          if (rows <= kBeamInline) {
            si = beam_inline(slot, rows); ti = beam_inline(tok, rows);
          } else {
            HIP_TRY(hipMemcpyAsync(bp.d_stage, slot, sizeof(int) * 2 * kBeamCompRows, hipMemcpyHostToDevice, s));
            si = beam_list(bp.d_stage); ti = beam_list(bp.d_stage + kBeamCompRows);
          }
          beam_enqueue_logits(m, ws, bp.e_all + (size_t)t * d.Hj, 1, bp.p, si, rows, s);
          beam_token_logp_kernel<<<(unsigned)rows, 256, 0, s>>>(ws.logits, V1, ti, (float *)bp.d_res + kBeamResComp);
          rc = check_launch("beam prefix step");
          if (rc) return rc;
          HIP_TRY(hipStreamSynchronize(s));
          std::memcpy(lp.data() + r0, (float *)bp.h_res + kBeamResComp, sizeof(float) * rows);
          st.completion_rows += rows;
        }
        std::vector<double> before(hyps.size());
        for (size_t i = 0; i < hyps.size(); ++i) before[i] = hyps[i].score;
        std::vector<char> removed(hyps.size(), 0);
        std::vector<int> chain;
        for (const Pair &pr : pairs) {
          double completion = 0.0;
          // labels in sequence order: collect the chain from B up to A, then add from A's side
          chain.clear();
          for (int x = hyps[pr.b].node; x != hyps[pr.a].node; x = nodes[x].parent) chain.push_back(x);
          for (size_t i = chain.size(); i-- > 0;) completion += (double)lp[(size_t)row_of[chain[i]]];
          hyps[pr.b].score = beam_logaddexp(hyps[pr.b].score, before[pr.a] + completion);
          removed[pr.a] = 1;
          ++st.completions;
        }
        if (prefix_mode == WIND_PREFIX_REMOVE) {
          std::vector<BeamHyp> kept;
          for (size_t i = 0; i < hyps.size(); ++i)
            if (!removed[i]) kept.push_back(std::move(hyps[i]));
          hyps.swap(kept);
        }
      }
    }

    // step 3: the K most probable (ties: shorter, then lexicographically smaller label sequence)
    {
      std::vector<std::vector<int>> toks(hyps.size());
      std::vector<size_t> order(hyps.size());
      for (size_t i = 0; i < hyps.size(); ++i) { order[i] = i; }
      auto less = [&](size_t a, size_t b) {
        if (hyps[a].score != hyps[b].score) return hyps[a].score > hyps[b].score;
        const int da = nodes[hyps[a].node].depth, db = nodes[hyps[b].node].depth;
        if (da != db) return da < db;
        if (toks[a].empty() && da) toks[a] = tokens_of(hyps[a].node);
        if (toks[b].empty() && db) toks[b] = tokens_of(hyps[b].node);
        return toks[a] < toks[b];
      };
      std::sort(order.begin(), order.end(), less);
      std::vector<BeamHyp> kept;
      for (size_t i = 0; i < order.size() && i < (size_t)K; ++i) kept.push_back(std::move(hyps[order[i]]));
      hyps.swap(kept);
    }
    const int Bh = (int)hyps.size();

    // prediction-network step for the survivors whose label sequence is new
    {
      int rows = 0, parent[kBeamMaxK], child[kBeamMaxK], tok[kBeamMaxK];
      for (const BeamHyp &h : hyps) {
        BeamNode &nd = nodes[h.node];
        if (nd.slot >= 0) continue;
        nd.slot = next_slot++;
        parent[rows] = nodes[nd.parent].slot; child[rows] = nd.slot; tok[rows] = nd.token;
        ++rows;
      }
      if (rows) {
        if (next_slot > bp.cap) {
          rc = beam_pool_reserve(m, next_slot, s);
          if (rc) return rc;
        }
        beam_enqueue_decoder_step(m, rows, parent, child, tok, s);
        st.decoder_steps += rows;
      }
    }

    // scoring step: the window's joiner rows, P' and the K best pairs of every hypothesis
    const int n = std::min(window, T - t);
    {
      int slots[kBeamMaxK];
      for (int b = 0; b < Bh; ++b) slots[b] = nodes[hyps[b].node].slot;
      beam_enqueue_logits(m, ws, bp.e_all + (size_t)t * d.Hj, n, bp.p, beam_inline(slots, Bh), Bh, s);
    }
    beam_enqueue_topk(m, ws, n, Bh, K, (int32_t *)bp.d_res + kBeamResLabels, (int32_t *)bp.d_res + kBeamResJumps,
                      (float *)bp.d_res + kBeamResScores, s);
    rc = check_launch("beam scoring");
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(s));
    st.hyps_scored += Bh;
    const float *scores = (const float *)bp.h_res + kBeamResScores;
    const int32_t *labels = (const int32_t *)bp.h_res + kBeamResLabels, *jumps = (const int32_t *)bp.h_res + kBeamResJumps;

    if (on_round) {
      cb_len.clear(); cb_tok.clear(); cb_fr.clear(); cb_sym.clear(); cb_score.clear();
      for (const BeamHyp &h : hyps) {
        const std::vector<int> tk = tokens_of(h.node);
        cb_len.push_back((int)tk.size());
        cb_tok.insert(cb_tok.end(), tk.begin(), tk.end());
        cb_fr.insert(cb_fr.end(), h.frames.begin(), h.frames.end());
        cb_sym.push_back(h.sym);
        cb_score.push_back(h.score);
      }
      on_round(user, t, n, Bh, cb_len.data(), cb_tok.data(), cb_fr.data(), cb_score.data(), cb_sym.data(), K, labels, jumps,
               scores);
    }

    // expansion: every chosen pair becomes a hypothesis at the frame it leads to
    for (int b = 0; b < Bh; ++b) {
      for (int k = 0; k < K; ++k) {
        const int label = labels[b * K + k], jump = jumps[b * K + k];
        if (label < 0) continue;
        BeamHyp nh;
        nh.score = hyps[b].score + (double)scores[b * K + k];
        if (label != V) {
          nh.node = child_node(hyps[b].node, label);
          nh.frames = hyps[b].frames;
          nh.frames.push_back(t + jump);
          nh.sym = jump == 0 ? hyps[b].sym + 1 : 1;
          int tn = t + jump;
          if (nh.sym >= S) { tn += 1; nh.sym = 0; }   // safeguard: leave the frame after S labels
          resting[tn].push_back(std::move(nh));
        } else {
          nh.node = hyps[b].node;
          nh.frames = hyps[b].frames;
          nh.sym = 0;
          resting[t + n].push_back(std::move(nh));
        }
      }
    }
  }

  std::vector<BeamHyp> fin;
  if (!resting.empty() && resting.begin()->first == T) fin = std::move(resting.begin()->second);
  if (fin.empty()) return fail(WIND_ERR_HIP, "beam search ended without a hypothesis");
  recombine(fin);
  size_t best = 0;
  std::vector<int> best_tok = tokens_of(fin[0].node);
  for (size_t i = 1; i < fin.size(); ++i) {
    bool better = fin[i].score > fin[best].score;
    if (fin[i].score == fin[best].score) {
      const std::vector<int> tk = tokens_of(fin[i].node);
      better = tk.size() < best_tok.size() || (tk.size() == best_tok.size() && tk < best_tok);
    }
    if (better) { best = i; best_tok = tokens_of(fin[i].node); }
  }
  st.nodes = (int64_t)nodes.size();
  if (stats) *stats = st;
  *out_score = fin[best].score;
  *out_count = (int32_t)best_tok.size();
  if ((int)best_tok.size() > cap) return fail(WIND_ERR_OVERFLOW, "the best hypothesis has more labels than cap");
  for (size_t i = 0; i < best_tok.size(); ++i) { out_tokens[i] = best_tok[i]; out_frames[i] = fin[best].frames[i]; }
  return WIND_OK;
}

}  // namespace

// The search keeps its hypotheses in standard containers; nothing they throw may cross the C boundary.
extern "C" int wind_beam_decode(wind_model *m, const float *enc_out, int T, int window, int K, int S, int prefix_mode,
                                int32_t *out_tokens, int32_t *out_frames, int cap, int32_t *out_count, double *out_score,
                                wind_beam_stats *stats, wind_beam_round_fn on_round, void *user, void *stream) {
  try {
    return beam_decode(m, enc_out, T, window, K, S, prefix_mode, out_tokens, out_frames, cap, out_count, out_score, stats,
                       on_round, user, stream);
  } catch (const std::exception &e) {
    return fail(WIND_ERR_HIP, std::string("beam search: ") + e.what());
  } catch (...) {
    return fail(WIND_ERR_HIP, "beam search: unknown exception");
  }
}
