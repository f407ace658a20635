"""Pins of the CPU oracle to things other than itself (CPU only).

Each test names the passage of the paper, or the piece of mathematics, that fixes the expected
value.  The five workloads' absolute token values are printed nowhere in the paper, so they stay
"parity unpinned"; what is pinned is every step that produces them.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import wind_inputs as wi
from parity import compare_utterance, wind_counts_from_trace

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_model(seed, V=3, D=5, E=4, Hp=6, Hj=7, L=1, blank_bias=0.0, gain=3.0):
    cfg = wi.WindConfig(f"t{seed}", seed, 1, 6, 6, D, E, L, Hp, Hj, V, "f32", (2,), 4, 0.5)
    w = wi.make_weights(cfg, blank_bias=blank_bias, pred_gain=gain)
    return cfg, w


def make_enc(seed, T, D):
    return np.random.default_rng([seed, 99]).standard_normal((T, D)).astype(np.float32)


def mixed_model(seed, T, S=4, target=0.6, **kw):
    """A tiny model whose blank bias is picked from a grid so blanks and labels both occur."""
    best = None
    for bias in np.arange(-2.0, 6.01, 0.125):
        cfg, w = tiny_model(seed, blank_bias=float(bias), **kw)
        o = oracle.Oracle.from_config(cfg, w)
        _, _, log = o.greedy(make_enc(seed, T, cfg.D), S)
        rate = float((log["label"] == cfg.V).mean())
        if best is None or abs(rate - target) < best[0]:
            best = (abs(rate - target), cfg, w)
    assert best[0] < 0.4
    return best[1], best[2]


# ---------------------------------------------------------------------------------------------
# Method, remark after Algorithm 2 and Table 1: the windowed loop returns what the sequential
# loop returns, for every window size.
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_alg2_equals_alg1_every_window(seed):
    T = 23
    cfg, w = mixed_model(seed, T, V=4, L=1 + seed % 2)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(seed, T, cfg.D)
    for S in (1, 2, 4):
        tok, fr, log = o.greedy(enc, S)
        assert 0 < len(tok) and (log["label"] == cfg.V).any()
        for W in range(1, T + 4):
            tok2, fr2, calls, hist = o.wind(enc, W, S)
            assert tok2.tolist() == tok.tolist(), (S, W)
            assert fr2.tolist() == fr.tolist(), (S, W)


def test_alg2_equals_alg1_on_tiny_workload():
    cfg = wi.CONFIGS["tiny"]
    w = wi.make_weights(cfg)
    enc, lens = wi.make_batch(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    tok, fr, log = o.greedy(enc[0], cfg.S)
    assert len(tok) > 0
    for W in (1, 2, 3, 4, 5, 8, 16, 63, 64, 65, 67):
        tok2, fr2, _, _ = o.wind(enc[0], W, cfg.S)
        assert tok2.tolist() == tok.tolist() and fr2.tolist() == fr.tolist()


# Table 1 caption: window-size 1 is the standard algorithm: same joiner calls, in the same order.
@pytest.mark.parametrize("seed", [0, 5])
def test_window_one_makes_the_same_joiner_calls(seed):
    cfg, w = mixed_model(seed, 30, S=3, V=4)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(seed, 30, cfg.D)
    tok, fr, log = o.greedy(enc, 3)
    assert len(tok) > 0 and (log["label"] == cfg.V).any()
    tok2, fr2, calls, hist = o.wind(enc, 1, 3)
    assert calls[:, 0].tolist() == log["t"].tolist()
    assert (calls[:, 1] == 1).all()


# ---------------------------------------------------------------------------------------------
# Brute force on a tiny vocabulary.  For every label prefix up to a depth the decoder output is
# computed from nothing (decoder(hyp) as Algorithm 1 writes it), the table argmax joiner(enc[t],
# decoder(prefix)) is filled for every (t, prefix), and the lattice is walked with the two rules of
# "Background: RNN-T".  The oracle, which carries its decoder state incrementally, must agree.
def lattice_walk(table, T, blank, S):
    hyp, frames, t, sym = (), [], 0, 0
    while t < T:
        label = table[(t, hyp)]
        if label != blank:
            frames.append(t)
            hyp = hyp + (label,)
            sym += 1
            if sym == S:
                t, sym = t + 1, 0
        else:
            t, sym = t + 1, 0
    return list(hyp), frames


BRUTE_CASES = [(0, 2, 6, 9), (1, 3, 5, 9), (2, 2, 6, 2), (3, 3, 6, 1), (4, 1, 6, 3)]


def brute_model(seed, V, T, S, depth):
    """Smallest blank bias on a grid for which the hypothesis is non-empty and within `depth`."""
    for bias in np.arange(0.0, 6.01, 0.2):
        cfg, w = tiny_model(seed, V=V, blank_bias=float(bias))
        o = oracle.Oracle.from_config(cfg, w)
        tok, _, _ = o.greedy(make_enc(seed, T, cfg.D), S)
        if 0 < len(tok) <= depth:
            return cfg, w
    raise AssertionError("no usable bias")


@pytest.mark.parametrize("seed,V,T,S", BRUTE_CASES)
def test_brute_force_lattice(seed, V, T, S):
    depth = 5
    cfg, w = brute_model(seed, V, T, S, depth)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(seed, T, cfg.D)
    tok, fr, log = o.greedy(enc, S)
    table = {}
    for d in range(depth + 1):
        for prefix in itertools.product(range(V), repeat=d):
            g = o.decoder_from_scratch(prefix)
            for t in range(T):
                logits = o.joiner(enc[t], g)
                table[(t, prefix)] = int(np.argmax(logits))   # numpy: first maximum
    hyp, frames = lattice_walk(table, T, V, S)
    assert hyp == tok.tolist() and frames == fr.tolist()
    if S >= depth:
        # Algorithm 2, step "smallest index so that labels[i] != blank": with no cap on labels per
        # frame in play, the next emission frame is the first non-blank row of the table for the
        # current prefix, scanning from the pointer.
        for k in range(len(tok)):
            prefix = tuple(tok[:k].tolist())
            start = 0 if k == 0 else fr[k - 1]
            nb = [t for t in range(start, T) if table[(t, prefix)] != V]
            assert nb and nb[0] == fr[k]
        prefix = tuple(tok.tolist())
        assert all(table[(t, prefix)] == V for t in range(fr[-1], T))


# ---------------------------------------------------------------------------------------------
# Special case = library routine: torch.nn.LSTM and torch linear layers in fp64.
@pytest.mark.parametrize("L", [1, 2, 3])
def test_decoder_matches_torch_lstm(L):
    import torch

    cfg, w = tiny_model(7, V=5, E=9, Hp=8, Hj=6, L=L)
    o = oracle.Oracle.from_config(cfg, w)
    lstm = torch.nn.LSTM(cfg.E, cfg.Hp, num_layers=L).double()
    with torch.no_grad():
        for l in range(L):
            getattr(lstm, f"weight_ih_l{l}").copy_(torch.from_numpy(w[f"w_ih{l}"]).double())
            getattr(lstm, f"weight_hh_l{l}").copy_(torch.from_numpy(w[f"w_hh{l}"]).double())
            getattr(lstm, f"bias_ih_l{l}").copy_(torch.from_numpy(w[f"b_ih{l}"]).double())
            getattr(lstm, f"bias_hh_l{l}").copy_(torch.from_numpy(w[f"b_hh{l}"]).double())
    seq = [cfg.V, 2, 0, 4, 4, 1]
    x = torch.from_numpy(w["emb"][seq]).double().unsqueeze(1)          # [len, 1, E]
    with torch.no_grad():
        out, (hn, cn) = lstm(x)
    h = np.zeros(L * cfg.Hp)
    c = np.zeros(L * cfg.Hp)
    for i, tok in enumerate(seq):
        o.decoder_step(tok, h, c)
        np.testing.assert_allclose(h[(L - 1) * cfg.Hp:], out[i, 0].numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(h, hn[:, 0].numpy().ravel(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(c, cn[:, 0].numpy().ravel(), rtol=0, atol=1e-12)
    g = o.decoder_from_scratch(seq[1:])
    np.testing.assert_allclose(g, out[-1, 0].numpy(), rtol=0, atol=1e-12)


def test_joiner_matches_torch_linear():
    import torch
    import torch.nn.functional as F

    cfg, w = tiny_model(11, V=6, D=10, Hp=8, Hj=12)
    o = oracle.Oracle.from_config(cfg, w)
    rng = np.random.default_rng(3)
    f = rng.standard_normal(cfg.D).astype(np.float32)
    g = rng.standard_normal(cfg.Hp)
    t = lambda k: torch.from_numpy(w[k]).double()
    z = F.relu(F.linear(torch.from_numpy(f).double(), t("w_enc"), t("b_enc"))
               + F.linear(torch.from_numpy(g), t("w_pred"), t("b_pred")))
    ref = F.linear(z, t("w_out"), t("b_out")).numpy()
    got = o.joiner(f, g)
    assert got.shape == (cfg.V + 1,)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert (z.numpy() == 0).any() and (z.numpy() > 0).any()          # the activation is exercised


def test_encoder_projection_matches_torch_linear_and_the_joiner():
    """The exported encoder half of the joiner's hidden vector: torch's linear in fp64, and the joiner
    itself rebuilt around it (with the decoder half from torch), so that a wrong operand, a dropped bias
    or a transposed matrix in it shows."""
    import torch
    import torch.nn.functional as F

    cfg, w = tiny_model(12, V=5, D=9, Hp=7, Hj=11)
    o = oracle.Oracle.from_config(cfg, w)
    rng = np.random.default_rng(4)
    f = rng.standard_normal(cfg.D).astype(np.float32)
    g = rng.standard_normal(cfg.Hp)
    t = lambda k: torch.from_numpy(w[k]).double()
    e = o.encoder_projection(f)
    np.testing.assert_allclose(e, F.linear(torch.from_numpy(f).double(), t("w_enc"), t("b_enc")).numpy(), rtol=0, atol=1e-12)
    z = F.relu(torch.from_numpy(e) + F.linear(torch.from_numpy(g), t("w_pred"), t("b_pred")))
    np.testing.assert_allclose(o.joiner(f, g), F.linear(z, t("w_out"), t("b_out")).numpy(), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# Closed forms.
def test_always_blank_model():
    cfg, w = tiny_model(2, V=4, blank_bias=1e6)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(2, 37, cfg.D)
    tok, fr, log = o.greedy(enc, 3)
    assert len(tok) == 0 and log["t"].tolist() == list(range(37))
    for W in (1, 2, 5, 8, 37, 40):
        tok2, fr2, calls, hist = o.wind(enc, W, 3)
        assert len(tok2) == 0 and len(calls) == math.ceil(37 / W)
        assert calls[:, 0].tolist() == list(range(0, 37, W))
        assert hist.sum() == len(calls)


def test_never_blank_model():
    cfg, w = tiny_model(3, V=4, blank_bias=-1e6)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(3, 11, cfg.D)
    for S in (1, 2, 5):
        tok, fr, log = o.greedy(enc, S)
        assert len(tok) == 11 * S
        assert fr.tolist() == [t for t in range(11) for _ in range(S)]
        assert len(log) == 11 * S                                      # no call after the S-th label
        for W in (1, 3, 16):
            tok2, fr2, calls, hist = o.wind(enc, W, S)
            assert tok2.tolist() == tok.tolist() and fr2.tolist() == fr.tolist()
            assert len(calls) == 11 * S


def test_decoder_blind_model():
    """With W_pred = 0 and b_pred = 0 the logits depend on the frame only: a non-blank frame emits
    the same label S times, and that label is the frame's own argmax."""
    cfg, w = mixed_model(4, 40, S=3, V=5)
    w["w_pred"][:] = 0
    w["b_pred"][:] = 0
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(4, 40, cfg.D)
    S = 3
    tok, fr, log = o.greedy(enc, S)
    g0 = np.zeros(cfg.Hp)
    per_frame = [int(np.argmax(o.joiner(enc[t], g0))) for t in range(40)]
    expect_tok = [l for l in per_frame if l != cfg.V for _ in range(S)]
    expect_fr = [t for t, l in enumerate(per_frame) if l != cfg.V for _ in range(S)]
    assert 0 < len(expect_tok) < 40 * S
    assert tok.tolist() == expect_tok and fr.tolist() == expect_fr


def test_argmax_ties_go_to_lowest_id():
    cfg, w = tiny_model(5, V=4, blank_bias=0.0)
    # make label 3 an exact copy of label 1 and blank an exact copy of label 1 as well
    for k in (3, cfg.V):
        w["w_out"][k] = w["w_out"][1]
        w["b_out"][k] = w["b_out"][1]
    w["w_out"][[0, 2]] = 0
    w["b_out"][[0, 2]] = -1e6
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(5, 6, cfg.D)
    tok, fr, log = o.greedy(enc, 2)
    assert (tok == 1).all() and len(tok) == 12
    assert (log["top1"] == 1).all() and (log["v1"] == log["v2"]).all()


# ---------------------------------------------------------------------------------------------
# Invariants of the output, and the closed form that ties Algorithm 2's window count and jump
# sizes to the sequential trace.
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_invariants_and_window_count_closed_form(seed):
    T = 60
    cfg, w = mixed_model(seed, T, V=6, D=8, Hp=8, Hj=10)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(seed, T, cfg.D)
    for S in (1, 2, 4):
        tok, fr, log = o.greedy(enc, S)
        assert (np.diff(fr) >= 0).all() and (fr < T).all() and ((tok >= 0) & (tok < cfg.V)).all()
        per = np.bincount(fr, minlength=T)
        assert per.max() <= S
        forced_adv = int((per == S).sum())
        assert len(log) == T + len(tok) - forced_adv
        assert (log["u"] == np.concatenate([[0], np.cumsum(log["label"] != cfg.V)[:-1]])).all()
        for W in (1, 2, 4, 8, 16):
            tok2, fr2, calls, hist = o.wind(enc, W, S)
            n, h = wind_counts_from_trace(fr.tolist(), T, W, S)
            assert len(calls) == n, (S, W)
            assert hist.tolist() == h.tolist(), (S, W)
            assert (calls[:, 1] <= W).all() and (calls[:, 1] >= 1).all()


def test_jump_range_matches_prose():
    lo, hi_is_w = [int(x) for x in open(os.path.join(GOLDEN, "jump_prose.txt")).read().split("\n")[-2].split()]
    cfg = wi.CONFIGS["tiny"]
    o = oracle.Oracle.from_config(cfg, wi.make_weights(cfg))
    enc, _ = wi.make_batch(cfg)
    for W in (1, 2, 4):
        _, _, calls, hist = o.wind(enc[0], W, cfg.S)
        assert len(hist) == W + 1 and hist.sum() == len(calls)
        nz = np.nonzero(hist)[0]
        assert nz.min() >= lo and (nz.max() == W) == bool(hi_is_w)


def test_memory_claim():
    W, V1, floats = [int(x) for x in open(os.path.join(GOLDEN, "memory_claim.txt")).read().split("\n")[-2].split()]
    assert W * V1 == floats
    cfg = wi.CONFIGS["greedy_b1"]
    assert cfg.V + 1 == V1 and max(cfg.windows) == W


# ---------------------------------------------------------------------------------------------
# The forced-choice hook used by the comparison protocol.
def test_forced_choice_follows_the_lattice():
    V, T, S = 2, 6, 9
    cfg, w = tiny_model(0, V=V, blank_bias=0.8)
    o = oracle.Oracle.from_config(cfg, w)
    enc = make_enc(0, T, cfg.D)
    tok, fr, log = o.greedy(enc, S)
    assert 0 < len(tok) <= 3
    # force a blank where the oracle emitted its first label
    node = (int(fr[0]), 0)
    tok_f, fr_f, log_f = o.greedy(enc, S, forced=[(node[0], node[1], V)])
    table = {}
    for d in range(6):
        for prefix in itertools.product(range(V), repeat=d):
            g = o.decoder_from_scratch(prefix)
            for t in range(T):
                table[(t, prefix)] = int(np.argmax(o.joiner(enc[t], g)))
    table[(node[0], ())] = V
    hyp, frames = lattice_walk(table, T, V, S)
    assert hyp == tok_f.tolist() and frames == fr_f.tolist()
    e = log_f[(log_f["t"] == node[0]) & (log_f["u"] == 0)][0]
    assert e["label"] == V and e["top1"] == tok[0] and e["vlabel"] <= e["v1"]


def test_batch_equals_single_and_ignores_padding():
    cfg = wi.scaled(wi.CONFIGS["tiny"], 5, 7, 40)
    w = wi.make_weights(cfg)
    enc, lens = wi.make_batch(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    toks, frs, logs = o.greedy_batch(enc, lens, cfg.S, want_log=True)
    poisoned = enc.copy()
    for b in range(cfg.B):
        poisoned[b, lens[b]:] = np.nan
    toks_p, frs_p, _ = o.greedy_batch(poisoned, lens, cfg.S)
    for b in range(cfg.B):
        tok, fr, log = o.greedy(enc[b, : lens[b]], cfg.S)
        assert toks[b].tolist() == tok.tolist() == toks_p[b].tolist()
        assert frs[b].tolist() == fr.tolist() == frs_p[b].tolist()
        assert logs[b]["t"].tolist() == log["t"].tolist()
