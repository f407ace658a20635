"""Pins for the beam-scoring oracle (oracle/beam_scores.py): the definitions of the section "A Novel
Beam-search Algorithm for WIND" (Eq. 1; Algorithm 3's choice of the K best pairs) checked against things other than
the oracle's own formula: the probabilities' total mass, the one-frame special case against a
library softmax, a brute-force evaluation with explicit products of probabilities, limiting cases,
and brute-force top-K."""
import itertools

import numpy as np
import pytest
from scipy.special import log_softmax as scipy_log_softmax, softmax as scipy_softmax

from oracle import beam_scores as bs


def rand_logits(seed, w, V1, scale=2.0):
    return np.random.default_rng(seed).normal(0.0, scale, size=(w, V1))


@pytest.mark.parametrize("w,V1,seed", [(1, 5, 0), (3, 4, 1), (8, 33, 2), (16, 129, 3)])
def test_first_output_probabilities_sum_to_one(w, V1, seed):
    # "v is the first output in the window at frame t" over all (v, t), plus "nothing but blanks",
    # partitions the sample space: the masses must add up to one.
    lp = bs.window_log_scores(rand_logits(seed, w, V1))
    assert np.isclose(np.exp(lp[np.isfinite(lp)]).sum(), 1.0, rtol=0, atol=1e-12)


def test_zero_entries_are_exactly_the_early_blanks():
    lp = bs.window_log_scores(rand_logits(4, 5, 7))
    zero = ~np.isfinite(lp)
    expect = np.zeros_like(zero)
    expect[:4, 6] = True          # blank before the last frame of the window
    assert (zero == expect).all()


def test_one_frame_window_is_the_plain_softmax():
    x = rand_logits(5, 1, 40)
    lp = bs.window_log_scores(x)
    assert np.allclose(lp[0], scipy_log_softmax(x[0]), rtol=0, atol=1e-12)
    assert np.allclose(bs.log_softmax(x), scipy_log_softmax(x, axis=-1), rtol=0, atol=1e-12)


@pytest.mark.parametrize("w,V1,seed", [(2, 3, 10), (4, 4, 11), (5, 3, 12)])
def test_against_products_of_probabilities(w, V1, seed):
    # Eq. 1 evaluated literally, with probabilities and products instead of logs and running sums
    x = rand_logits(seed, w, V1)
    P = scipy_softmax(x, axis=-1)
    blank = V1 - 1
    lp = bs.window_log_scores(x)
    for t in range(w):
        before = 1.0
        for tp in range(t):
            before *= P[tp, blank]
        for v in range(V1):
            if v != blank:
                want = P[t, v] * before
            elif t == w - 1:
                want = before * P[t, blank]
            else:
                want = 0.0
            got = np.exp(lp[t, v]) if np.isfinite(lp[t, v]) else 0.0
            assert np.isclose(got, want, rtol=1e-12, atol=1e-300), (t, v)


def test_limiting_cases():
    w, V1 = 6, 9
    x = rand_logits(6, w, V1)
    certain_blank = x.copy()
    certain_blank[:, -1] += 80.0                       # blank certain on every frame
    lp = bs.window_log_scores(certain_blank)
    assert np.isclose(np.exp(lp[w - 1, -1]), 1.0, atol=1e-12)
    never_blank_first = x.copy()
    never_blank_first[0, -1] -= 80.0                   # frame 0 never blank: all the mass sits on t = 0
    lp = bs.window_log_scores(never_blank_first)
    assert np.isclose(np.exp(lp[0, :-1]).sum(), 1.0, atol=1e-12)
    assert np.exp(lp[1:][np.isfinite(lp[1:])]).sum() < 1e-30


@pytest.mark.parametrize("w,V1,K,seed", [(1, 4, 3, 20), (3, 5, 4, 21), (4, 6, 30, 22), (2, 3, 8, 23)])
def test_top_expansions_against_sorting_everything(w, V1, K, seed):
    lp = bs.window_log_scores(rand_logits(seed, w, V1))
    labels, jumps, scores = bs.top_expansions(lp, K)
    flat = [(lp[t, v], t, v) for t, v in itertools.product(range(w), range(V1)) if np.isfinite(lp[t, v])]
    flat.sort(key=lambda e: (-e[0], e[1], e[2]))
    n = min(K, len(flat))
    assert [(int(jumps[k]), int(labels[k])) for k in range(n)] == [(t, v) for _, t, v in flat[:n]]
    assert np.allclose(scores[:n], [s for s, _, _ in flat[:n]], rtol=0, atol=0)
    assert (labels[n:] == -1).all() and (jumps[n:] == -1).all() and np.isneginf(scores[n:]).all()
    assert (np.diff(scores[:n]) <= 0).all()
    # blank can only be chosen as "jump out of the window"
    for k in range(n):
        if labels[k] == V1 - 1:
            assert jumps[k] == w - 1


def test_ties_go_to_the_earlier_frame_then_the_lower_label():
    # all logits equal: every entry of a frame has probability 1/4, so the three labels of frame 0
    # tie at log(1/4) and beat everything on frame 1 (log(1/4) + log(1/4)); among the tied entries
    # the lower label comes first
    x = np.zeros((2, 4))
    lp = bs.window_log_scores(x)
    labels, jumps, scores = bs.top_expansions(lp, 3)
    assert jumps.tolist() == [0, 0, 0] and labels.tolist() == [0, 1, 2]
    # and with the first frame's blank certain, frame 1 ties with nothing on frame 0: earlier frame first
    y = np.zeros((2, 3))
    y[0, :2] = -80.0
    lp = bs.window_log_scores(y)
    labels, jumps, scores = bs.top_expansions(lp, 2)
    assert jumps.tolist() == [1, 1] and labels.tolist() == [0, 1]


def test_beam_window_uses_the_joiner():
    import wind_inputs as wi
    import oracle

    cfg = wi.CONFIGS["tiny"]
    w = wi.make_weights(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    enc, lens = wi.make_batch(cfg)
    g = np.stack([o.decoder_from_scratch([]), o.decoder_from_scratch([3, 1])])
    labels, jumps, scores, full = bs.beam_window(o, enc[0, 5:9], g, 4)
    assert full.shape == (2, 4, cfg.V + 1)
    for b in range(2):
        logits = np.stack([o.joiner(enc[0, 5 + t], g[b]) for t in range(4)])
        assert np.allclose(full[b], bs.window_log_scores(logits), equal_nan=True)
        assert np.isclose(np.exp(full[b][np.isfinite(full[b])]).sum(), 1.0, atol=1e-12)
