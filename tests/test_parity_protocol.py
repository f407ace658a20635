"""The comparison protocol itself, on the CPU: planted mistakes must fail, a legitimate
near-tie divergence must pass and be counted."""
import numpy as np
import pytest

import oracle
import wind_inputs as wi
from parity import compare_utterance


def model(V=4, seed=3, bias=0.9):
    cfg = wi.WindConfig("p", seed, 1, 30, 30, 8, 6, 1, 8, 10, V, "f32", (4,), 3, 0.5)
    return cfg, wi.make_weights(cfg, blank_bias=bias, pred_gain=3.0)


def enc_for(cfg, T=30):
    return np.random.default_rng(5).standard_normal((T, cfg.D)).astype(np.float32)


def test_identical_sequences_pass():
    cfg, w = model()
    o = oracle.Oracle.from_config(cfg, w)
    enc = enc_for(cfg)
    tok, fr, _ = o.greedy(enc, cfg.S)
    assert len(tok) > 2
    assert compare_utterance(o, enc, cfg.S, tok, fr) == 0


@pytest.mark.parametrize("mistake", ["wrong_token", "shifted_frame", "dropped", "extra"])
def test_planted_mistakes_fail(mistake):
    cfg, w = model()
    o = oracle.Oracle.from_config(cfg, w)
    enc = enc_for(cfg)
    tok, fr, _ = o.greedy(enc, cfg.S)
    tok, fr = tok.copy(), fr.copy()
    if mistake == "wrong_token":
        tok[1] = (tok[1] + 1) % cfg.V
    elif mistake == "shifted_frame":
        fr[1:] += 1
        fr = np.minimum(fr, len(enc) - 1)
    elif mistake == "dropped":
        tok, fr = np.delete(tok, 1), np.delete(fr, 1)
    else:
        tok, fr = np.insert(tok, 1, tok[0]), np.insert(fr, 1, fr[0])
    with pytest.raises(AssertionError):
        compare_utterance(o, enc, cfg.S, tok, fr)


def test_exact_tie_is_followed_and_counted():
    cfg, w = model(V=5)
    o = oracle.Oracle.from_config(cfg, w)
    enc = enc_for(cfg)
    tok, fr, _ = o.greedy(enc, cfg.S)
    a = int(tok[0])
    b = (a + 1) % cfg.V
    w["w_out"][b] = w["w_out"][a]      # label b now ties with label a exactly
    w["b_out"][b] = w["b_out"][a]
    o = oracle.Oracle.from_config(cfg, w)
    tok, fr, log = o.greedy(enc, cfg.S)
    lo, hi = min(a, b), max(a, b)
    assert tok[0] == lo, "ties go to the lowest id"
    # a decoder that resolves the tie the other way, then continues as the oracle would from there
    tok2, fr2, _ = o.greedy(enc, cfg.S, forced=[(int(fr[0]), 0, hi)])
    assert tok2[0] == hi
    assert compare_utterance(o, enc, cfg.S, tok2, fr2) >= 1
