"""GPU parity of wind_beam_window_scores (Eq. 1 and the scoring step of Algorithm 3) against the fp64 oracle
in oracle/beam_scores.py on the same seeded inputs.  Scores: 1e-4 absolute for fp32 models, 2e-2 for
bf16 models (the tolerances of the logits they are made of).  The chosen (label, jump) pairs must
be the oracle's, except that entries whose oracle scores lie closer together than the tolerance may
swap places or, at the K-th position, replace one another."""
import numpy as np
import pytest

import oracle
import wind_inputs as wi
from oracle import beam_scores as bs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def hypotheses(o, cfg, rng, Bh, max_len):
    prefixes = [[]] + [rng.integers(0, cfg.V, size=rng.integers(1, max_len + 1)).tolist() for _ in range(Bh - 1)]
    return np.stack([o.decoder_from_scratch(p) for p in prefixes])


def check_against_oracle(cfg, full, K, labels, jumps, scores, tol):
    """full: oracle log P' [Bh, n, V+1]."""
    Bh, n, V1 = full.shape
    for b in range(Bh):
        ref_l, ref_j, ref_s = bs.top_expansions(full[b], K)
        n_ref = int((ref_l >= 0).sum())
        got = [(int(jumps[b, k]), int(labels[b, k])) for k in range(K)]
        assert all(g == (-1, -1) for g in got[n_ref:]) and np.isneginf(scores[b, n_ref:]).all()
        seen = set()
        for k in range(n_ref):
            t, v = got[k]
            assert 0 <= t < n and 0 <= v < V1 and (t, v) not in seen
            assert v != V1 - 1 or t == n - 1, "blank only as a jump out of the window"
            seen.add((t, v))
            true = full[b, t, v]
            assert abs(scores[b, k] - true) <= tol, (b, k, scores[b, k], true)          # the score is that entry's
            assert abs(true - ref_s[k]) <= 2 * tol, (b, k, true, ref_s[k])               # and the k-th best, up to near-ties
            if (t, v) != (int(ref_j[k]), int(ref_l[k])):
                assert abs(true - ref_s[k]) <= 2 * tol
        assert (np.diff(scores[b, :n_ref]) <= 0).all()


@pytest.mark.parametrize("n,Bh,K", [(1, 1, 1), (4, 3, 5), (16, 6, 8), (7, 2, 32)])
def test_fp32_model(torch_cuda, n, Bh, K):
    from paper_2505_13765_amd import WindModel

    cfg = wi.CONFIGS["tiny"]
    w = wi.make_weights(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    enc, lens = wi.make_batch(cfg)
    rng = np.random.default_rng(100 + n)
    g = hypotheses(o, cfg, rng, Bh, 6)
    t0 = 9
    win = np.ascontiguousarray(enc[0, t0:t0 + n])
    _, _, _, full = bs.beam_window(o, win, g, K)
    lab, jmp, sc = m.beam_window_scores(torch_cuda.from_numpy(win).cuda(), torch_cuda.from_numpy(g.astype(np.float32)).cuda(), K)
    check_against_oracle(cfg, full, K, lab, jmp, sc, 1e-4)
    # total mass of the returned entries never exceeds one
    assert (np.exp(sc.astype(np.float64)).sum(axis=1) <= 1.0 + 1e-4).all()
    m.close()


@pytest.mark.parametrize("name,n,Bh,K", [("greedy_b1", 16, 5, 8), ("greedy_b1", 3, 40, 4), ("largevocab_b128", 8, 4, 16)])
def test_bf16_models(torch_cuda, name, n, Bh, K):
    from paper_2505_13765_amd import WindModel

    cfg = wi.scaled(wi.CONFIGS[name], 1, 64, 64)
    w = wi.make_weights(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    enc, lens = wi.make_batch(cfg)
    rng = np.random.default_rng(7)
    g = hypotheses(o, cfg, rng, Bh, 5)
    win = np.ascontiguousarray(enc[0, 20:20 + n])
    _, _, _, full = bs.beam_window(o, win, g, K)
    lab, jmp, sc = m.beam_window_scores(torch_cuda.from_numpy(win).cuda(), torch_cuda.from_numpy(g.astype(np.float32)).cuda(), K)
    check_against_oracle(cfg, full, K, lab, jmp, sc, 2e-2)
    m.close()


def test_argument_errors(torch_cuda):
    from paper_2505_13765_amd import WindModel
    from paper_2505_13765_amd.binding import WindError

    cfg = wi.CONFIGS["tiny"]
    m = WindModel.from_config(cfg, wi.make_weights(cfg))
    win = torch_cuda.zeros((4, cfg.D), device="cuda")
    g = torch_cuda.zeros((2, cfg.Hp), device="cuda")
    for K in (0, 33):
        with pytest.raises(WindError):
            m.beam_window_scores(win, g, K)
    with pytest.raises(WindError):
        m.beam_window_scores(torch_cuda.zeros((65, cfg.D), device="cuda"), g, 4)
    m.close()
