"""GPU parity of wind_beam_decode (section "A Novel Beam-search Algorithm for WIND", Algorithm 3)
against the fp64 oracle in oracle/beam_search.py on the same seeded inputs, by the replay protocol
of tests/beam_parity.py: the oracle's arithmetic runs along the device's route and every choice of
every pass (surviving hypotheses, their scores, time stamps and label counts, the chosen (label,
jump) pairs and their scores, the final result) must be valid under the oracle's scores, exact
wherever no alternative lies within the error bound.  A run in which the device never chose
differently from the oracle must equal the free-running oracle's result.
Whatever happened, the returned hypothesis must be well formed, and its score can not be below the
probability of the single alignment that its own labels and time stamps spell out (that alignment
is one of the paths summed into it), evaluated by the oracle.
Error of one window's log P' (`step`): 2e-4 where logits are fp32-accurate (fp32 models; bf16 models
with option beam_exact), 4e-2 for the bf16 MFMA pass; times the gain where the output layer has been
scaled to make the soft-max peaked (wind_inputs.sharpened), since the logits' error scales with it.
"""
import numpy as np
import pytest
from scipy.special import log_softmax

import oracle
import wind_inputs as wi
from beam_parity import follow
from oracle import beam_search as obs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def alignment_log_prob(o, enc, tokens, frames, S):
    T, V = enc.shape[0], o.V
    lp, u, t, sym = 0.0, 0, 0, 0
    while t < T:
        dist = log_softmax(o.joiner(enc[t], o.decoder_from_scratch(list(tokens[:u]))))
        if u < len(tokens) and frames[u] == t:
            lp += dist[tokens[u]]
            u, sym = u + 1, sym + 1
            if sym >= S:
                t, sym = t + 1, 0
        else:
            lp += dist[V]
            t, sym = t + 1, 0
    assert u == len(tokens)
    return lp


def replay(o, m, torch, enc, N, K, S, prefix, step, free_run=True):
    """Runs the device search, replays it against the oracle, and returns the protocol's counters."""
    got_trace = []
    tok, frm, score, st = m.beam_decode(torch.from_numpy(enc).cuda(), N, K, S, prefix, trace=got_trace)
    T, V = enc.shape[0], o.V
    # well-formed, whatever the route
    assert len(tok) == len(frm) and np.isfinite(score) and score <= 1e-6
    assert all(0 <= v < V for v in tok) and all(0 <= f < T for f in frm) and (np.diff(frm) >= 0).all()
    assert len(frm) == 0 or np.bincount(frm).max() <= S
    assert st.rounds == len(got_trace) and st.hyps_scored == sum(len(g["hyps"]) for g in got_trace)
    own = alignment_log_prob(o, enc, [int(v) for v in tok], [int(f) for f in frm], S)
    assert score >= own - (len(got_trace) + 2 + S) * step, (score, own)
    stats = follow(o, enc, N, K, S, prefix, got_trace, (tok, frm, score), step)
    assert stats["passes"] == st.rounds
    if free_run and stats["other_survivors"] == stats["other_pairs"] == stats["other_stamps"] == 0:
        best, _, _ = obs.wind_beam_search(o, enc, N, K, S, prefix_step=prefix)
        assert [int(v) for v in tok] == list(best.tokens) and [int(f) for f in frm] == list(best.frames)
        stats["equals_free_oracle"] = True
    stats["completions"] = st.completions
    return stats


# gain > 1: output layer scaled so that the soft-max is peaked like a trained model's and whole-window
# blank jumps are taken; gain 1: the flat soft-max of random weights, where the search stays on labels
@pytest.mark.parametrize("N,K,S,prefix,gain", [(4, 4, 5, "keep", 8), (16, 4, 5, "keep", 8), (16, 8, 5, "remove", 4),
                                               (1, 3, 2, "keep", 8), (8, 2, 3, "off", 8), (64, 4, 4, "keep", 4),
                                               (4, 4, 5, "keep", 1), (3, 5, 1, "keep", 1), (5, 32, 3, "keep", 1)])
def test_fp32_model_replay(torch_cuda, N, K, S, prefix, gain):
    from paper_2505_13765_amd import WindModel

    cfg = wi.CONFIGS["tiny"]
    w = wi.sharpened(wi.make_weights(cfg), float(gain))
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    enc, _ = wi.make_batch(cfg)
    stats = replay(o, m, torch_cuda, np.ascontiguousarray(enc[0, :48]), N, K, S, prefix, 2e-4 * gain)
    print(f"fp32 N={N} K={K} S={S} {prefix} gain={gain}: {stats}")
    assert stats["max_pair_err"] < 1e-4 * gain
    m.close()


@pytest.mark.parametrize("name,T,N,K,S,exact,gain", [("greedy_b1", 24, 8, 4, 3, 1, 8), ("greedy_b1", 24, 16, 4, 3, 0, 8),
                                                     ("greedy_b1", 12, 16, 4, 3, 0, 1), ("largevocab_b128", 12, 4, 3, 2, 1, 8),
                                                     ("lowblank_b256", 16, 16, 4, 3, 1, 8)])
def test_bf16_models_replay(torch_cuda, name, T, N, K, S, exact, gain):
    from paper_2505_13765_amd import WindModel

    cfg = wi.scaled(wi.CONFIGS[name], 1, T, T)
    w = wi.sharpened(wi.make_weights(cfg), float(gain))
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    m.set_option("beam_exact", exact)
    enc, _ = wi.make_batch(cfg)
    # the logits' error scales with the output layer
    stats = replay(o, m, torch_cuda, np.ascontiguousarray(enc[0]), N, K, S, "keep", (2e-4 if exact else 4e-2) * gain,
                   free_run=False)
    print(f"{name} exact={exact} gain={gain}: {stats}")
    if exact:
        assert stats["other_survivors"] == stats["other_pairs"] == stats["other_stamps"] == 0
    m.close()


@pytest.mark.parametrize("Hj,V,exact", [(640, 300, 1), (1088, 77, 1), (1088, 300, 0)])
def test_unusual_shapes_bf16_replay(torch_cuda, Hj, V, exact):
    """bf16 models with vocabularies that are not a multiple of the column tiles, small D, E, Hp, and a
    joint hidden size above 1024 (logits then come from the 128 x 128 tile kernel)."""
    from paper_2505_13765_amd import WindModel

    cfg = wi.WindConfig("odd_beam", 12, 1, 18, 18, 64, 64, 1, 64, Hj, V, "bf16", (8,), 3, 0.7)
    w = wi.sharpened(wi.make_weights(cfg, blank_bias=2.0, pred_gain=4.0), 4.0)
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    m.set_option("beam_exact", exact)
    enc, _ = wi.make_batch(cfg)
    stats = replay(o, m, torch_cuda, np.ascontiguousarray(enc[0]), 8, 4, cfg.S, "keep", (2e-4 if exact else 4e-2) * 4,
                   free_run=False)
    print(f"odd shapes Hj={Hj} V={V} exact={exact}: {stats}")
    m.close()


def test_beam_one_window_one_is_the_greedy_decoder(torch_cuda):
    # K = 1, N = 1: the best pair of every pass is the frame's argmax, so the search must return what
    # wind_sequential_decode returns (fp32 model: both take their decisions on fp32 logits).
    from paper_2505_13765_amd import WindModel

    cfg = wi.CONFIGS["tiny"]
    w = wi.make_weights(cfg)
    m = WindModel.from_config(cfg, w)
    enc, lens = wi.make_batch(cfg)
    e = torch_cuda.from_numpy(enc).cuda()
    toks, frs = m.decode(e, torch_cuda.from_numpy(lens).cuda(), None, cfg.S)
    tok, frm, score, st = m.beam_decode(e[0, : int(lens[0])].contiguous(), 1, 1, cfg.S)
    assert tok.tolist() == toks[0].tolist() and frm.tolist() == frs[0].tolist()
    assert st.completions == 0
    m.close()


def test_edges_and_errors(torch_cuda):
    from paper_2505_13765_amd import WindModel
    from paper_2505_13765_amd.binding import WindError, WIND_ERR_OVERFLOW

    cfg = wi.CONFIGS["tiny"]
    w = wi.make_weights(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    enc, _ = wi.make_batch(cfg)
    e = torch_cuda.from_numpy(enc[0]).cuda()
    tok, frm, score, st = m.beam_decode(e[:0].contiguous(), 4, 4, 3)              # no frames
    assert len(tok) == 0 and score == 0.0 and st.rounds == 0
    tok, frm, score, st = m.beam_decode(e[:1].contiguous(), 4, 4, 3)              # one frame, window larger than T
    best, _, _ = obs.wind_beam_search(o, enc[0, :1], 4, 4, 3)
    assert tok.tolist() == list(best.tokens) and abs(score - best.score) < 1e-3
    for bad in (dict(N=0), dict(N=65), dict(K=0), dict(K=33), dict(S=0)):
        args = dict(N=4, K=4, S=3)
        args.update(bad)
        with pytest.raises(WindError):
            m.beam_decode(e[:8].contiguous(), args["N"], args["K"], args["S"])
    # a result longer than cap is reported, not truncated silently
    full = m.beam_decode(e[:40].contiguous(), 4, 4, 3)
    assert len(full[0]) > 1
    with pytest.raises(WindError) as ei:
        m.beam_decode(e[:40].contiguous(), 4, 4, 3, cap=1)
    assert ei.value.code == WIND_ERR_OVERFLOW
    # the model is still usable and repeatable after the error
    again = m.beam_decode(e[:40].contiguous(), 4, 4, 3)
    assert again[0].tolist() == full[0].tolist() and again[2] == full[2]
    m.close()


def test_state_pool_growth(torch_cuda):
    # more label sequences than the pool's first allocation: states must survive the move
    from paper_2505_13765_amd import WindModel

    cfg = wi.CONFIGS["tiny"].replace(len_lo=56, len_hi=56)
    w = wi.make_weights(cfg)
    o = oracle.Oracle.from_config(cfg, w)
    m = WindModel.from_config(cfg, w)
    enc, _ = wi.make_batch(cfg)
    stats = replay(o, m, torch_cuda, np.ascontiguousarray(enc[0]), 4, 8, 4, "keep", 2e-4, free_run=False)
    tok, frm, score, st = m.beam_decode(torch_cuda.from_numpy(enc[0]).cuda(), 4, 8, 4)
    print(f"pool growth: {st.decoder_steps} decoder steps, {stats}")
    assert st.decoder_steps > 1024
    m.close()
