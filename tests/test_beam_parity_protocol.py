"""The replay protocol of tests/beam_parity.py, exercised on the CPU: the oracle's own trace must pass
with no divergence, a trace with a near-tie resolved the other way must pass and be counted, and
planted mistakes (a wrong survivor, a wrong pair, a shifted score, a wrong time stamp, a search
that stops early) must each be caught."""
import copy

import numpy as np
import pytest

import oracle
import wind_inputs as wi
from beam_parity import follow
from oracle import beam_search as obs


def setup(seed=3, T=14, V=6):
    cfg = wi.WindConfig("bp", seed, 1, T, T, 8, 6, 1, 8, 10, V, "f32", (4,), 3, 0.5)
    o = oracle.Oracle.from_config(cfg, wi.make_weights(cfg, blank_bias=1.0, pred_gain=3.0))
    enc = np.random.default_rng([seed, 5]).standard_normal((T, cfg.D)).astype(np.float32)
    return o, enc


def as_device_trace(trace):
    return [{"t": r.t, "n": r.n, "hyps": [(h.tokens, h.frames, h.score, h.sym) for h in r.hyps],
             "expansions": [list(e) for e in r.expansions]} for r in trace]


@pytest.mark.parametrize("N,K,S,prefix", [(4, 3, 3, "keep"), (2, 4, 2, "remove"), (8, 2, 4, "off"), (1, 2, 2, "keep")])
def test_oracle_trace_replays_cleanly(N, K, S, prefix):
    o, enc = setup()
    trace = []
    best, _, _ = obs.wind_beam_search(o, enc, N, K, S, prefix_step=prefix, trace=trace)
    st = follow(o, enc, N, K, S, prefix, as_device_trace(trace), (best.tokens, best.frames, best.score), 1e-9)
    assert st["passes"] == len(trace) and st["other_survivors"] == st["other_pairs"] == st["other_stamps"] == 0
    assert st["max_score_err"] < 1e-9 and st["max_pair_err"] < 1e-12


def run(N=4, K=3, S=3, prefix="keep"):
    o, enc = setup()
    trace = []
    best, _, _ = obs.wind_beam_search(o, enc, N, K, S, prefix_step=prefix, trace=trace)
    return o, enc, as_device_trace(trace), (best.tokens, best.frames, best.score), (N, K, S, prefix)


def test_planted_mistakes_are_caught():
    o, enc, good, res, (N, K, S, prefix) = run()
    step = 1e-6

    def check(bad, result=res):
        with pytest.raises(AssertionError):
            follow(o, enc, N, K, S, prefix, bad, result, step)

    i = next(i for i, g in enumerate(good) if len(g["hyps"]) == K and len(g["expansions"][0]) == K)
    bad = copy.deepcopy(good)                     # a pair that is not among the K best
    l, j, s = bad[i]["expansions"][0][-1]
    worst = [(v, 0) for v in range(o.V) if (v, 0) not in {(a, b) for a, b, _ in bad[i]["expansions"][0]}][-1]
    bad[i]["expansions"][0][-1] = (worst[0], worst[1], s)
    check(bad)
    bad = copy.deepcopy(good)                     # a pair's score off by more than the bound
    l, j, s = bad[i]["expansions"][0][0]
    bad[i]["expansions"][0][0] = (l, j, s + 1e-3)
    check(bad)
    bad = copy.deepcopy(good)                     # a hypothesis' score off
    tk, fr, sc, sym = bad[i]["hyps"][1]
    bad[i]["hyps"][1] = (tk, fr, sc - 1e-2, sym)
    check(bad)
    bad = copy.deepcopy(good)                     # a survivor dropped
    bad[i]["hyps"].pop()
    bad[i]["expansions"].pop()
    check(bad)
    bad = copy.deepcopy(good)                     # a wrong time stamp
    k = next(k for k, g in enumerate(good) if any(len(h[0]) for h in g["hyps"]))
    b = next(b for b, h in enumerate(good[k]["hyps"]) if len(h[0]))
    tk, fr, sc, sym = bad[k]["hyps"][b]
    bad[k]["hyps"][b] = (tk, tuple(f + 1 for f in fr), sc, sym)
    check(bad)
    check(copy.deepcopy(good)[:-1])               # stops before the map is exhausted
    check(good, (res[0] + (0,), res[1] + (enc.shape[0] - 1,), res[2]))   # a result that is not in the final list
    check(good, (res[0], res[1], res[2] + 1.0))                          # the result's score off


def test_near_tie_resolved_the_other_way_is_accepted_and_counted():
    o, enc, good, res, (N, K, S, prefix) = run()
    # with a wide error bound every choice is ambiguous: swap the last chosen pair of some pass for the
    # best pair left out, give it its true score, and replay the oracle from there on that route
    step = 5.0
    from oracle import beam_scores as bs
    dec = obs.DecoderCache(o)
    i = next(i for i, g in enumerate(good) if len(g["expansions"][0]) == K)
    g = good[i]
    tokens = tuple(g["hyps"][0][0])
    full = bs.beam_window(o, enc[g["t"]:g["t"] + g["n"]], np.stack([dec.out(tokens)]), K + 1)
    l, j, s = int(full[0][0, K]), int(full[1][0, K]), float(full[2][0, K])
    swapped = copy.deepcopy(good[: i + 1])
    swapped[i]["expansions"][0][-1] = (l, j, s)
    # the rest of the route is unknown without rerunning; stop the trace here and expect the protocol to object
    # only to the early stop, not to the swap
    with pytest.raises(AssertionError, match="stopped with hypotheses left"):
        follow(o, enc, N, K, S, prefix, swapped, res, step)
