"""Comparison protocol for the whole beam search (Algorithm 3 of the section "A Novel Beam-search
Algorithm for WIND"): the device's search is replayed pass by pass against the fp64 oracle.

A search is a long chain of discrete choices taken on floating-point scores; two correct
implementations in different precision part ways at the first near-tie and never meet again, so the
final outputs alone say little.  Instead the oracle's arithmetic is run along the device's own
route, and every choice the device took is checked against the oracle's scores at that point:

  pass i (error bound of an accumulated score: bound_i = (i + 2 + S) * step, one step per window on the
  route plus the labels of a completion; of one window's log P': step)
    * the device must be working on the smallest frame of the map, with the window the algorithm gives;
    * its surviving hypotheses must be a valid "K most probable" of the oracle's list after
      recombination and the prefix step: right count, each survivor within 2 bound_i of the K-th
      best score, nothing better than that left out; their scores within bound_i of the oracle's;
      their time stamps and label counts those of a duplicate within 2 bound_i of the most
      probable duplicate (exactly the oracle's where no duplicate is that close);
    * the pairs chosen for each survivor must be a valid "K best" of the oracle's log P' for that
      hypothesis and window, within 2 step, and each score within step of the oracle's entry;
    * the oracle then adopts the device's choices (with its own scores) and goes on.
  end: the map must be exhausted at frame T, and the returned hypothesis must be a valid "most
  probable" of the oracle's final list, with its score within the bound.

Every place where the device's choice differs from the oracle's own is counted; a run without any
must reproduce the free-running oracle exactly.  Only oracle functions do arithmetic here.
"""
import numpy as np

from oracle import beam_scores as bs
from oracle import beam_search as obs


def follow(o, enc, N, K, S, prefix, got_trace, got_result, step):
    """got_trace: passes as recorded by WindModel.beam_decode; got_result = (tokens, frames, score).
    Returns a dict of counters.  Raises AssertionError on the first invalid choice."""
    enc = np.asarray(enc, dtype=np.float32)
    T, V = enc.shape[0], o.V
    dec = obs.DecoderCache(o)
    resting = {0: [obs.Hyp((), (), 0.0, 0)]}
    stats = {"passes": 0, "other_survivors": 0, "other_pairs": 0, "other_stamps": 0, "max_score_err": 0.0,
             "max_pair_err": 0.0}
    for i, g in enumerate(got_trace):
        bound = (i + 2 + S) * step
        assert resting, f"pass {i}: the device goes on after the map is empty"
        t = min(resting)
        assert t < T and g["t"] == t and g["n"] == min(N, T - t), (i, g["t"], t)
        pending = resting.pop(t)
        groups = {}
        for h in pending:
            groups.setdefault(h.tokens, []).append(h)
        dist = {}

        def log_prob(prefix_tokens, v):
            if prefix_tokens not in dist:
                dist[prefix_tokens] = bs.log_softmax(o.joiner(enc[t], dec.out(prefix_tokens)))
            return float(dist[prefix_tokens][v])

        ranked, _, _ = obs.merge_extend_prune(pending, 10 ** 9, S, log_prob, prefix)   # steps 1, 2; no pruning
        by_tokens = {h.tokens: h for h in ranked}
        got_h = {tuple(int(v) for v in h[0]): h for h in g["hyps"]}
        assert len(got_h) == len(g["hyps"]) == min(K, len(ranked)), (i, len(g["hyps"]), len(ranked))
        assert set(got_h) <= set(by_tokens), (i, sorted(set(got_h) - set(by_tokens)))
        kth = ranked[len(got_h) - 1].score
        for tokens, h in by_tokens.items():
            if tokens in got_h:
                assert h.score >= kth - 2 * bound, (i, tokens, h.score, kth)
            else:
                assert h.score <= kth + 2 * bound, (i, tokens, h.score, kth)
        if set(got_h) != {h.tokens for h in ranked[:len(got_h)]}:
            stats["other_survivors"] += 1
        survivors = []
        for gh in g["hyps"]:
            tokens = tuple(int(v) for v in gh[0])
            h = by_tokens[tokens]
            err = abs(gh[2] - h.score)
            assert err <= bound, (i, tokens, gh[2], h.score)
            stats["max_score_err"] = max(stats["max_score_err"], err)
            stamps = (tuple(int(f) for f in gh[1]), int(gh[3]))
            if stamps != (h.frames, h.sym):
                top = max(d.score for d in groups[tokens])
                assert any((d.frames, d.sym) == stamps and d.score >= top - 2 * bound for d in groups[tokens]), (i, tokens)
                stats["other_stamps"] += 1
            survivors.append(obs.Hyp(tokens, stamps[0], h.score, stamps[1]))

        n = g["n"]
        dec_out = np.stack([dec.out(h.tokens) for h in survivors])
        _, _, _, full = bs.beam_window(o, enc[t:t + n], dec_out, K)
        for b, hyp in enumerate(survivors):
            entries = np.sort(full[b][np.isfinite(full[b])])[::-1]
            chosen = {(int(l), int(j)): float(s) for l, j, s in g["expansions"][b]}
            assert len(chosen) == len(g["expansions"][b]) == min(K, entries.size), (i, b)
            kth_pair = entries[len(chosen) - 1]
            ref_l, ref_j, _ = bs.top_expansions(full[b], K)
            if set(chosen) != {(int(l), int(j)) for l, j in zip(ref_l, ref_j) if l >= 0}:
                stats["other_pairs"] += 1
            n_above = int((entries > kth_pair + 2 * step).sum())        # these must all have been chosen
            assert sum(1 for (l, j) in chosen if full[b][j, l] > kth_pair + 2 * step) == n_above, (i, b)
            for (label, jump), s in chosen.items():
                assert 0 <= jump < n and 0 <= label <= V and (label != V or jump == n - 1), (i, b, label, jump)
                true = full[b][jump, label]
                assert true >= kth_pair - 2 * step, (i, b, label, jump, true, kth_pair)
                assert abs(s - true) <= step, (i, b, label, jump, s, true)
                stats["max_pair_err"] = max(stats["max_pair_err"], abs(s - true))
                if label != V:
                    sym = hyp.sym + 1 if jump == 0 else 1
                    tn = t + jump
                    if sym >= S:
                        tn, sym = tn + 1, 0
                    resting.setdefault(tn, []).append(obs.Hyp(hyp.tokens + (label,), hyp.frames + (t + jump,),
                                                             hyp.score + true, sym))
                else:
                    resting.setdefault(t + n, []).append(obs.Hyp(hyp.tokens, hyp.frames, hyp.score + true, 0))
        stats["passes"] += 1

    assert set(resting) <= {T}, f"the device stopped with hypotheses left at frames {sorted(resting)}"
    pending = resting.get(T, [obs.Hyp((), (), 0.0, 0)])
    final, _ = obs.recombine(pending)
    final.sort(key=lambda h: (-h.score, len(h.tokens), h.tokens))
    bound = (len(got_trace) + 2 + S) * step
    tok, frm, score = got_result
    tokens = tuple(int(v) for v in tok)
    mine = [h for h in final if h.tokens == tokens]
    assert mine, "the returned label sequence is not in the final list"
    assert mine[0].score >= final[0].score - 2 * bound and abs(score - mine[0].score) <= bound, (score, mine[0].score, final[0].score)
    stamps = tuple(int(f) for f in frm)
    if stamps != mine[0].frames:
        top = max(d.score for d in pending if d.tokens == tokens)
        assert any(d.frames == stamps and d.score >= top - 2 * bound for d in pending if d.tokens == tokens)
        stats["other_stamps"] += 1
    if tokens != final[0].tokens:
        stats["other_survivors"] += 1
    stats["max_score_err"] = max(stats["max_score_err"], abs(score - mine[0].score))
    return stats
