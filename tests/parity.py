"""Comparison protocol between a decoder under test and the CPU oracle.

Token and frame sequences must be equal, except that the two may part ways at a joiner
evaluation where the oracle's own top-2 logits are closer than `tol` (1e-3): there more than one
answer is correct.  At such a point the oracle is re-run for that utterance with the other
decision forced, and the comparison goes on from there.  Anything else is a failure.
"""
from __future__ import annotations

import numpy as np

INF = 1 << 30


def first_mismatch(tok_a, fr_a, tok_b, fr_b):
    n = min(len(tok_a), len(tok_b))
    for k in range(n):
        if tok_a[k] != tok_b[k] or fr_a[k] != fr_b[k]:
            return k
    return None if len(tok_a) == len(tok_b) else n


def compare_utterance(o, enc_b, S, got_tok, got_fr, tol=1e-3, max_forced=64, oracle_result=None):
    """enc_b [len, D].  Returns the number of near-tie evaluations that had to be excluded.
    Raises AssertionError on a real mismatch."""
    V = o.V
    forced = []
    tok, fr, log = oracle_result if oracle_result is not None else o.greedy(enc_b, S)
    while True:
        k = first_mismatch(tok, fr, got_tok, got_fr)
        if k is None:
            return len(forced)
        assert len(forced) < max_forced, "too many near-tie divergences"
        f_o = int(fr[k]) if k < len(tok) else INF
        f_g = int(got_fr[k]) if k < len(got_tok) else INF
        t_node = min(f_o, f_g)
        label = V if f_g > f_o else int(got_tok[k])
        assert 0 <= label <= V, f"label {label} out of range"
        assert t_node < enc_b.shape[0]
        forced.append((t_node, k, label))
        tok, fr, log = o.greedy(enc_b, S, forced=forced)
        e = log[(log["t"] == t_node) & (log["u"] == k)]
        assert len(e) == 1, f"decoder under test decided at a lattice node (t={t_node}, u={k}) the oracle never visits"
        gap = float(e[0]["v1"] - e[0]["vlabel"])
        assert gap < tol, (f"mismatch at frame {t_node}, label index {k}: got {label}, oracle argmax "
                           f"{int(e[0]['top1'])} ahead by {gap:.3e} (> {tol})")


def compare_batch(o, enc, lengths, S, got_toks, got_frs, utterances=None, tol=1e-3, threads=0):
    """enc [B,T,D].  Compares the listed utterances (default all).  Returns total exclusions."""
    B = enc.shape[0]
    utterances = list(range(B)) if utterances is None else list(utterances)
    sub_enc = np.ascontiguousarray(enc[utterances])
    sub_len = np.ascontiguousarray(np.asarray(lengths)[utterances])
    toks, frs, logs = o.greedy_batch(sub_enc, sub_len, S, want_log=True, threads=threads)
    excluded = 0
    for i, b in enumerate(utterances):
        excluded += compare_utterance(o, enc[b, : lengths[b]], S, got_toks[b], got_frs[b], tol=tol,
                                      oracle_result=(toks[i], frs[i], logs[i]))
    return excluded


def wind_counts_from_trace(frames, T, W, S):
    """Windows Algorithm 2 needs, and its jump histogram, from the emission frames of the sequential
    result: from a pointer t, a label at frame f costs (f - t) // W all-blank windows and one
    emitting window; the trailing blank frames cost ceil(r / W)."""
    hist = np.zeros(W + 1, np.int64)
    t, sym, n = 0, 0, 0
    prev = None
    for f in frames:
        full, rem = divmod(f - t, W)
        hist[W] += full
        n += full + 1
        sym = sym + 1 if (full == 0 and rem == 0 and prev == f) else 1
        t = f
        jump = rem
        if sym == S:
            t, sym, jump = t + 1, 0, jump + 1
        hist[jump] += 1
        prev = f
    full, rem = divmod(T - t, W)
    hist[W] += full
    n += full
    if rem:
        hist[rem] += 1
        n += 1
    return n, hist
