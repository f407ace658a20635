"""CPU oracle for the scoring step of WIND beam search (test infrastructure, not a product path).

Follows the section "A Novel Beam-search Algorithm for WIND": for one hypothesis and a window of w
frames starting at t0, P'(v, t) is the probability that v is the FIRST output in the window and
that it comes at frame t0 + t (Eq. 1):

    P'(blank, t)  = 0                                   for t < w - 1
    P'(blank, w-1) = prod_{t' < w} P(blank | t0 + t')
    P'(v, t)      = P(v | t0 + t) * prod_{t' < t} P(blank | t0 + t')     for v != blank

with P(. | t) the softmax of the joiner's V+1 logits at that frame.  Algorithm 3 then takes, for
every hypothesis, the K best (label, jump) pairs under P'.  Everything here is
fp64 numpy written straight from those definitions; plain and slow on purpose.

Readings where the paper is silent: scores are returned as log P' (the algorithm's update lines
add the logarithm of the chosen entry to the hypothesis score); equal scores are ordered by
earlier frame, then lower label id (blank, id V, counts as frame w-1); K may exceed the number of
entries with non-zero probability, in which case the tail is filled with label -1, jump -1,
score -inf.
"""
from __future__ import annotations

import numpy as np


def log_softmax(logits: np.ndarray) -> np.ndarray:
    """Row-wise log P(v | t) for logits [..., V+1], fp64."""
    x = np.asarray(logits, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    return x - m - np.log(np.exp(x - m).sum(axis=-1, keepdims=True))


def window_log_scores(logits: np.ndarray) -> np.ndarray:
    """log P'(v, t) for one hypothesis: logits [w, V+1] (blank = last column) -> [w, V+1], with
    -inf where Eq. 1 gives probability zero."""
    lp = log_softmax(logits)
    w, V1 = lp.shape
    blank = V1 - 1
    out = np.full((w, V1), -np.inf, dtype=np.float64)
    run = 0.0                                  # sum of log P(blank | t') over t' < t
    for t in range(w):
        out[t, :blank] = lp[t, :blank] + run   # v != blank: blanks before t, then v at t
        run += lp[t, blank]
    out[w - 1, blank] = run                    # blank: blanks on every frame of the window
    return out


def top_expansions(logp: np.ndarray, K: int):
    """The K best (label, jump) pairs of one hypothesis under log P' [w, V+1].  Order: score
    descending, then frame ascending, then label ascending.  Returns int32 labels [K], int32
    jumps [K] (frame offset inside the window), float64 scores [K]."""
    w, V1 = logp.shape
    entries = []
    for t in range(w):
        for v in range(V1):
            s = logp[t, v]
            if s > -np.inf:
                entries.append((-s, t, v))
    entries.sort()
    labels = np.full(K, -1, np.int32)
    jumps = np.full(K, -1, np.int32)
    scores = np.full(K, -np.inf, np.float64)
    for k, (ns, t, v) in enumerate(entries[:K]):
        labels[k], jumps[k], scores[k] = v, t, -ns
    return labels, jumps, scores


def beam_window(oracle_model, enc_window: np.ndarray, dec_out: np.ndarray, K: int):
    """Scoring step for Bh hypotheses on one window: enc_window [w, D] encoder frames, dec_out
    [Bh, Hp] prediction-network outputs of the hypotheses.  Uses the oracle's joiner for the logits.
    Returns labels [Bh, K], jumps [Bh, K], scores [Bh, K] and the full log P' [Bh, w, V+1]."""
    enc_window = np.asarray(enc_window)
    dec_out = np.asarray(dec_out, dtype=np.float64)
    Bh, w = dec_out.shape[0], enc_window.shape[0]
    V1 = oracle_model.V + 1
    full = np.zeros((Bh, w, V1), np.float64)
    labels = np.zeros((Bh, K), np.int32)
    jumps = np.zeros((Bh, K), np.int32)
    scores = np.zeros((Bh, K), np.float64)
    for b in range(Bh):
        logits = np.stack([oracle_model.joiner(enc_window[t], dec_out[b]) for t in range(w)])
        full[b] = window_log_scores(logits)
        labels[b], jumps[b], scores[b] = top_expansions(full[b], K)
    return labels, jumps, scores, full
