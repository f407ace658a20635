"""CPU oracle for the whole WIND beam search (test infrastructure, not a product path).

Follows the section "A Novel Beam-search Algorithm for WIND", Algorithm 3, step by step: a map
(`resting`) from frame to the hypotheses that rest there; the hypotheses of the smallest frame are
taken out, merged, extended by their prefixes and pruned (merge_extend_prune: the three steps the
section lists under the algorithm), scored on the window
enc[t : t+n] with P'(v, t) of Eq. 1 (oracle/beam_scores.py), and each of their K best (label, jump)
pairs is put back at the frame it leads to.  Scores are natural-log probabilities in fp64; the
model pieces (decoder step, joiner) are the C oracle's.

Readings where the paper is silent or leaves the detail to its implementation:
  * Safeguard (footnote to Algorithm 3): the greedy rule is reused.  A hypothesis counts the labels
    it has put on its current frame (`sym`); a label found at jump 0 adds one, a label found further
    in restarts the count at 1; when the count reaches S the hypothesis moves one frame on and the
    count clears, at no cost in score.  An all-blank window clears the count.
  * Step 1 of merge_extend_prune, duplicates: probabilities are added (log-add-exp); the
    time stamps and the label count of the more probable duplicate are kept (equal scores: the
    lexicographically smaller time stamps, then the smaller count).
  * Step 2, prefixes: for every pair (A, B) with A a proper prefix of B, the probability of
    completing A into B on the current frame t is prod_k P(B[k] | t, decoder(B[:k])), k from |A| to
    |B|-1.  A completion must be a path the safeguard allows: sym(A) + |B| - |A| < S.  Every B
    receives, from each such A, A's probability AS IT WAS BEFORE THIS STEP times the completion
    (so that mass handed A0 -> A -> B is not counted again on top of A0 -> B).
    What happens to A: the section's sentence says A is removed; the work it credits for this
    function (Kim et al. 2020, Section II-B) only adds to B and leaves A in the set.  Taken
    literally the removal deletes the most probable short hypothesis whenever any extension of it
    rests on the same frame, and on the synthetic models here the search then returns
    near-maximal-length outputs with far lower scores (tests/test_oracle_beam_search_pins.py
    measures it).  Default: the credited definition, A stays ("keep"; A's own later expansion on
    this frame may then put the same paths into B's sequence a second time, as in that work); the
    literal sentence is available as prefix_step="remove"; "off" skips step 2.
  * Step 3: the K most probable survive (equal scores: shorter, then lexicographically smaller
    token sequence).
  * An expansion slot with probability zero (K larger than the number of non-zero entries) adds
    nothing.
  * The result is the most probable entry of resting[T] after its duplicates have been combined as
    in step 1 (no prefix step: no frame is left to complete on).  T = 0 returns the empty
    hypothesis with score 0.

Every discrete choice (which K pairs, which duplicate's time stamps, which K hypotheses, which
final hypothesis) is recorded together with its margin: the score gap to the best alternative not
chosen.  Choices between hypotheses compare accumulated scores; the choice of a hypothesis' K
pairs compares entries of one window, whose common history cancels: the two kinds are kept apart.  An implementation in lower precision may legitimately choose differently where a margin
is below its error, and only there; the comparison protocol in tests/ uses these margins.

Pins (tests/test_oracle_beam_search_pins.py): brute-force enumeration of every alignment of tiny
lattices, the greedy decoder at beam 1 / window 1, alignment log-probabilities at beam 1, hand-built
prefix sets, and a second writing of the whole search from the section's prose (flat table, decoder
rebuilt from nothing, probabilities multiplied as Eq. 1 prints them) that must agree on every final
hypothesis in all three prefix modes.  Parity unpinned: the readings listed above themselves (safeguard, duplicates, what
happens to a prefix, tie rules), for which the paper refers to its implementation; the pins fix
what follows from Eq. 1 and the printed steps of Algorithm 3 under those readings.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

from . import beam_scores as bs


def logaddexp(a: float, b: float) -> float:
    if a == -np.inf:
        return b
    if b == -np.inf:
        return a
    m = max(a, b)
    return m + float(np.log(np.exp(a - m) + np.exp(b - m)))


@dataclass
class Hyp:
    tokens: Tuple[int, ...]
    frames: Tuple[int, ...]      # frame at which each token was emitted
    score: float                 # log probability
    sym: int = 0                 # labels already placed on the frame the hypothesis rests on


@dataclass
class Round:
    """What one pass of the while-loop saw and chose (for the lockstep comparison)."""
    t: int
    n: int
    hyps: List[Hyp]                                  # after merge_extend_prune, best first
    expansions: List[List[Tuple[int, int, float]]]   # per hypothesis: (label, jump, log P'), best first
    margin: float                                    # smallest gap of a choice between hypotheses (steps 1, 3)
    expansion_margin: float = np.inf                 # smallest gap between a hypothesis' K-th and (K+1)-th pair
    n_completions: int = 0                           # (A, B) pairs handled by the prefix step


class DecoderCache:
    """decoder(tokens) for every token sequence the search touches, each computed from its parent by
    one step of the C oracle's prediction network."""

    def __init__(self, model):
        self.model = model
        L, Hp = model.L, model.Hp
        h = np.zeros(L * Hp, np.float64)
        c = np.zeros(L * Hp, np.float64)
        model.decoder_step(model.V, h, c)            # decoder([]): the start id from zero state
        self.state: Dict[Tuple[int, ...], Tuple[np.ndarray, np.ndarray]] = {(): (h, c)}

    def out(self, tokens: Tuple[int, ...]) -> np.ndarray:
        if tokens not in self.state:
            self.out(tokens[:-1])
            h, c = (a.copy() for a in self.state[tokens[:-1]])
            self.model.decoder_step(tokens[-1], h, c)
            self.state[tokens] = (h, c)
        h = self.state[tokens][0]
        Hp = self.model.Hp
        return h[(self.model.L - 1) * Hp:]


def _hyp_order(h: Hyp):
    return (-h.score, len(h.tokens), h.tokens)


def recombine(hyps: List[Hyp]) -> Tuple[List[Hyp], float]:
    """Step 1: one entry per token sequence (in order of first appearance), probabilities added in
    list order.  Also returns the smallest score gap between the duplicate whose time stamps are
    kept and a duplicate with other time stamps or label count."""
    margin = np.inf
    groups: Dict[Tuple[int, ...], List[Hyp]] = {}
    for h in hyps:
        groups.setdefault(h.tokens, []).append(h)
    out = []
    for tokens, g in groups.items():
        rep = min(g, key=lambda h: (-h.score, h.frames, h.sym))
        total = -np.inf
        for h in g:
            total = logaddexp(total, h.score)
            if (h.frames, h.sym) != (rep.frames, rep.sym):
                margin = min(margin, rep.score - h.score)
        out.append(Hyp(tokens, rep.frames, total, rep.sym))
    return out, margin


def merge_extend_prune(hyps: List[Hyp], K: int, S: int,
                                  log_prob: Callable[[Tuple[int, ...], int], float],
                                  prefix_step: str = "keep") -> Tuple[List[Hyp], float, int]:
    """The three steps listed under Algorithm 3.  log_prob(prefix, v) = log P(v | current frame,
    decoder(prefix)).  Returns (survivors best first, margin, number of (A, B) completions)."""
    hyps, margin = recombine(hyps)
    n_pairs = 0
    assert prefix_step in ("keep", "remove", "off")
    if prefix_step != "off":
        before = {h.tokens: h.score for h in hyps}
        removed = set()
        for B in hyps:
            for A in hyps:
                la, lb = len(A.tokens), len(B.tokens)
                if la >= lb or B.tokens[:la] != A.tokens or A.sym + lb - la >= S:
                    continue
                completion = 0.0
                for k in range(la, lb):
                    completion += log_prob(B.tokens[:k], B.tokens[k])
                B.score = logaddexp(B.score, before[A.tokens] + completion)
                removed.add(A.tokens)
                n_pairs += 1
        if prefix_step == "remove":
            hyps = [h for h in hyps if h.tokens not in removed]
    hyps.sort(key=_hyp_order)
    if len(hyps) > K:
        margin = min(margin, hyps[K - 1].score - hyps[K].score)
        hyps = hyps[:K]
    return hyps, margin, n_pairs


def expansion_margin(logp: np.ndarray, K: int) -> float:
    """Gap between the K-th and the (K+1)-th best entry of log P' (inf if there is no (K+1)-th)."""
    flat = np.sort(logp[np.isfinite(logp)])[::-1]
    return float(flat[K - 1] - flat[K]) if flat.size > K else np.inf


def wind_beam_search(model, enc: np.ndarray, N: int, K: int, S: int, prefix_step: str = "keep",
                     expansions_per_hyp: Optional[int] = None, trace: Optional[List[Round]] = None):
    """Algorithm 3 on one utterance: enc [T, D] encoder outputs, window N, beam K, at most S labels
    per frame.  expansions_per_hyp defaults to K (the algorithm's [B, K] arrays); the brute-force
    pin sets both to "everything".  Returns (best Hyp, final list of resting[T] after recombination,
    smallest margin of the final choice)."""
    enc = np.asarray(enc, dtype=np.float32)
    T = enc.shape[0]
    Kx = K if expansions_per_hyp is None else expansions_per_hyp
    dec = DecoderCache(model)
    resting: Dict[int, List[Hyp]] = {0: [Hyp((), (), 0.0, 0)]}
    while resting:
        t = min(resting.keys())
        if t == T:
            break
        hyps = resting.pop(t)

        dist = {}                                  # log P(. | t, decoder(prefix)), evaluated once per prefix

        def log_prob(prefix, v, t=t, dist=dist):
            if prefix not in dist:
                dist[prefix] = bs.log_softmax(model.joiner(enc[t], dec.out(prefix)))
            return float(dist[prefix][v])

        hyps, margin, n_pairs = merge_extend_prune(hyps, K, S, log_prob, prefix_step)
        n = min(N, T - t)
        dec_out = np.stack([dec.out(h.tokens) for h in hyps])
        labels, jumps, scores, full = bs.beam_window(model, enc[t:t + n], dec_out, Kx)
        rec = Round(t, n, [Hyp(h.tokens, h.frames, h.score, h.sym) for h in hyps], [], margin, n_completions=n_pairs)
        for b, hyp in enumerate(hyps):
            rec.expansion_margin = min(rec.expansion_margin, expansion_margin(full[b], Kx))
            rec.expansions.append([(int(labels[b, k]), int(jumps[b, k]), float(scores[b, k]))
                                   for k in range(Kx) if labels[b, k] >= 0])
            for k in range(Kx):
                label, jump = int(labels[b, k]), int(jumps[b, k])
                if label < 0:
                    continue
                if label != model.V:
                    sym = hyp.sym + 1 if jump == 0 else 1
                    tn = t + jump
                    if sym >= S:                       # safeguard: leave the frame after S labels
                        tn, sym = tn + 1, 0
                    new = Hyp(hyp.tokens + (label,), hyp.frames + (t + jump,), hyp.score + scores[b, k], sym)
                    resting.setdefault(tn, []).append(new)
                else:
                    new = Hyp(hyp.tokens, hyp.frames, hyp.score + scores[b, k], 0)
                    resting.setdefault(t + n, []).append(new)
        if trace is not None:
            trace.append(rec)
    final, margin = recombine(resting.get(T, [Hyp((), (), 0.0, 0)]) if T > 0 else [Hyp((), (), 0.0, 0)])
    final.sort(key=_hyp_order)
    if len(final) > 1:
        margin = min(margin, final[0].score - final[1].score)
    return final[0], final, margin
