"""Stochastic acceptance at temperature T > 0 (test oracle).

Section 3.3, Eq. 6 of the paper: draft token d drawn from P_S is kept with
probability min(1, P_H(d) / P_S(d)); every draft before the first rejection is
kept; at the rejection a correction token is drawn from the residual
distribution norm(max(0, P_H - P_S)).  The committed token then follows P_H
exactly, whatever P_S was.

Readings the paper leaves open: (1) when all k drafts are kept the round emits
one more token drawn from P_H at position k+1 (the rule of the work Eq. 6 cites;
the greedy path does the same with the argmax); (2) P = softmax(logits / T);
(3) drawing from a distribution p with a uniform u in [0, 1) is the inverse
CDF in index order: the smallest i with p_0 + ... + p_i > u * sum(p).

The random numbers come from a counter-based generator so that any decision can
be recomputed alone: uniform(seed, b, idx, purpose) is the (c+1)-th output of
SplitMix64 (Steele, Lea, Flood 2014) started at `seed`, c = b * 2^34 + idx * 4
+ purpose, reduced to its top 24 bits; b is the sequence, idx the position of
the token in the sequence's generated stream, purpose 0 = draw a draft token,
1 = acceptance test, 2 = correction / bonus / first token.  24 bits are exact
in float32 and float64 alike.

Every function also reports a margin: how far the uniform was from flipping
the decision, so tests can reject seeds whose decisions a rounding error could
change (the analogue of the top-1/top-2 gap audit of the greedy path).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

PURPOSE_DRAFT, PURPOSE_ACCEPT, PURPOSE_CORRECT = 0, 1, 2
_MASK = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15


def splitmix64_at(seed: int, counter: int) -> int:
    """Output number `counter` (from 0) of SplitMix64 seeded with `seed`."""
    z = (seed + (counter + 1) * _GAMMA) & _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def uniform(seed: int, b: int, idx: int, purpose: int) -> float:
    """24-bit uniform in [0, 1) for (sequence b, stream position idx, purpose)."""
    c = (b << 34) + (idx << 2) + purpose
    return (splitmix64_at(seed, c) >> 40) * 2.0 ** -24


def softmax_t(logits: np.ndarray, temperature: float) -> np.ndarray:
    """softmax(logits / T) in float64."""
    z = (np.asarray(logits, np.float64) - np.max(logits)) / temperature
    e = np.exp(z)
    return e / e.sum()


def draw(p: np.ndarray, u: float) -> Tuple[int, float]:
    """Inverse CDF in index order: smallest i with p_0 + .. + p_i > u * sum(p).
    Returns (i, margin); margin = distance of u * sum(p) to the nearest CDF
    edge, relative to sum(p)."""
    c = np.cumsum(np.asarray(p, np.float64))
    total = c[-1]
    assert total > 0.0
    t = u * total
    i = int(np.searchsorted(c, t, side="right"))   # first index with c[i] > t
    if i >= len(c):
        i = len(c) - 1
    return i, float(np.min(np.abs(c - t)) / total)


def residual(p_h: np.ndarray, p_s: np.ndarray) -> np.ndarray:
    """Unnormalised residual distribution max(0, P_H - P_S) of Eq. 6."""
    return np.maximum(0.0, np.asarray(p_h, np.float64) - np.asarray(p_s, np.float64))


def stochastic_round(p_s: Sequence[np.ndarray], p_h: Sequence[np.ndarray], drafts: Sequence[int],
                     u_accept: Sequence[float], u_correct_at) -> Tuple[int, int, float]:
    """Acceptance of one round.  p_s[i], drafts[i]: draft distribution and token of
    position i (k of them); p_h[i]: full-model distribution of position i (k + 1);
    u_accept[i]: uniform of the test at position i; u_correct_at(n): uniform for the
    token emitted after n kept drafts.  Returns (n, token, margin)."""
    k = len(drafts)
    margin = np.inf
    n = k
    for i in range(k):
        d = int(drafts[i])
        if not 0 <= d < len(p_h[i]):          # not a token: rejected where it stands
            n = i
            break
        ratio = p_h[i][d] / p_s[i][d]
        margin = min(margin, abs(u_accept[i] - ratio))
        if not u_accept[i] < ratio:           # keep with probability min(1, ratio)
            n = i
            break
    if n < k:
        r = residual(p_h[n], p_s[n])
        if r.sum() > 0.0:
            tok, m = draw(r, u_correct_at(n))
        else:
            # Eq. 6 leaves this case open: the residual has no mass (in exact arithmetic a rejection
            # implies mass elsewhere, so it only arises from rounding, or from a draft id that is no
            # token).  Reading: draw from P_H with the same uniform; should that be the rejected
            # draft itself, take its successor in index order, so that the targets row (entry n
            # differs from the draft) still encodes n.
            tok, m = draw(np.asarray(p_h[n], np.float64), u_correct_at(n))
            if tok == int(drafts[n]):
                tok = (tok + 1) % len(p_h[n])
    else:
        tok, m = draw(p_h[k], u_correct_at(k))
    return n, tok, min(margin, m)


def stochastic_targets(drafts: Sequence[int], n: int, tok: int) -> List[int]:
    """The round's result in the form the commit step consumes: entry i equals the
    draft for the kept positions, entry n is the emitted token, later entries -1
    (the longest-matching-prefix rule then returns n, since a correction token never
    equals the rejected draft: the residual is zero there)."""
    k = len(drafts)
    return [int(drafts[i]) for i in range(n)] + [int(tok)] + [-1] * (k - n)
