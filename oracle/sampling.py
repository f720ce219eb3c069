"""TEST INFRASTRUCTURE ONLY - non-greedy verification: draft tokens are sampled from the averaged
draft distributions and checked by the rejection test of speculative sampling, so that the emitted
stream is distributed exactly like token-by-token sampling from the backbone.

The paper evaluates a match test between draft and greedy prediction (Sec. 3.3) but speaks of
predicted distributions that are averaged (supplement, "Integrating the three levels"); this module is the
reading of "verify" for sampled decoding, with the standard acceptance rule:

  target   p = softmax(logits[:n] / T) over the n admissible tokens,
  proposal q = the averaged draft distribution over the same n tokens, renormalised
             (a draft token that did not come from q - replayed, corrected or supplied by the caller -
              counts as a proposal that puts all its mass on that token),
  accept the draft x with probability min(1, p(x) / q(x));  on the first rejection emit a token from
  the residual max(p - q, 0) / sum and stop;  if every draft is accepted emit one more token from p.

Random numbers are counter based, keyed by (seed, sequence, absolute position of the token decided,
purpose): purpose 0 draws the draft, 1 decides acceptance, 2 draws the residual / extra token.  Both
sides implement the same integer recipe (synth_inputs.replay_uniform), so they draw identical numbers.

Sampling from weights w with a uniform u is the inverse CDF in index order:
the smallest i with w_0 + ... + w_i > u * sum(w).
"""
from __future__ import annotations

import numpy as np

import synth_inputs as si

DRAFT, ACCEPT, RESAMPLE = 0, 1, 2


def uniform(seed: int, seq: int, pos: int, purpose: int) -> float:
    return si.replay_uniform(seed * 3 + purpose, seq, pos)


def inverse_cdf(w, u: float) -> int:
    """Smallest index whose cumulative weight exceeds u * total; weights need not be normalised."""
    w = np.asarray(w, dtype=np.float64)
    c = np.cumsum(w)
    hit = np.nonzero(c > u * c[-1])[0]
    if len(hit):
        return int(hit[0])
    return int(np.nonzero(w > 0)[0][-1])     # only reachable through rounding when u is next to 1


def target_row(logits, n: int, temperature: float):
    z = np.asarray(logits[:n], dtype=np.float64) / temperature
    e = np.exp(z - z.max())
    return e / e.sum()


def proposal_row(dist, n: int):
    q = np.asarray(dist[:n], dtype=np.float64)
    return q / q.sum()


def accept_draft(p, q, x: int, u_acc: float) -> bool:
    """Rejection test for draft token x; q = None stands for the proposal with all its mass on x."""
    if x >= len(p):
        return False
    qx = 1.0 if q is None else q[x]
    return u_acc * qx < p[x]


def residual(p, q, x: int):
    """Weights the replacement of a rejected draft is drawn from."""
    if q is None:
        r = p.copy()
        if x < len(p):
            r[x] = 0.0
    else:
        r = np.maximum(p - q, 0.0)
    return r if r.sum() > 0.0 else p


def verify_rows(ps, qs, block, us_acc, us_res):
    """ps[i]: target row after block[i]; qs[i]: proposal block[i + 1] was drawn from (None = point mass).
    Returns (accepted length a, the token emitted after block[a - 1])."""
    B = len(block)
    a = 1
    while a < B and accept_draft(ps[a - 1], qs[a - 1], block[a], us_acc[a - 1]):
        a += 1
    i = a - 1
    w = ps[i] if a == B else residual(ps[i], qs[i], block[a])
    return a, inverse_cdf(w, us_res[i])
