"""CPU oracle for probabilistic verification: VERIFY with the draft model's probabilities.

TEST INFRASTRUCTURE ONLY (see oracle/oracle.py).

The paper's VERIFY takes the draft tokens together with the draft model's probability
distributions (Background, Eq. 2; Methodology Step 2, Eq. 5; Appendix "System Design", Alg. 2,
LISTENER) and leaves the criterion to the speculative-decoding scheme it builds on (its
reference for Eq. 1-2: speculative sampling).  That scheme, restated:

  q_i = softmax(z_i / T) is the target model's distribution at row i (z_i = logits of the row
  whose input is the token before draft i+1), p_i the draft model's distribution from which
  draft x_{i+1} was drawn.  Going through the drafts in order, draft x is kept with probability
  min(1, q_i(x) / p_i(x)); at the first draft that is not kept the row emits a token drawn from
  the normalised positive part of q_i - p_i and the round ends; if all gamma drafts are kept,
  row gamma emits a token drawn from q_gamma.  The emitted sequence is then distributed exactly
  as if the target model had sampled it.

The random numbers are inputs: u[i] decides whether draft i+1 is kept (kept iff
u[i] * p_i(x) < q_i(x)), v[i] picks the token row i emits, by inversion of the cumulative sum
taken in token order: the first token k with  sum_{j<=k} w_j > v[i] * sum_j w_j.

Every head of a pass (exits and final) applies the same rule to its own logits with the same u
and v.  Everything is float64; no blocking or reordering.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence

import numpy as np


def target_distribution(z: np.ndarray, temperature: float) -> np.ndarray:
    """softmax(z / T) of one row."""
    z = np.asarray(z, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())
    return e / e.sum()


def inverse_cdf(w: np.ndarray, v: float):
    """Token drawn from the weights w (>= 0, not all zero) with the uniform number v in [0, 1):
    the first k whose cumulative weight exceeds v * total.  Also returns how far v * total is
    from the two ends of that token's interval (in units of w)."""
    w = np.asarray(w, dtype=np.float64)
    c = np.cumsum(w)
    target = float(v) * c[-1]
    k = int(np.searchsorted(c, target, side="right"))   # first k with c[k] > target
    if k >= w.size:                                     # only by rounding: v * total == total
        k = int(np.nonzero(w > 0)[0][-1])
    lo = c[k - 1] if k > 0 else 0.0
    return k, min(target - lo, c[k] - target)


def residual_weights(q: np.ndarray, p: np.ndarray) -> np.ndarray:
    """Positive part of q - p: what the target model wants more of than the draft model gave."""
    return np.maximum(q - np.asarray(p, dtype=np.float64), 0.0)


@dataclass
class SampledHead:
    accept_len: int            # delta: drafts kept
    tokens: np.ndarray         # [gamma+1] token row i emits if the round ends at row i
    kept: np.ndarray           # [gamma] draft i+1 passes its own test (independent of earlier rows)
    keep_gap: np.ndarray       # [gamma] |u p(x) - q(x)|: distance of the keep test from its threshold
    q_draft: np.ndarray        # [gamma] q_i(x_{i+1})
    cdf_gap: np.ndarray        # [gamma+1] distance of v * total from the chosen token's interval ends
    next_token: int            # tokens[accept_len]


def speculative_verify(logits: np.ndarray, drafts: Sequence[int], draft_probs: np.ndarray, u: Sequence[float],
                       v: Sequence[float], temperature: float = 1.0) -> SampledHead:
    """One head: logits [gamma+1][V], drafts [gamma], draft_probs [gamma][V], u [gamma], v [gamma+1]."""
    logits = np.asarray(logits, dtype=np.float64)
    gamma = len(drafts)
    assert logits.shape[0] == gamma + 1 and len(u) == gamma and len(v) == gamma + 1
    tokens = np.zeros(gamma + 1, dtype=np.int64)
    kept = np.zeros(gamma, dtype=bool)
    keep_gap = np.zeros(gamma)
    q_draft = np.zeros(gamma)
    cdf_gap = np.zeros(gamma + 1)
    for i in range(gamma + 1):
        q = target_distribution(logits[i], temperature)
        if i < gamma:
            p = np.asarray(draft_probs[i], dtype=np.float64)
            x = int(drafts[i])
            kept[i] = float(u[i]) * p[x] < q[x]
            keep_gap[i] = abs(float(u[i]) * p[x] - q[x])
            q_draft[i] = q[x]
            w = residual_weights(q, p)
            if not w.sum() > 0.0:      # q == p: the draft is always kept and this row never emits
                w = q
        else:
            w = q
        tokens[i], cdf_gap[i] = inverse_cdf(w, float(v[i]))
    delta = 0
    while delta < gamma and kept[delta]:
        delta += 1
    return SampledHead(delta, tokens, kept, keep_gap, q_draft, cdf_gap, int(tokens[delta]))
