"""Speculative-sampling verification of a drafted block on the CPU, in float64 (Sec. II-A: the acceptance
probability eq. ss_accept_prob, the residual distribution eq. ss_residual, and their sequential use over
a K-token block).

TEST INFRASTRUCTURE ONLY: imported by tests/.  The product never imports this module and this module
imports nothing of the product.

The definitions are written out as the section states them; nothing is blocked, fused or reordered.
What the section leaves open is fixed here (the same readings the library documents):
  * the uniform numbers are inputs: u_j decides position j (accept iff u_j < alpha_j), v picks the emitted
    token by inverse CDF in token-id order: the smallest id whose cumulative weight exceeds v times the total;
  * position 0 of a block is checked against the stream's pending token (the token the previous round
    emitted): its target distribution is the point mass there, so alpha_0 is 1 or 0 and a rejection at
    position 0 emits the pending token; the drafter's distribution of position 0 is not used;
  * a drafted token to which the drafter gives probability zero is accepted (the ratio is unbounded);
  * when every position is accepted the emitted token is drawn from the target distribution after the block.
"""
from __future__ import annotations

import numpy as np


def softmax(logits) -> np.ndarray:
    """p_T( . | x): the softmax of one row of logits, float64."""
    z = np.asarray(logits, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def accept_prob(p_t: np.ndarray, p_d: np.ndarray, y: int) -> float:
    """alpha(x, y) = min{1, p_T(y|x) / p_D(y|x)} (eq. ss_accept_prob)."""
    if p_d[y] <= p_t[y]:          # ratio >= 1, zero denominators included
        return 1.0
    return float(p_t[y] / p_d[y])


def residual(p_t: np.ndarray, p_d: np.ndarray) -> np.ndarray:
    """The unnormalised residual weights p_T - alpha(x, .) p_D (eq. ss_residual).  alpha(x, i) p_D(i) is
    min{p_D(i), p_T(i)}, which is how it is evaluated: the weight is exactly zero where p_D >= p_T."""
    p_t = np.asarray(p_t, dtype=np.float64)
    p_d = np.asarray(p_d, dtype=np.float64)
    return p_t - np.minimum(p_d, p_t)


def inverse_cdf(w: np.ndarray, v: float) -> int:
    """The smallest index i with w_0 + ... + w_i > v * sum(w), for nonnegative weights and v in [0, 1)."""
    w = np.asarray(w, dtype=np.float64)
    c = np.cumsum(w)
    target = float(v) * c[-1]
    hit = np.nonzero(c > target)[0]
    if hit.size:
        return int(hit[0])
    return int(np.nonzero(w > 0)[0][-1])    # v * total rounded up to the total itself


def verify_block(logits, pending: int, tokens, draft_probs, u, v: float):
    """One stream, one block.  logits [k, V]: row j is the target's output after tokens[j]; tokens [k];
    draft_probs [k, V]: row j is the drafter's distribution tokens[j] was drawn from (row 0 unused);
    u [k], v: uniforms in [0, 1).  Returns (accepted length A, emitted token, alpha [k])."""
    tokens = np.asarray(tokens)
    k = tokens.size
    p_t = [None] + [softmax(logits[j - 1]) for j in range(1, k)]
    alpha = np.empty(k, dtype=np.float64)
    alpha[0] = 1.0 if int(tokens[0]) == int(pending) else 0.0
    for j in range(1, k):
        alpha[j] = accept_prob(p_t[j], np.asarray(draft_probs[j], dtype=np.float64), int(tokens[j]))
    for j in range(k):
        if u[j] < alpha[j]:
            continue
        if j == 0:
            return 0, int(pending), alpha
        return j, inverse_cdf(residual(p_t[j], draft_probs[j]), v), alpha
    return k, inverse_cdf(softmax(logits[k - 1]), v), alpha
