"""Wireless-informed cost-aware relabelling of speculative-decoding episodes (Sec. V-B, stage 2): smoothed
importance (eq. smooth_importance_short), the budgeted relabelling problem (eq. budget_opt_short), the threshold
rule of its Lagrangian relaxation (eq. lagrangian_short) and the entropy-regularised soft policy
(eq. soft_policy), plus the supervised instances they give the decision head (Sec. V-A, eq. bce).

Host-side arithmetic on small per-episode arrays; nothing here touches the GPU path.  The section leaves the
channel summaries open: the repair budget B(c), the multiplier lambda(c), the quality score q(c) and the
constants alpha, rho are arguments here, not models.

As the equations stand, b~_t = 1 wherever b_t = 1 (the maximum includes k = t), and a_t <= b_t confines repairs
to those positions: within one episode every admissible repair has the same weight, the threshold rule repairs all
important mismatches or none, and the soft policy is one probability per episode.  The smoothing only spreads
weight onto positions that may not be repaired.  The functions compute what is printed.
"""
from __future__ import annotations

import math
from typing import Sequence, Tuple

import numpy as np


def smoothed_importance(b: Sequence[int], alpha: float) -> np.ndarray:
    """b~_t = max over critical mismatches k of alpha^|t - k| (0 for an episode without a critical one)."""
    b = np.asarray(b, dtype=np.int64)
    crit = np.nonzero(b == 1)[0]
    if crit.size == 0:
        return np.zeros(b.size)
    t = np.arange(b.size)
    return np.power(float(alpha), np.abs(t[:, None] - crit[None, :]).min(axis=1).astype(np.float64))


def relabel_objective(b: Sequence[int], a: Sequence[int], b_tilde: Sequence[float]) -> float:
    """sum_t (b_t - a_t) b~_t: the importance mass left unrepaired."""
    return float(np.sum((np.asarray(b) - np.asarray(a)) * np.asarray(b_tilde, dtype=np.float64)))


def budget_relabel(b: Sequence[int], b_tilde: Sequence[float], budget: float) -> np.ndarray:
    """A minimiser of eq. budget_opt_short: repair the floor(budget) critical mismatches of largest b~ (earlier
    positions first among equals); a_t <= b_t and sum a_t <= budget hold by construction."""
    b = np.asarray(b, dtype=np.int64)
    bt = np.asarray(b_tilde, dtype=np.float64)
    a = np.zeros(b.size, dtype=np.int64)
    n = int(math.floor(budget + 1e-12))
    if n <= 0:
        return a
    crit = np.nonzero(b == 1)[0]
    order = crit[np.argsort(-bt[crit], kind="stable")]
    a[order[:n]] = 1
    return a


def lagrangian_rule(b: Sequence[int], b_tilde: Sequence[float], lam: float) -> np.ndarray:
    """a*_t = b_t 1{b~_t > lambda(c)}: the separable minimiser of eq. lagrangian_short."""
    return (np.asarray(b, dtype=np.int64) * (np.asarray(b_tilde, dtype=np.float64) > lam)).astype(np.int64)


def lagrangian_value(b: Sequence[int], a: Sequence[int], b_tilde: Sequence[float], lam: float, budget: float) -> float:
    """L(a; lambda) of eq. lagrangian_short."""
    return relabel_objective(b, a, b_tilde) + lam * (float(np.sum(a)) - budget)


def soft_policy(b: Sequence[int], b_tilde: Sequence[float], lam: float, rho: float) -> np.ndarray:
    """pi_t = b_t sigma((b~_t - lambda(c)) / rho) (eq. soft_policy)."""
    x = (np.asarray(b_tilde, dtype=np.float64) - lam) / rho
    return np.asarray(b, dtype=np.float64) / (1.0 + np.exp(-x))


def sample_actions(pi: Sequence[float], u: Sequence[float]) -> np.ndarray:
    """Bernoulli draws of the policy from uniform numbers in [0, 1) that the caller supplies: a_t = 1{u_t < pi_t}."""
    return (np.asarray(u, dtype=np.float64) < np.asarray(pi, dtype=np.float64)).astype(np.int64)


def training_instances(features: np.ndarray, b: Sequence[int], alpha: float, lams: Sequence[float], rho: float,
                       u: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Supervised instances of one episode (Sec. V-B "Training instances"): for every sampled channel state (one
    multiplier lambda(c) each, u[s] its uniform numbers) every mismatch t gives (x_t, y_t = a_t).  features
    [T, d]; returns (X [S T, d], y [S T])."""
    bt = smoothed_importance(b, alpha)
    xs, ys = [], []
    for s, lam in enumerate(lams):
        xs.append(np.asarray(features))
        ys.append(sample_actions(soft_policy(b, bt, lam, rho), u[s]))
    return np.concatenate(xs, axis=0), np.concatenate(ys, axis=0)


def bce_loss(p: Sequence[float], y: Sequence[int], pos_weight: float = 1.0) -> float:
    """Binary cross-entropy of eq. bce, mean over the instances; pos_weight scales the y = 1 terms (class
    balancing)."""
    p = np.clip(np.asarray(p, dtype=np.float64), 1e-12, 1.0 - 1e-12)
    y = np.asarray(y, dtype=np.float64)
    return float(np.mean(-(pos_weight * y * np.log(p) + (1.0 - y) * np.log(1.0 - p))))
