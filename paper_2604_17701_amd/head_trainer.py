"""Offline supervised training of the decision head (Sec. V-A: eq. mlp_form for the model, eq. bce for the loss,
"weight decay and class balancing where necessary"; Sec. V-B supplies the relabelled instances).

Host-side numpy arithmetic in float64; nothing here touches the GPU path.  The head is
    u = W1 z + b1,  s = w2 . act(u) + b2,  p = sigmoid(s)   (p: rejection probability, y = 1 means reject)
with z = [h^D ; h^T ; c] as the library builds it.  The paper fixes neither the optimiser nor the feature scaling:
this trainer standardises the features with the training set's mean and deviation, minimises the class-weighted
BCE plus an L2 penalty on W1 and w2 with Adam (Kingma & Ba), and folds the standardisation back into (W1, b1) on
export, so that the exported head runs on the raw features the verify round feeds it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

ACT_SILU, ACT_RELU = 0, 1


def _act(u: np.ndarray, act: int) -> Tuple[np.ndarray, np.ndarray]:
    """Activation and its derivative."""
    if act == ACT_RELU:
        return np.maximum(u, 0.0), (u > 0.0).astype(np.float64)
    sg = 1.0 / (1.0 + np.exp(-u))
    return u * sg, sg * (1.0 + u * (1.0 - sg))


@dataclass
class HeadParams:
    w1: np.ndarray   # [d_J, d_in]
    b1: np.ndarray   # [d_J]
    w2: np.ndarray   # [d_J]
    b2: float

    def copy(self) -> "HeadParams":
        return HeadParams(self.w1.copy(), self.b1.copy(), self.w2.copy(), float(self.b2))


def init_params(d_in: int, d_hidden: int, seed: int) -> HeadParams:
    rng = np.random.default_rng(seed)
    return HeadParams(rng.normal(0.0, 1.0 / np.sqrt(d_in), (d_hidden, d_in)), np.zeros(d_hidden),
                      rng.normal(0.0, 1.0 / np.sqrt(d_hidden), d_hidden), 0.0)


def forward(p: HeadParams, x: np.ndarray, act: int) -> np.ndarray:
    """Rejection probabilities sigmoid(s) of the rows of x (eq. head_forward)."""
    h, _ = _act(x @ p.w1.T + p.b1, act)
    return 1.0 / (1.0 + np.exp(-(h @ p.w2 + p.b2)))


def loss_and_grad(p: HeadParams, x: np.ndarray, y: np.ndarray, act: int, pos_weight: float = 1.0,
                  weight_decay: float = 0.0) -> Tuple[float, HeadParams]:
    """Class-weighted BCE (eq. bce; pos_weight scales the y = 1 terms) + weight_decay / 2 (|W1|^2 + |w2|^2), and
    its gradient."""
    n = x.shape[0]
    u = x @ p.w1.T + p.b1
    h, dh = _act(u, act)
    s = h @ p.w2 + p.b2
    # log sigmoid(s) and log(1 - sigmoid(s)) without overflow
    log_p = -np.logaddexp(0.0, -s)
    log_q = -np.logaddexp(0.0, s)
    loss = float(np.mean(-(pos_weight * y * log_p + (1.0 - y) * log_q)))
    loss += 0.5 * weight_decay * (float(np.sum(p.w1 ** 2)) + float(np.sum(p.w2 ** 2)))
    sig = np.exp(log_p)
    ds = (pos_weight * y * (sig - 1.0) + (1.0 - y) * sig) / n          # d loss / d s
    dw2 = h.T @ ds + weight_decay * p.w2
    du = np.outer(ds, p.w2) * dh
    return loss, HeadParams(du.T @ x + weight_decay * p.w1, du.sum(axis=0), dw2, float(ds.sum()))


def balanced_pos_weight(y: np.ndarray) -> float:
    """Class balancing: the y = 1 terms weigh as much in total as the y = 0 terms."""
    pos = float(np.sum(y))
    return (len(y) - pos) / pos if 0.0 < pos < len(y) else 1.0


def train(x: np.ndarray, y: np.ndarray, d_hidden: int, act: int = ACT_RELU, steps: int = 500, lr: float = 1e-2,
          weight_decay: float = 1e-4, balance: bool = True, batch: int = 0, seed: int = 0) -> Dict[str, object]:
    """Trains a head on instances (x [n, d_in] raw features, y [n] in {0, 1}).  Returns the parameters for raw
    features ("params"), the loss after every step ("losses") and the class weight used ("pos_weight").
    batch = 0: full-batch steps; otherwise seeded minibatches."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    mean, std = x.mean(axis=0), x.std(axis=0)
    std = np.where(std > 0.0, std, 1.0)
    xs = (x - mean) / std
    p = init_params(x.shape[1], d_hidden, seed)
    pw = balanced_pos_weight(y) if balance else 1.0
    rng = np.random.default_rng(seed + 1)
    m = HeadParams(np.zeros_like(p.w1), np.zeros_like(p.b1), np.zeros_like(p.w2), 0.0)
    v = m.copy()
    b1m, b2m, eps = 0.9, 0.999, 1e-8
    losses = []
    for t in range(1, steps + 1):
        idx = rng.choice(x.shape[0], batch, replace=False) if 0 < batch < x.shape[0] else slice(None)
        loss, g = loss_and_grad(p, xs[idx], y[idx], act, pw, weight_decay)
        losses.append(loss)
        for name in ("w1", "b1", "w2", "b2"):
            gn = np.asarray(getattr(g, name), dtype=np.float64)
            mn = b1m * np.asarray(getattr(m, name)) + (1.0 - b1m) * gn
            vn = b2m * np.asarray(getattr(v, name)) + (1.0 - b2m) * gn * gn
            step = lr * (mn / (1.0 - b1m ** t)) / (np.sqrt(vn / (1.0 - b2m ** t)) + eps)
            new = np.asarray(getattr(p, name)) - step
            setattr(m, name, mn if name != "b2" else float(mn))
            setattr(v, name, vn if name != "b2" else float(vn))
            setattr(p, name, new if name != "b2" else float(new))
    # fold the standardisation into the first layer: W1 ((x - mean) / std) + b1 = (W1 / std) x + (b1 - W1 mean / std)
    raw = HeadParams(p.w1 / std, p.b1 - (p.w1 / std) @ mean, p.w2.copy(), float(p.b2))
    return {"params": raw, "losses": losses, "pos_weight": pw}


def export_weights(p: HeadParams) -> Dict[str, np.ndarray]:
    """The four tensors in the layout wisv_weights takes: head_w1 [d_J, d_draft + d_model + d_csi] with columns
    ordered [h^D ; h^T ; c], head_b1 [d_J], head_w2 [d_J], head_b2 [1] (float32; cast to the target's dtype)."""
    return {"head_w1": p.w1.astype(np.float32), "head_b1": p.b1.astype(np.float32),
            "head_w2": p.w2.astype(np.float32), "head_b2": np.array([p.b2], np.float32)}
