"""Shared pieces of the GPU-vs-oracle parity tests: building a workload's inputs on both sides and
comparing one round's outputs under the stated tolerances."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import spec_sampling as ss
from oracle import wisv_oracle as wo
from paper_2604_17701_amd import binding
from wisv_inputs import configs, gen
from wisv_inputs.configs import PROTO_FH, PROTO_SH, Workload


@dataclass
class Tolerance:
    p_abs: float            # |p_accept(gpu) - p_accept(oracle)|
    logit_rel: float        # max_v |z_gpu - z_orc| / max_v |z_orc| per row
    hidden_rel: float       # same for h^T rows
    tie_margin_rel: float   # a target token may differ when the oracle's top-1 lead is below this * |top1|...
    tie_margin_abs: float   # ... or below this absolute lead
    tau_margin: float       # a gated decision may differ when |p_accept(oracle) - tau| is below this


# fp32 path: only summation order differs between the two sides.
TOL_F32 = Tolerance(p_abs=1e-5, logit_rel=1e-5, hidden_rel=1e-5, tie_margin_rel=0.0, tie_margin_abs=2e-5, tau_margin=1e-5)
# bf16 path (bf16 weights and KV cache, float activations fed to the matrix cores as two bf16 terms) against
# the oracle in its matching mode (bf16 weights, KV cache rounded to bf16, float activations).  What remains:
# float accumulation order, the 2^-17 residue of the two-term split, and rare one-ulp flips of cached k / v.
# The stated bounds are 2e-2 on logits and 1e-3 on probabilities; the path is held to far tighter ones.
TOL_BF16 = Tolerance(p_abs=1e-4, logit_rel=1e-3, hidden_rel=1e-3, tie_margin_rel=2e-2, tie_margin_abs=0.0, tau_margin=1e-4)

# Rounds of more than 16 rows (bound by the matrix cores) feed each activation to the products as ONE half-precision
# term (2^-12 relative rounding per operand instead of 2^-17).  Bounds derived from measurement at the 8B shape
# (32 layers): see the table in the design doc; still well inside the stated 2e-2 / 1e-3.
# Measured with the default classes (gate/up, down, LM head) on configs 3 and 4: logits and h^T <= 2.9e-3 relative,
# probabilities <= 5.0e-4; with all five classes 4.6e-3 and 5.4e-4.  The probability bound is the stated one.
TOL_BF16_MANY = Tolerance(p_abs=1e-3, logit_rel=1e-2, hidden_rel=1e-2, tie_margin_rel=2e-2, tie_margin_abs=0.0, tau_margin=1e-3)

# A cache filled by a real prefill through all 32 layers (instead of synthetic contents written identically on both
# sides): cached k, v are bf16, so wherever the two sides' float values straddle a rounding boundary an entry differs
# by a whole bf16 step (2^-9 relative), and those steps feed the later layers and tokens.  Measured at the 8B shape
# after 64 prefilled tokens: half the entries of the last layer's cache differ by such a step, logits and h^T of the
# following round agree to 1.7e-3 (5e-5 on identical caches).  Inherent in the bf16-cache contract, well inside the
# stated 2e-2 / 1e-3.
TOL_BF16_PREFILL = Tolerance(p_abs=5e-4, logit_rel=5e-3, hidden_rel=5e-3, tie_margin_rel=2e-2, tie_margin_abs=0.0, tau_margin=5e-4)


STATS_LOG = []     # (test tag, statistics) of every parity comparison; conftest prints them at the end of the run


def record(tag: str, stats: Dict[str, object]):
    STATS_LOG.append((tag, dict(stats)))
    print(f"\n[{tag}] {stats}", flush=True)


def to_host_weights(weights: Dict[str, object]) -> Dict[str, object]:
    return {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in weights.items()}


@dataclass
class StreamInputs:
    draft: np.ndarray
    hd: torch.Tensor            # [k, d_draft] on the host
    pred_next: int
    mismatch: List[int]         # positions the oracle localises as mismatches


class OracleSide:
    """The oracle's copy of a workload: one cache per sampled stream."""

    def __init__(self, w: Workload, host_weights, round_bf16: Optional[bool] = None):
        self.w = w
        self.orc = wo.Oracle(w.model, host_weights, round_bf16)
        self.cache: Dict[int, np.ndarray] = {}
        self.pred_next: Dict[int, int] = {}
        self._memo: Dict[int, dict] = {}

    def prefill(self, stream: int):
        c = self.orc.new_cache(self.w.ctx + self.w.k)
        self.pred_next[stream] = self.orc.prefill(c, gen.context_tokens(self.w, stream))
        self.cache[stream] = c

    def load_synthetic_kv(self, stream: int, device="cpu"):
        c = self.orc.new_cache(self.w.ctx + self.w.k)
        for l in range(self.w.model.n_layers):
            k, v = gen.synthetic_kv(self.w, stream, l, device)
            c[l, 0, :, :self.w.ctx] = k.float().cpu().numpy()
            c[l, 1, :, :self.w.ctx] = v.float().cpu().numpy()
        self.cache[stream] = c
        self.pred_next[stream] = gen.synthetic_pred_next(self.w, stream)

    def next_token_fn(self, stream: int):
        memo = self._memo.setdefault(stream, {})

        def nt(prefix):
            if not prefix:
                return self.pred_next[stream]
            key = tuple(int(t) for t in prefix)
            if key not in memo:
                memo[key] = int(self.orc.forward_block(self.cache[stream], self.w.ctx, list(key))["argmax"][-1])
            return memo[key]
        return nt

    def stream_inputs(self, stream: int) -> StreamInputs:
        draft = gen.build_drafts(self.w, stream, self.next_token_fn(stream))
        hd = gen.draft_hidden(self.w, stream)
        nt = self.next_token_fn(stream)
        mism = [j for j in range(self.w.k) if int(draft[j]) != nt([int(t) for t in draft[:j]])]
        return StreamInputs(draft, hd, self.pred_next[stream], mism)

    def round(self, stream: int, si: StreamInputs, proto: int, hd_rows, hd_row_map, csi, tau, gate_all=False,
              want_logits=False):
        return self.orc.verify_round(self.cache[stream], self.w.ctx, si.pred_next, si.draft, proto, hd_rows,
                                     hd_row_map, csi, tau, gate_all, want_logits)


def row_rel_err(a: np.ndarray, ref: np.ndarray) -> float:
    a, ref = a.astype(np.float64), ref.astype(np.float64)
    return float(np.max(np.max(np.abs(a - ref), axis=-1) / np.max(np.abs(ref), axis=-1)))


def compare_stream(gpu: Dict[str, np.ndarray], b: int, orc: Dict[str, object], k: int, tau: float, tol: Tolerance,
                   stats: Dict[str, int], gpu_logits: Optional[np.ndarray] = None):
    """Compares stream b of a GPU round with the oracle's round of that stream.

    Integers must match exactly.  The only licence: a position where the oracle's own top-1 lead is within
    the tie margin, or whose oracle accept probability is within tau_margin of tau, may decide either way;
    what depends on such a position (the rest of the stream's round) is then counted as exempt, not compared.
    The tie margin is the stated ceiling (tie_margin_rel * |top1|, or tie_margin_abs); when the GPU's logits
    of the stream's rows are given it is tightened to twice the largest logit deviation seen in that row,
    which is what a change of argmax needs.
    """
    t_g, t_o = gpu["target_argmax"][b], orc["t"]
    assert t_g[0] == t_o[0], "pred_next differs"
    stats["streams"] = stats.get("streams", 0) + 1
    for j in range(k):                                         # t[j+1] comes from logits row j
        if t_g[j + 1] != t_o[j + 1]:
            lead = float(orc["gap"][j])
            margin = max(tol.tie_margin_abs, tol.tie_margin_rel * abs(float(orc["top1"][j])))
            if gpu_logits is not None and orc.get("logits") is not None:
                dev = float(np.max(np.abs(gpu_logits[j].astype(np.float64) - orc["logits"][j])))
                margin = min(margin, 2.0 * dev)
            assert lead <= margin, \
                f"stream {b} row {j}: target token {t_g[j + 1]} != {t_o[j + 1]}, oracle lead {lead} > margin {margin}"
            stats["exempt_tie"] = stats.get("exempt_tie", 0) + 1
            return
    assert int(gpu["mismatch_mask"][b]) == orc["mismatch_mask"]
    p_g, p_o = gpu["p_accept"][b], orc["p_accept"]
    np.testing.assert_allclose(p_g, p_o, rtol=0, atol=tol.p_abs, err_msg=f"stream {b} p_accept")
    stats["max_dp"] = max(stats.get("max_dp", 0.0), float(np.max(np.abs(p_g - p_o))))
    if (int(gpu["accepted_len"][b]), int(gpu["correction_token"][b])) != (orc["accepted_len"], orc["correction_token"]):
        near = [j for j in range(k) if (orc["mismatch_mask"] >> j) & 1 and abs(float(p_o[j]) - tau) < tol.tau_margin]
        assert near, (f"stream {b}: (A, y*) = ({gpu['accepted_len'][b]}, {gpu['correction_token'][b]}) vs oracle "
                      f"({orc['accepted_len']}, {orc['correction_token']}), no probability near tau")
        stats["exempt_tau"] = stats.get("exempt_tau", 0) + 1
        return
    assert int(gpu["status"][b]) == orc["status"]
    stats["exact"] = stats.get("exact", 0) + 1


def check_invariants(gpu: Dict[str, np.ndarray], drafts: np.ndarray, k: int):
    """Properties that hold for any round whatever the values (Sec. II-A, Sec. IV-B): accepted length in
    [0, k], the correction is the target token at the first rejected position, matches are never rejected
    under the default rule."""
    a, y, t = gpu["accepted_len"], gpu["correction_token"], gpu["target_argmax"]
    drafts = drafts.reshape(-1, k)
    for b in range(a.size):
        assert 0 <= a[b] <= k
        assert y[b] == t[b, a[b]]
        mask = int(gpu["mismatch_mask"][b])
        for j in range(k):
            assert ((mask >> j) & 1) == int(drafts[b, j] != t[b, j])
        if a[b] < k:
            assert (mask >> int(a[b])) & 1, "the first rejected position must be a mismatch"
            assert y[b] != drafts[b, a[b]]
        p = gpu["p_accept"][b]
        assert np.all((p >= 0) & (p <= 1))


# ---- speculative sampling (Sec. II-A) -----------------------------------------------------------

def check_ss_stream(logits, pending, tokens, q, u, v, got_a, got_tok, got_alpha, tol, stats):
    """One stream against the oracle; logits are the oracle side's (float32 inputs or its own forward)."""
    k = len(tokens)
    a, tok, alpha = ss.verify_block(logits, pending, tokens, q, u, v)
    np.testing.assert_allclose(got_alpha, alpha, rtol=tol, atol=tol * 1e-3)
    stats["alpha_err"] = max(stats.get("alpha_err", 0.0), float(np.max(np.abs(got_alpha - alpha) / np.maximum(alpha, 1e-30))))
    decisive = all(abs(float(u[j]) - alpha[j]) > tol * max(alpha[j], 1e-30) for j in range(min(a + 1, k)))
    stats["streams"] = stats.get("streams", 0) + 1
    if not decisive:
        stats["a_inside_margin"] = stats.get("a_inside_margin", 0) + 1
        # the first position whose decision a rounding error could turn bounds what is valid
        first_soft = min(j for j in range(min(a + 1, k)) if abs(float(u[j]) - alpha[j]) <= tol * max(alpha[j], 1e-30))
        assert first_soft <= got_a <= k
        return
    assert got_a == a, (got_a, a, alpha, u)
    if a == 0:
        assert got_tok == pending
        return
    w = ss.residual(ss.softmax(logits[a - 1]), q[a]) if a < k else ss.softmax(logits[k - 1])
    c = np.cumsum(w)
    target = float(v) * c[-1]
    assert w[got_tok] > 0.0, "a token of zero weight was emitted"
    lo = c[got_tok - 1] if got_tok else 0.0
    assert lo - tol * c[-1] <= target <= c[got_tok] + tol * c[-1], (got_tok, tok, lo, c[got_tok], target)
    stats["tokens"] = stats.get("tokens", 0) + 1
    stats["tokens_equal"] = stats.get("tokens_equal", 0) + int(got_tok == tok)
