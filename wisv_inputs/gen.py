"""Seeded synthetic inputs for the WISV verify round (weights, KV cache, drafts, h^D, CSI).

Every array is a pure function of (seed, tag, element index): a counter is hashed
with the splitmix64 finaliser (Steele, Lea & Flood 2014; Vigna's public-domain
constants), 16-bit fields of the hash index a table of standard-normal quantiles.
All steps are integer or correctly-rounded IEEE element-wise operations written as
torch tensor ops, so the same call returns the same bits on the CPU and on a GPU;
the CPU oracle's side and the HIP path's side may therefore each generate their own
copy, on their own device, of any slice they need.

Nothing of the method's arithmetic lives here.
"""
from __future__ import annotations

import hashlib
import math
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch

from .configs import ModelShape, Workload, PROTO_FH, PROTO_SH

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_CHUNK = 1 << 26   # elements generated per pass (bounds the int64 temporaries)


def _signed(u: int) -> int:
    u &= _MASK64
    return u - (1 << 64) if u >= (1 << 63) else u


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def _key(seed: int, tag: str) -> int:
    h = hashlib.blake2b(tag.encode(), digest_size=8).digest()
    return _mix_int(int.from_bytes(h, "little") ^ _mix_int(seed))


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    return (x >> k) & ((1 << (64 - k)) - 1)


def _hash_words(key: int, first: int, count: int, device) -> torch.Tensor:
    """splitmix64 outputs number first .. first+count-1 of the stream `key` (int64 bit patterns)."""
    w = torch.arange(first + 1, first + 1 + count, dtype=torch.int64, device=device)
    z = w * _signed(_GOLDEN) + _signed(key)
    z = (z ^ _lsr(z, 30)) * _signed(_M1)
    z = (z ^ _lsr(z, 27)) * _signed(_M2)
    return z ^ _lsr(z, 31)


def _u16_fields(key: int, start: int, n: int, device) -> torch.Tensor:
    """Elements start .. start+n-1 of the 16-bit stream: element e is field e&3 of word e>>2."""
    w0, w1 = start >> 2, (start + n + 3) >> 2
    z = _hash_words(key, w0, w1 - w0, device)
    f = torch.stack([(z >> s) & 0xFFFF for s in (0, 16, 32, 48)], dim=1).reshape(-1)
    off = start - 4 * w0
    return f[off:off + n]


_QTABLE: Dict[str, torch.Tensor] = {}


def _quantiles(device) -> torch.Tensor:
    """65536 mid-point quantiles of N(0,1), float32; computed once on the host in float64."""
    k = str(device)
    if k not in _QTABLE:
        if "cpu" not in _QTABLE:
            from scipy.special import ndtri
            q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
            _QTABLE["cpu"] = torch.from_numpy(q.astype(np.float32))
        _QTABLE[k] = _QTABLE["cpu"].to(device)
    return _QTABLE[k]


def normal(seed: int, tag: str, shape: Sequence[int], std: float, dtype: torch.dtype,
           device="cpu", start: int = 0) -> torch.Tensor:
    """std * N(0,1) values (inverse-CDF sampling at 16-bit resolution), rounded once to `dtype`.

    `start` offsets into the element stream, so a slice of a large tensor can be regenerated alone.
    """
    n = int(np.prod(shape)) if len(shape) else 1
    out = torch.empty(n, dtype=dtype, device=device)
    key = _key(seed, tag)
    table = _quantiles(device)
    s = torch.tensor(std, dtype=torch.float32, device=device)
    for c0 in range(0, n, _CHUNK):
        c = min(_CHUNK, n - c0)
        u = _u16_fields(key, start + c0, c, device)
        out[c0:c0 + c] = (table[u] * s).to(dtype)
    return out.reshape(tuple(shape))


def randint(seed: int, tag: str, shape: Sequence[int], high: int, device="cpu") -> torch.Tensor:
    """Integers in [0, high) from 32 hash bits each (int64 tensor)."""
    n = int(np.prod(shape)) if len(shape) else 1
    z = _hash_words(_key(seed, tag), 0, (n + 1) // 2, device)
    f = torch.stack([z & 0xFFFFFFFF, _lsr(z, 32)], dim=1).reshape(-1)[:n]
    return (f % high).reshape(tuple(shape))


def uniform01(seed: int, tag: str, n: int) -> np.ndarray:
    """n float64 values in [0,1) (host only; for the handful of scalar draws)."""
    z = _hash_words(_key(seed, tag), 0, n, "cpu")
    return (_lsr(z, 11).double() / float(1 << 53)).numpy()


# --------------------------------------------------------------------------- model weights

def torch_dtype(model: ModelShape) -> torch.dtype:
    return torch.float32 if model.dtype == "f32" else torch.bfloat16


def make_weights(model: ModelShape, seed: int, device="cpu") -> Dict[str, object]:
    """Random-init target decoder + decision head in canonical [out, in] row-major layout.

    Matrices and the embedding ~ N(0, weight_std^2); RMSNorm gains 1; head biases 0.
    """
    dt = torch_dtype(model)
    d, f, v = model.d_model, model.d_ff, model.vocab
    std = model.weight_std

    def mat(tag, rows, cols):
        return normal(seed, tag, (rows, cols), std, dt, device)

    w: Dict[str, object] = {
        "embed": mat("embed", v, d),
        "lm_head": mat("lm_head", v, d),
        "final_norm": torch.ones(d, dtype=dt, device=device),
    }
    per = {k: [] for k in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")}
    for l in range(model.n_layers):
        per["attn_norm"].append(torch.ones(d, dtype=dt, device=device))
        per["wq"].append(mat(f"l{l}/wq", model.d_q, d))
        per["wk"].append(mat(f"l{l}/wk", model.d_kv, d))
        per["wv"].append(mat(f"l{l}/wv", model.d_kv, d))
        per["wo"].append(mat(f"l{l}/wo", d, model.d_q))
        per["ffn_norm"].append(torch.ones(d, dtype=dt, device=device))
        per["w_gate"].append(mat(f"l{l}/w_gate", f, d))
        per["w_up"].append(mat(f"l{l}/w_up", f, d))
        per["w_down"].append(mat(f"l{l}/w_down", d, f))
    w.update(per)
    # decision head; W1 columns ordered [h^D ; h^T ; c]  (Sec. V-A, eq. feature_concat)
    w["head_w1"] = mat("head/w1", model.d_head_hidden, model.d_in)
    w["head_b1"] = torch.zeros(model.d_head_hidden, dtype=dt, device=device)
    w["head_w2"] = normal(seed, "head/w2", (model.d_head_hidden,), std, dt, device)
    w["head_b2"] = torch.zeros(1, dtype=dt, device=device)
    return w


# --------------------------------------------------------------------------- per-stream inputs

def context_tokens(w: Workload, stream: int) -> torch.Tensor:
    return randint(w.seed, f"ctx/{stream}", (w.ctx,), w.model.vocab).to(torch.int32)


def synthetic_pred_next(w: Workload, stream: int) -> int:
    return int(randint(w.seed, f"pred_next/{stream}", (1,), w.model.vocab)[0])


def kv_std(model: ModelShape) -> float:
    """Scale of a K/V entry of this random-init decoder: weight_std * sqrt(d_model) (unit-RMS input)."""
    return model.weight_std * math.sqrt(model.d_model)


def synthetic_kv(w: Workload, stream: int, layer: int, device="cpu"):
    """Stand-in cache contents of one (stream, layer): K and V, each [n_kv_heads, ctx, head_dim]."""
    m = w.model
    shape = (m.n_kv_heads, w.ctx, m.head_dim)
    dt = torch_dtype(m)
    k = normal(w.seed, f"kv/{stream}/{layer}/k", shape, kv_std(m), dt, device)
    v = normal(w.seed, f"kv/{stream}/{layer}/v", shape, kv_std(m), dt, device)
    return k, v


def draft_hidden(w: Workload, stream: int, device="cpu") -> torch.Tensor:
    """Drafter final-layer hidden states of the K drafted positions, [k, d_draft], N(0,1)."""
    return normal(w.seed, f"hd/{stream}", (w.k, w.model.d_draft), 1.0, torch_dtype(w.model), device)


def csi_features(w: Workload) -> np.ndarray:
    """[batch, 4] float32: SNR dB, bandwidth MHz, rate = bw*log2(1+SNR_linear) Mbit/s, latency ms."""
    b = w.batch
    u = uniform01(w.seed, "csi", 4 * b).reshape(b, 4)
    if w.rayleigh_snr:
        snr_lin = 10.0 ** 1.5 * (-np.log1p(-u[:, 0]))     # Exp(1) power fading round 15 dB
        snr_db = 10.0 * np.log10(np.maximum(snr_lin, 1e-12))
    else:
        snr_db = 30.0 * u[:, 0]
        snr_lin = 10.0 ** (snr_db / 10.0)
    bw = np.array([5.0, 10.0, 20.0])[np.minimum((u[:, 1] * 3).astype(np.int64), 2)]
    rate = bw * np.log2(1.0 + snr_lin)
    lat = 5.0 + 45.0 * u[:, 3]
    return np.stack([snr_db, bw, rate, lat], axis=1).astype(np.float32)


def match_rates(w: Workload) -> np.ndarray:
    lo, hi = w.match_rate
    return lo + (hi - lo) * uniform01(w.seed, "match_rate", w.batch)


def draft_plan(w: Workload, stream: int):
    """Random part of a stream's draft block: per position a keep-the-target's-token flag and a
    uniformly drawn alternative token."""
    r = match_rates(w)[stream]
    keep = uniform01(w.seed, f"draft/keep/{stream}", w.k) < r
    alt = randint(w.seed, f"draft/alt/{stream}", (w.k,), w.model.vocab).numpy().astype(np.int64)
    if w.uniform_drafts:
        keep = np.zeros(w.k, dtype=bool)
    return keep, alt


def build_drafts(w: Workload, stream: int, next_token: Callable[[List[int]], int]) -> np.ndarray:
    """Draft block of one stream, built against a target's greedy chain.

    `next_token(prefix)` returns the target's argmax token for the position that follows the
    cached context and the already-drafted `prefix` (whoever calls decides which implementation
    supplies it).  A kept position copies that token; any other takes the random alternative
    (moved by one if it happens to coincide), so the kept flags are exactly the match pattern.
    Uniform-draft workloads ignore the chain.
    """
    keep, alt = draft_plan(w, stream)
    v = w.model.vocab
    if w.uniform_drafts:
        return alt.astype(np.int32)
    out: List[int] = []
    for j in range(w.k):
        t = int(next_token(list(out)))
        if keep[j]:
            out.append(t)
        else:
            a = int(alt[j])
            out.append(a if a != t else (a + 1) % v)
    return np.asarray(out, dtype=np.int32)


def pack_hidden(w: Workload, hd_by_stream: Sequence[torch.Tensor],
                mismatch_by_stream: Sequence[Sequence[int]]):
    """Assemble the uploaded drafter-hidden buffer and its row map for one round.

    FH streams upload all K rows; SH streams only the rows of their mismatch positions, in
    ascending (stream, position) order.  Returns (hd [n_hd, d_draft], hd_row int32 [batch*k]).
    """
    rows, row_map = [], np.full(w.batch * w.k, -1, dtype=np.int32)
    for b in range(w.batch):
        if w.protos[b] == PROTO_FH:
            pos = range(w.k)
        else:
            pos = sorted(mismatch_by_stream[b])
        for j in pos:
            row_map[b * w.k + j] = len(rows)
            rows.append(hd_by_stream[b][j])
    if rows:
        hd = torch.stack(rows, dim=0).contiguous()
    else:
        hd = torch.zeros((0, w.model.d_draft), dtype=torch_dtype(w.model))
    return hd, row_map


# --------------------------------------------------------------------------- speculative-sampling inputs

def unit_uniforms(seed: int, tag: str, n: int) -> np.ndarray:
    """n float32 values in [0, 1): the uniform numbers a stochastic verifier consumes (inputs on both sides)."""
    u = uniform01(seed, tag, n).astype(np.float32)
    return np.minimum(u, np.float32(1.0) - np.float32(2.0 ** -24))


def target_logits(seed: int, rows: int, vocab: int, scale: float) -> np.ndarray:
    """Stand-in target logits [rows, vocab]: N(0, scale^2); a scale of 3-4 gives the peaked next-token
    distributions of a trained decoder, a scale below 1 the flat ones of a random-weight target."""
    return normal(seed, "ss_logits", (rows, vocab), scale, torch.float32).numpy()


def draft_distributions(seed: int, rows: int, vocab: int, tokens: np.ndarray, token_mass: np.ndarray,
                        zero_frac: float = 0.25) -> np.ndarray:
    """Stand-in drafter distributions [rows, vocab] (float32, each row sums to 1 up to rounding): log-normal
    weights, a share zero_frac of the entries exactly zero (a truncated drafter), normalised to 1 - token_mass[r],
    plus token_mass[r] on the drafted token tokens[r]."""
    w = torch.exp(normal(seed, "ss_q", (rows, vocab), 1.5, torch.float32).double())
    keep = randint(seed, "ss_q_zero", (rows, vocab), 1 << 16) >= int(zero_frac * (1 << 16))
    w = (w * keep).numpy()
    w[:, 0] += 1e-3                                     # no row is empty
    mass = np.asarray(token_mass, dtype=np.float64).reshape(rows, 1)
    q = w / w.sum(axis=1, keepdims=True) * (1.0 - mass)
    q[np.arange(rows), np.asarray(tokens).reshape(rows)] += mass[:, 0]
    return q.astype(np.float32)
