"""ctypes front end of the CPU oracle (oracle/wisv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product (the HIP library and its binding) never
imports this module, and this module imports nothing of the product.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wisv_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libwisv_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (portable x86-64 code; about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-shared", "-fPIC",
                               "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim",
                                         "d_ff", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("storage", "round_bf16", "d_draft", "d_csi", "d_j", "head_act")]


_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "lm_head", "final_norm")] + \
               [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER] + \
               [(n, C.c_void_p) for n in ("head_w1", "head_b1", "head_w2", "head_b2")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_round_bf16.restype = C.c_float
        _lib.orc_round_bf16.argtypes = [C.c_float]
        _lib.orc_head_flops.restype = C.c_int64
        _lib.orc_head_flops.argtypes = [C.c_int, C.c_int]
    return _lib


def _fp(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    if torch.is_tensor(a):
        a = a.detach().to("cpu", torch.float32).numpy()
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    if torch.is_tensor(a):
        a = a.detach().cpu().numpy()
    return np.ascontiguousarray(a, dtype=np.int32)


# ---- stand-alone building blocks (for the pins) ------------------------------------------------

def round_bf16(x: float) -> float:
    return float(lib().orc_round_bf16(C.c_float(x)))


def num_threads() -> int:
    return int(lib().orc_num_threads())


def head_flops(d_in: int, d_j: int) -> int:
    return int(lib().orc_head_flops(d_in, d_j))


def rmsnorm(x, g, eps: float) -> np.ndarray:
    x, g = _f32(x), _f32(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_fp(x), _fp(g), 0, C.c_int(x.size), C.c_float(eps), _fp(out))
    return out


def linear(x, w) -> np.ndarray:
    x, w = _f32(x), _f32(w)
    rows, n_in = x.shape
    y = np.empty((rows, w.shape[0]), dtype=np.float32)
    lib().orc_linear(_fp(x), _fp(w), 0, rows, n_in, w.shape[0], _fp(y))
    return y


def rope(v, pos: int, theta: float) -> np.ndarray:
    v = _f32(v).copy()
    lib().orc_rope(_fp(v), C.c_int(v.size), C.c_int(pos), C.c_float(theta))
    return v


def attend(q, k, v) -> np.ndarray:
    """q [hd]; k, v [n, hd] -> softmax(q k^T / sqrt(hd)) v."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    n, hd = k.shape
    out = np.empty(hd, dtype=np.float32)
    buf = np.empty(n, dtype=np.float64)
    lib().orc_attend(_fp(q), _fp(k), _fp(v), n, hd, _fp(out), _fp(buf))
    return out


def argmax(z):
    z = _f32(z)
    idx, gap = C.c_int32(), C.c_float()
    lib().orc_argmax(_fp(z), C.c_int(z.size), C.byref(idx), C.byref(gap), None)
    return idx.value, gap.value


def decide(draft, t, scored, p_acc, tau: float, gate_all: bool = False):
    """Localize + threshold + first reject for one stream; see orc_decide."""
    draft, t, scored, p_acc = _i32(draft), _i32(t), _i32(scored), _f32(p_acc)
    k = draft.size
    assert t.size == k + 1 and scored.size == k and p_acc.size == k
    a, y = C.c_int32(), C.c_int32()
    mask, status = C.c_uint32(), C.c_uint32()
    lib().orc_decide(k, _fp(draft), _fp(t), _fp(scored), _fp(p_acc), C.c_float(tau), int(gate_all),
                     C.byref(a), C.byref(y), C.byref(mask), C.byref(status))
    return a.value, y.value, mask.value, status.value


# ---- the model -----------------------------------------------------------------------------------

class Oracle:
    """One target decoder + decision head held on the host.

    `weights` maps the canonical names (embed, lm_head, final_norm, attn_norm[l], wq[l], ...,
    head_w1, head_b1, head_w2, head_b2) to CPU torch tensors, float32 or bfloat16, [out, in].
    round_bf16 selects what a bf16 target keeps in bf16 besides its weights:
      "kv"   the KV cache only (default for bf16 weights): k and v are rounded when cached;
      "all"  every matrix-product operand is rounded to bf16 where it is produced;
      "none" nothing (default for float weights).  True / False mean "all" / "none".
    """

    def __init__(self, model, weights: Dict[str, object], round_bf16: Optional[bool] = None):
        self.shape = model
        bf16 = model.dtype == "bf16"
        if round_bf16 is None:
            round_bf16 = "kv" if bf16 else "none"
        mode = {"none": 0, False: 0, "kv": 1, "all": 3, True: 3}[round_bf16]
        self._keep = []
        self.m = _Model(model.n_layers, model.d_model, model.n_heads, model.n_kv_heads, model.head_dim,
                        model.d_ff, model.vocab, model.rms_eps, model.rope_theta,
                        1 if bf16 else 0, mode,
                        model.d_draft, model.d_csi, model.d_head_hidden, model.head_act)
        self.w = _Weights()
        want = torch.bfloat16 if bf16 else torch.float32

        def ptr(t: torch.Tensor):
            assert t.device.type == "cpu" and t.dtype == want and t.is_contiguous(), (t.dtype, t.device)
            self._keep.append(t)
            return C.c_void_p(t.data_ptr())

        for name in ("embed", "lm_head", "final_norm", "head_w1", "head_b1", "head_w2", "head_b2"):
            setattr(self.w, name, ptr(weights[name]))
        for name in _PER_LAYER:
            arr = (C.c_void_p * model.n_layers)(*[ptr(t) for t in weights[name]])
            self._keep.append(arr)
            setattr(self.w, name, C.cast(arr, C.POINTER(C.c_void_p)))

    # -- cache ---------------------------------------------------------------------------------
    def new_cache(self, l_max: int) -> np.ndarray:
        s = self.shape
        return np.zeros((s.n_layers, 2, s.n_kv_heads, l_max, s.head_dim), dtype=np.float32)

    # -- Verify --------------------------------------------------------------------------------
    def forward_block(self, cache: np.ndarray, L: int, tokens, want_logits: bool = False):
        s = self.shape
        tokens = _i32(tokens)
        k = tokens.size
        h_t = np.empty((k, s.d_model), dtype=np.float32)
        logits = np.empty((k, s.vocab), dtype=np.float32) if want_logits else None
        amax = np.empty(k, dtype=np.int32)
        gap = np.empty(k, dtype=np.float32)
        top1 = np.empty(k, dtype=np.float32)
        assert cache.dtype == np.float32 and cache.flags.c_contiguous
        rc = lib().orc_forward_block(C.byref(self.m), C.byref(self.w), _fp(cache), cache.shape[3], L,
                                     _fp(tokens), k, _fp(h_t), _fp(logits) if want_logits else None,
                                     _fp(amax), _fp(gap), _fp(top1))
        if rc:
            raise ValueError("orc_forward_block rejected its arguments")
        return {"h_t": h_t, "logits": logits, "argmax": amax, "gap": gap, "top1": top1}

    def prefill(self, cache: np.ndarray, tokens, chunk: int = 0) -> int:
        """Fill the cache from position 0 and return the argmax after the last token."""
        tokens = _i32(tokens)
        n = tokens.size
        chunk = chunk or n
        last = None
        for c0 in range(0, n, chunk):
            last = self.forward_block(cache, c0, tokens[c0:c0 + chunk])
        return int(last["argmax"][-1])

    # -- head ------------------------------------------------------------------------------------
    def head(self, h_d, h_t, c):
        h_d, h_t, c = _f32(h_d), _f32(h_t), _f32(c)
        s, pr, pa = C.c_float(), C.c_float(), C.c_float()
        lib().orc_head(C.byref(self.m), C.byref(self.w), _fp(h_d), _fp(h_t), _fp(c),
                       C.byref(s), C.byref(pr), C.byref(pa))
        return s.value, pr.value, pa.value

    # -- the whole round, one stream -------------------------------------------------------------
    def verify_round(self, cache: np.ndarray, L: int, pred_next: int, draft, proto: int, hd, hd_row,
                     csi, tau: float, gate_all: bool = False, want_logits: bool = False):
        s = self.shape
        draft, hd_row, csi = _i32(draft), _i32(hd_row), _f32(csi)
        hd = _f32(hd).reshape(-1, s.d_draft)
        k = draft.size
        assert hd_row.size == k and csi.size == s.d_csi
        assert hd_row.max(initial=-1) < hd.shape[0]
        out = {
            "p_accept": np.empty(k, dtype=np.float32), "p_reject": np.empty(k, dtype=np.float32),
            "t": np.empty(k + 1, dtype=np.int32), "gap": np.empty(k, dtype=np.float32),
            "top1": np.empty(k, dtype=np.float32),
            "h_t": np.empty((k, s.d_model), dtype=np.float32),
            "logits": np.empty((k, s.vocab), dtype=np.float32) if want_logits else None,
        }
        a, y = C.c_int32(), C.c_int32()
        mask, status = C.c_uint32(), C.c_uint32()
        rc = lib().orc_verify_round(
            C.byref(self.m), C.byref(self.w), _fp(cache), cache.shape[3], L, int(pred_next),
            _fp(draft), k, int(proto), _fp(hd) if hd.size else None, _fp(hd_row), _fp(csi),
            C.c_float(tau), int(gate_all), C.byref(a), C.byref(y), _fp(out["p_accept"]),
            _fp(out["p_reject"]), _fp(out["t"]), _fp(out["gap"]), _fp(out["top1"]), C.byref(mask), C.byref(status),
            _fp(out["h_t"]), _fp(out["logits"]) if want_logits else None)
        if rc:
            raise ValueError("orc_verify_round rejected its arguments")
        out.update(accepted_len=a.value, correction_token=y.value, mismatch_mask=mask.value,
                   status=status.value)
        return out
