"""ctypes binding of libwisv.so: argument marshalling only.

Every step of the verify round runs in the library's HIP kernels.  PyTorch is used for
device memory (weights, inputs, outputs are torch tensors whose data_ptr() is handed over)
and for the HIP stream.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "libwisv.so")

WISV_OK, WISV_EINVAL, WISV_ENOMEM, WISV_EHIP, WISV_ESTATE, WISV_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
WISV_F32, WISV_BF16 = 0, 1
WISV_PROTO_FH, WISV_PROTO_SH = 0, 1
WISV_ACT_SILU, WISV_ACT_RELU = 0, 1
WISV_FLAG_GATE_ALL, WISV_FLAG_NO_COMMIT, WISV_FLAG_DEVICE_IO, WISV_FLAG_KEEP_LOGITS = 1, 2, 4, 8
WISV_FLAG_VERIFY_ONLY, WISV_FLAG_DECIDE_ONLY = 16, 32
WISV_STATUS_MISSING_HIDDEN = 1
WISV_DBG_HIDDEN, WISV_DBG_LOGITS = 0, 1
WISV_MAX_K = 16
WISV_OPT_ONE_TERM_CLASSES = 1
WISV_TERM_QKV, WISV_TERM_O, WISV_TERM_GATE_UP, WISV_TERM_DOWN, WISV_TERM_LM_HEAD = 1, 2, 4, 8, 16
WISV_TERM_ALL = 31

EXPORTS = ("wisv_ctx_create", "wisv_verify_round", "wisv_destroy", "wisv_prefill", "wisv_set_state",
           "wisv_get_state", "wisv_kv_import", "wisv_kv_export", "wisv_debug_copy", "wisv_last_round_ms",
           "wisv_profile_enable", "wisv_profile_collect", "wisv_profile_read", "wisv_calibration_copy", "wisv_last_error",
           "wisv_ss_verify_round", "wisv_ss_decide", "wisv_ss_decide_static", "wisv_set_option", "wisv_get_option")


class WisvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"wisv error {code}: {msg}")
        self.code = code


class wisv_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ff", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "d_draft", "d_csi", "d_head_hidden", "head_act", "max_batch",
                                         "max_ctx", "max_k", "device_id")] + \
               [("hip_stream", C.c_void_p), ("kv_cache", C.c_void_p), ("kv_bytes", C.c_size_t)]


_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class wisv_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "lm_head", "final_norm")] + \
               [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER] + \
               [(n, C.c_void_p) for n in ("head_w1", "head_b1", "head_w2", "head_b2")]


class wisv_round_in(C.Structure):
    _fields_ = [("batch", C.c_int32), ("k", C.c_int32), ("stream_ids", C.c_void_p), ("draft_tokens", C.c_void_p),
                ("proto", C.c_void_p), ("hd", C.c_void_p), ("hd_row", C.c_void_p), ("n_hd", C.c_int32),
                ("csi", C.c_void_p), ("tau", C.c_void_p), ("flags", C.c_uint32)]


class wisv_round_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("accepted_len", "correction_token", "p_accept", "target_argmax",
                                          "mismatch_mask", "status")]


class wisv_ss_in(C.Structure):
    _fields_ = [("batch", C.c_int32), ("k", C.c_int32), ("stream_ids", C.c_void_p), ("draft_tokens", C.c_void_p),
                ("draft_probs", C.c_void_p), ("u_accept", C.c_void_p), ("u_sample", C.c_void_p), ("flags", C.c_uint32)]


class wisv_ss_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("accepted_len", "correction_token", "alpha")]


_lib = None


def load_library() -> C.CDLL:
    """Loads libwisv.so; raises if it has not been built (there is nothing to fall back to)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_17701_amd.build` "
                              "(hipcc, gfx950); the verify round has no other implementation")
        lib = C.CDLL(LIB_PATH)
        lib.wisv_ctx_create.argtypes = [C.POINTER(wisv_config), C.POINTER(wisv_weights), C.POINTER(C.c_void_p),
                                        C.c_char_p, C.c_size_t]
        lib.wisv_verify_round.argtypes = [C.c_void_p, C.POINTER(wisv_round_in), C.POINTER(wisv_round_out)]
        lib.wisv_destroy.argtypes = [C.c_void_p]
        lib.wisv_prefill.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]
        lib.wisv_set_state.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        lib.wisv_get_state.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        lib.wisv_kv_import.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]
        lib.wisv_kv_export.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]
        lib.wisv_debug_copy.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t]
        lib.wisv_last_round_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        lib.wisv_profile_enable.argtypes = [C.c_void_p, C.c_int32]
        lib.wisv_profile_collect.argtypes = [C.c_void_p]
        lib.wisv_profile_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                          C.POINTER(C.c_int64)]
        lib.wisv_calibration_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
        lib.wisv_last_error.argtypes = [C.c_void_p]
        lib.wisv_ss_verify_round.argtypes = [C.c_void_p, C.POINTER(wisv_ss_in), C.POINTER(wisv_ss_out)]
        lib.wisv_ss_decide.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 9
        lib.wisv_ss_decide_static.argtypes = lib.wisv_ss_decide.argtypes
        lib.wisv_set_option.argtypes = [C.c_void_p, C.c_int32, C.c_int64]
        lib.wisv_get_option.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int64)]
        lib.wisv_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name != "wisv_last_error":
                getattr(lib, name).restype = C.c_int
        _lib = lib
    return _lib


def ctx_pad(max_ctx: int) -> int:
    """Positions per KV plane: max_ctx rounded up to a multiple of 32 (the V plane is stored in blocks of 32)."""
    return (max_ctx + 31) // 32 * 32


def new_kv_cache(model, max_batch: int, max_ctx: int, device) -> torch.Tensor:
    """A zeroed cache tensor to lend to a Context: [n_layers][max_batch][2][n_kv_heads][ctx_pad * head_dim]."""
    return torch.zeros((model.n_layers, max_batch, 2, model.n_kv_heads, ctx_pad(max_ctx) * model.head_dim),
                       dtype=torch.float32 if model.dtype == "f32" else torch.bfloat16, device=device)


def kv_fill(kv: torch.Tensor, model, layer: int, slot: int, k: torch.Tensor, v: torch.Tensor):
    """Writes k, v ([n_kv_heads, len, head_dim], positions 0..len-1) into a tensor from new_kv_cache, in the
    library's layout: K position-major, V in blocks of 32 positions with the feature index outside."""
    g, n, hd = k.shape
    cp = kv.shape[-1] // hd
    kv[layer, slot, 0].view(g, cp, hd)[:, :n] = k
    nb = (n + 31) // 32
    vp = torch.zeros((g, nb * 32, hd), dtype=kv.dtype, device=kv.device)
    vp[:, :n] = v
    kv[layer, slot, 1].view(g, cp // 32, hd, 32)[:, :nb] = vp.view(g, nb, 32, hd).transpose(2, 3)


def make_config(model, max_batch: int, max_ctx: int, max_k: int, device_id: int = 0, hip_stream: int = 0,
                kv_cache: int = 0, kv_bytes: int = 0) -> wisv_config:
    """`model` carries the fields of wisv_inputs.configs.ModelShape (any object with those attributes)."""
    return wisv_config(model.n_layers, model.d_model, model.n_heads, model.n_kv_heads, model.head_dim, model.d_ff,
                       model.vocab, model.rms_eps, model.rope_theta,
                       WISV_F32 if model.dtype == "f32" else WISV_BF16, model.d_draft, model.d_csi,
                       model.d_head_hidden, model.head_act, max_batch, max_ctx, max_k, device_id,
                       hip_stream or None, kv_cache or None, kv_bytes)


def _host_i32(a) -> np.ndarray:
    if torch.is_tensor(a):
        a = a.detach().cpu().numpy()
    return np.ascontiguousarray(a, dtype=np.int32)


def _host_f32(a) -> np.ndarray:
    if torch.is_tensor(a):
        a = a.detach().cpu().float().numpy()
    return np.ascontiguousarray(a, dtype=np.float32)


class Context:
    """Owner of one wisv_ctx.  Method names follow the C entry points."""

    def __init__(self, model, weights: Dict[str, object], max_batch: int, max_ctx: int, max_k: int,
                 device_id: int = 0, stream: Optional[torch.cuda.Stream] = None,
                 kv_cache: Optional[torch.Tensor] = None):
        self._lib = load_library()
        self._h = C.c_void_p()
        self.model = model
        self.max_batch, self.max_ctx, self.max_k = max_batch, max_ctx, max_k
        self.torch_dtype = torch.float32 if model.dtype == "f32" else torch.bfloat16
        self.device = torch.device("cuda", device_id)
        self._stream = stream
        self._kv = kv_cache
        cfg = self._config(device_id, stream, kv_cache)
        w = wisv_weights()
        keep = []

        def ptr(t: torch.Tensor) -> int:
            if not (torch.is_tensor(t) and t.is_cuda and t.is_contiguous() and t.dtype == self.torch_dtype):
                raise ValueError("weights must be contiguous CUDA tensors of the model's dtype")
            keep.append(t)
            return t.data_ptr()

        for name in ("embed", "lm_head", "final_norm", "head_w1", "head_b1", "head_w2", "head_b2"):
            setattr(w, name, ptr(weights[name]))
        for name in _PER_LAYER:
            arr = (C.c_void_p * model.n_layers)(*[ptr(t) for t in weights[name]])
            keep.append(arr)
            setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
        err = C.create_string_buffer(512)
        torch.cuda.synchronize(self.device)
        rc = self._lib.wisv_ctx_create(C.byref(cfg), C.byref(w), C.byref(self._h), err, 512)
        if rc != WISV_OK:
            self._h = C.c_void_p()
            raise WisvError(rc, err.value.decode(errors="replace"))

    def _config(self, device_id, stream, kv_cache) -> wisv_config:
        return make_config(self.model, self.max_batch, self.max_ctx, self.max_k, device_id,
                           stream.cuda_stream if stream is not None else 0,
                           kv_cache.data_ptr() if kv_cache is not None else 0,
                           kv_cache.numel() * kv_cache.element_size() if kv_cache is not None else 0)

    # ---------------------------------------------------------------- plumbing
    def _check(self, rc: int):
        if rc != WISV_OK:
            raise WisvError(rc, self._lib.wisv_last_error(self._h).decode(errors="replace"))

    def wisv_destroy(self):
        if self._h:
            self._lib.wisv_destroy(self._h)
            self._h = C.c_void_p()

    close = wisv_destroy

    def __del__(self):
        try:
            self.wisv_destroy()
        except Exception:
            pass

    # ---------------------------------------------------------------- the round, host buffers
    def wisv_verify_round(self, stream_ids, draft_tokens, proto, hd, hd_row, csi, tau, k: int, flags: int = 0):
        """Host-buffer round.  hd: tensor [n_hd, d_draft] (any device; model dtype) or None; hd_row: int
        array [batch*k] or None for the identity map.  Returns a dict of numpy arrays."""
        sid = _host_i32(stream_ids)
        b = sid.size
        toks, pr = _host_i32(draft_tokens).reshape(-1), _host_i32(proto)
        csi_a, tau_a = _host_f32(csi).reshape(-1), _host_f32(tau).reshape(-1)
        if toks.size != b * k or pr.size != b or csi_a.size != b * self.model.d_csi or tau_a.size != b:
            raise ValueError("round argument sizes do not match batch and k")
        if hd is None:
            hd_h, n_hd = None, 0
        else:
            hd_h = hd.detach().to("cpu", self.torch_dtype).contiguous().reshape(-1, self.model.d_draft)
            n_hd = hd_h.shape[0]
        row = None if hd_row is None else _host_i32(hd_row).reshape(-1)
        if row is not None and row.size != b * k:
            raise ValueError("hd_row must have batch*k entries")
        out = {
            "accepted_len": np.zeros(b, np.int32), "correction_token": np.zeros(b, np.int32),
            "p_accept": np.zeros(b * k, np.float32), "target_argmax": np.zeros(b * (k + 1), np.int32),
            "mismatch_mask": np.zeros(b, np.uint32), "status": np.zeros(b, np.uint32),
        }
        rin = wisv_round_in(b, k, sid.ctypes.data, toks.ctypes.data, pr.ctypes.data,
                            hd_h.data_ptr() if n_hd else None, row.ctypes.data if row is not None else None,
                            n_hd, csi_a.ctypes.data, tau_a.ctypes.data, flags & ~WISV_FLAG_DEVICE_IO)
        rout = wisv_round_out(*[out[n].ctypes.data for n in ("accepted_len", "correction_token", "p_accept",
                                                             "target_argmax", "mismatch_mask", "status")])
        self._check(self._lib.wisv_verify_round(self._h, C.byref(rin), C.byref(rout)))
        out["p_accept"] = out["p_accept"].reshape(b, k)
        out["target_argmax"] = out["target_argmax"].reshape(b, k + 1)
        return out

    # ---------------------------------------------------------------- the round, device buffers (enqueue only)
    def device_round(self, stream_ids, draft_tokens, proto, hd, hd_row, csi, tau, k: int, flags: int = 0):
        """Uploads one round's arguments once and returns a DeviceRound that re-enqueues it."""
        return DeviceRound(self, stream_ids, draft_tokens, proto, hd, hd_row, csi, tau, k, flags)

    # ---------------------------------------------------------------- speculative sampling
    def wisv_ss_verify_round(self, stream_ids, draft_tokens, draft_probs, u_accept, u_sample, k: int, flags: int = 0):
        """Host-buffer speculative-sampling round.  draft_probs: float array [batch*k, vocab]."""
        sid, toks = _host_i32(stream_ids), _host_i32(draft_tokens).reshape(-1)
        b = sid.size
        q, u, v = _host_f32(draft_probs), _host_f32(u_accept).reshape(-1), _host_f32(u_sample).reshape(-1)
        if toks.size != b * k or q.size != b * k * self.model.vocab or u.size != b * k or v.size != b:
            raise ValueError("round argument sizes do not match batch, k and the vocabulary")
        out = {"accepted_len": np.zeros(b, np.int32), "correction_token": np.zeros(b, np.int32),
               "alpha": np.zeros(b * k, np.float32)}
        sin = wisv_ss_in(b, k, sid.ctypes.data, toks.ctypes.data, q.ctypes.data, u.ctypes.data, v.ctypes.data,
                         flags & ~WISV_FLAG_DEVICE_IO)
        sout = wisv_ss_out(*[out[n].ctypes.data for n in ("accepted_len", "correction_token", "alpha")])
        self._check(self._lib.wisv_ss_verify_round(self._h, C.byref(sin), C.byref(sout)))
        out["alpha"] = out["alpha"].reshape(b, k)
        return out

    def ss_device_round(self, stream_ids, draft_tokens, draft_probs, u_accept, u_sample, k: int, flags: int = 0):
        """Uploads one speculative-sampling round's arguments once; the returned object's run() only enqueues."""
        return SsDeviceRound(self, stream_ids, draft_tokens, draft_probs, u_accept, u_sample, k, flags)

    def wisv_ss_decide(self, logits: torch.Tensor, pending_tokens: torch.Tensor, draft_tokens: torch.Tensor,
                       draft_probs: torch.Tensor, u_accept: torch.Tensor, u_sample: torch.Tensor, k: int, out=None,
                       entry: str = "wisv_ss_decide"):
        """The rule alone on device tensors: logits, draft_probs float [batch*k, vocab]; pending_tokens int32
        [batch]; draft_tokens int32 [batch*k]; u_accept float [batch*k]; u_sample float [batch].
        Returns device tensors (accepted_len, emitted_token, alpha); enqueue only.  `out`: the three output
        tensors, when the caller already holds them (then nothing is allocated here either)."""
        rows, vocab = logits.shape
        b = rows // k
        want = ((logits, torch.float32, rows * vocab), (draft_probs, torch.float32, rows * vocab),
                (pending_tokens, torch.int32, b), (draft_tokens, torch.int32, rows), (u_accept, torch.float32, rows),
                (u_sample, torch.float32, b))
        for t, dt, n in want:
            if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and t.numel() == n):
                raise ValueError("wisv_ss_decide takes contiguous CUDA tensors of the documented types and sizes")
        if out is None:
            out = (torch.zeros(b, dtype=torch.int32, device=logits.device), torch.zeros(b, dtype=torch.int32, device=logits.device),
                   torch.zeros(rows, dtype=torch.float32, device=logits.device))
        alen, tok, alpha = out
        torch.cuda.current_stream(logits.device).synchronize()   # the inputs may come from another stream
        self._check(getattr(self._lib, entry)(self._h, b, k, vocab, logits.data_ptr(), pending_tokens.data_ptr(),
                                              draft_tokens.data_ptr(), draft_probs.data_ptr(), u_accept.data_ptr(),
                                              u_sample.data_ptr(), alen.data_ptr(), tok.data_ptr(), alpha.data_ptr()))
        return alen, tok, alpha.view(b, k)

    def wisv_ss_decide_static(self, *args, **kw):
        """wisv_ss_decide on the library's static scratch (the entry point that allocates nothing)."""
        return self.wisv_ss_decide(*args, entry="wisv_ss_decide_static", **kw)

    # ---------------------------------------------------------------- state
    def wisv_prefill(self, stream_id: int, tokens):
        t = _host_i32(tokens)
        self._check(self._lib.wisv_prefill(self._h, stream_id, t.ctypes.data, t.size))

    def wisv_set_state(self, stream_id: int, kv_len: int, pred_next: int):
        self._check(self._lib.wisv_set_state(self._h, stream_id, kv_len, pred_next))

    def wisv_get_state(self, stream_id: int):
        a, b = C.c_int32(), C.c_int32()
        self._check(self._lib.wisv_get_state(self._h, stream_id, C.byref(a), C.byref(b)))
        return a.value, b.value

    def wisv_kv_import(self, stream_id: int, layer: int, k: torch.Tensor, v: torch.Tensor):
        """k, v: [n_kv_heads, len, head_dim] tensors of the model dtype (moved to the host if needed)."""
        kh = k.detach().to("cpu", self.torch_dtype).contiguous()
        vh = v.detach().to("cpu", self.torch_dtype).contiguous()
        if kh.shape != vh.shape or kh.dim() != 3 or kh.shape[0] != self.model.n_kv_heads or kh.shape[2] != self.model.head_dim:
            raise ValueError("k and v must be [n_kv_heads, len, head_dim]")
        self._check(self._lib.wisv_kv_import(self._h, stream_id, layer, kh.data_ptr(), vh.data_ptr(), kh.shape[1]))

    def wisv_kv_export(self, stream_id: int, layer: int, length: int):
        shape = (self.model.n_kv_heads, length, self.model.head_dim)
        k = torch.empty(shape, dtype=self.torch_dtype)
        v = torch.empty(shape, dtype=self.torch_dtype)
        self._check(self._lib.wisv_kv_export(self._h, stream_id, layer, k.data_ptr(), v.data_ptr(), length))
        return k, v

    # ---------------------------------------------------------------- options
    def wisv_set_option(self, option: int, value: int):
        self._check(self._lib.wisv_set_option(self._h, option, value))

    def wisv_get_option(self, option: int) -> int:
        v = C.c_int64()
        self._check(self._lib.wisv_get_option(self._h, option, C.byref(v)))
        return v.value

    # ---------------------------------------------------------------- diagnostics
    def wisv_debug_copy(self, what: int, rows: int) -> np.ndarray:
        cols = self.model.d_model if what == WISV_DBG_HIDDEN else self.model.vocab
        out = np.empty((rows, cols), np.float32)
        self._check(self._lib.wisv_debug_copy(self._h, what, out.ctypes.data, out.nbytes))
        return out

    def wisv_last_round_ms(self) -> float:
        ms = C.c_float()
        self._check(self._lib.wisv_last_round_ms(self._h, C.byref(ms)))
        return ms.value

    def wisv_calibration_copy(self, dst: torch.Tensor, src: torch.Tensor):
        n = src.numel() * src.element_size()
        self._check(self._lib.wisv_calibration_copy(self._h, dst.data_ptr(), src.data_ptr(), n))

    def wisv_profile_enable(self, on: bool):
        self._check(self._lib.wisv_profile_enable(self._h, 1 if on else 0))

    def wisv_profile_collect(self):
        self._check(self._lib.wisv_profile_collect(self._h))

    def wisv_profile_read(self):
        """{kernel class name: (total ms, launches)} accumulated since profiling was enabled."""
        res, i = {}, 0
        while True:
            name, ms, n = C.c_char_p(), C.c_double(), C.c_int64()
            if self._lib.wisv_profile_read(self._h, i, C.byref(name), C.byref(ms), C.byref(n)) != WISV_OK:
                break
            res[name.value.decode()] = (ms.value, n.value)
            i += 1
        return res


class DeviceRound:
    """One round whose inputs and outputs live in device tensors: run() only enqueues kernels."""

    def __init__(self, ctx: Context, stream_ids, draft_tokens, proto, hd, hd_row, csi, tau, k: int, flags: int):
        dev = ctx.device
        self.ctx, self.k = ctx, k
        i32 = lambda a: torch.from_numpy(_host_i32(a).reshape(-1)).to(dev)
        self.sid, self.toks, self.proto = i32(stream_ids), i32(draft_tokens), i32(proto)
        b = self.batch = self.sid.numel()
        self.csi = torch.from_numpy(_host_f32(csi).reshape(-1)).to(dev)
        self.tau = torch.from_numpy(_host_f32(tau).reshape(-1)).to(dev)
        self.hd = None if hd is None else hd.detach().to(dev, ctx.torch_dtype).contiguous().reshape(-1, ctx.model.d_draft)
        self.n_hd = 0 if self.hd is None else self.hd.shape[0]
        self.row = None if hd_row is None else i32(hd_row)
        if self.toks.numel() != b * k or self.proto.numel() != b or self.tau.numel() != b \
                or self.csi.numel() != b * ctx.model.d_csi or (self.row is not None and self.row.numel() != b * k):
            raise ValueError("round argument sizes do not match batch and k")
        self.out = {
            "accepted_len": torch.zeros(b, dtype=torch.int32, device=dev),
            "correction_token": torch.zeros(b, dtype=torch.int32, device=dev),
            "p_accept": torch.zeros(b * k, dtype=torch.float32, device=dev),
            "target_argmax": torch.zeros(b * (k + 1), dtype=torch.int32, device=dev),
            "mismatch_mask": torch.zeros(b, dtype=torch.int32, device=dev),
            "status": torch.zeros(b, dtype=torch.int32, device=dev),
        }
        self.rin = wisv_round_in(b, k, self.sid.data_ptr(), self.toks.data_ptr(), self.proto.data_ptr(),
                                 self.hd.data_ptr() if self.n_hd else None,
                                 self.row.data_ptr() if self.row is not None else None, self.n_hd,
                                 self.csi.data_ptr(), self.tau.data_ptr(), flags | WISV_FLAG_DEVICE_IO)
        self.rout = wisv_round_out(*[self.out[n].data_ptr() for n in ("accepted_len", "correction_token", "p_accept",
                                                                       "target_argmax", "mismatch_mask", "status")])
        torch.cuda.synchronize(dev)

    def run(self):
        self.ctx._check(self.ctx._lib.wisv_verify_round(self.ctx._h, C.byref(self.rin), C.byref(self.rout)))

    def results(self):
        torch.cuda.synchronize(self.ctx.device)
        b, k = self.batch, self.k
        r = {n: t.cpu().numpy() for n, t in self.out.items()}
        r["p_accept"] = r["p_accept"].reshape(b, k)
        r["target_argmax"] = r["target_argmax"].reshape(b, k + 1)
        r["mismatch_mask"] = r["mismatch_mask"].view(np.uint32)
        r["status"] = r["status"].view(np.uint32)
        return r


class SsDeviceRound:
    """One speculative-sampling round with device-resident arguments: run() only enqueues kernels."""

    def __init__(self, ctx: Context, stream_ids, draft_tokens, draft_probs, u_accept, u_sample, k: int, flags: int):
        dev = ctx.device
        self.ctx, self.k = ctx, k
        i32 = lambda a: torch.from_numpy(_host_i32(a).reshape(-1)).to(dev)
        f32 = lambda a: (a.detach().to(dev, torch.float32).contiguous().reshape(-1) if torch.is_tensor(a)
                         else torch.from_numpy(_host_f32(a).reshape(-1)).to(dev))
        self.sid, self.toks = i32(stream_ids), i32(draft_tokens)
        b = self.batch = self.sid.numel()
        self.q, self.u, self.v = f32(draft_probs), f32(u_accept), f32(u_sample)
        if self.toks.numel() != b * k or self.q.numel() != b * k * ctx.model.vocab or self.u.numel() != b * k \
                or self.v.numel() != b:
            raise ValueError("round argument sizes do not match batch, k and the vocabulary")
        self.out = {"accepted_len": torch.zeros(b, dtype=torch.int32, device=dev),
                    "correction_token": torch.zeros(b, dtype=torch.int32, device=dev),
                    "alpha": torch.zeros(b * k, dtype=torch.float32, device=dev)}
        self.sin = wisv_ss_in(b, k, self.sid.data_ptr(), self.toks.data_ptr(), self.q.data_ptr(), self.u.data_ptr(),
                              self.v.data_ptr(), flags | WISV_FLAG_DEVICE_IO)
        self.sout = wisv_ss_out(*[self.out[n].data_ptr() for n in ("accepted_len", "correction_token", "alpha")])
        torch.cuda.synchronize(dev)

    def run(self):
        self.ctx._check(self.ctx._lib.wisv_ss_verify_round(self.ctx._h, C.byref(self.sin), C.byref(self.sout)))

    def results(self):
        torch.cuda.synchronize(self.ctx.device)
        r = {n: t.cpu().numpy() for n, t in self.out.items()}
        r["alpha"] = r["alpha"].reshape(self.batch, self.k)
        return r


# module-level spellings of the three core entry points
def wisv_ctx_create(model, weights, max_batch: int, max_ctx: int, max_k: int, **kw) -> Context:
    return Context(model, weights, max_batch, max_ctx, max_k, **kw)


def wisv_verify_round(ctx: Context, *args, **kw):
    return ctx.wisv_verify_round(*args, **kw)


def wisv_destroy(ctx: Context):
    ctx.wisv_destroy()
