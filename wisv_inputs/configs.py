"""The five synthetic workloads of the WISV edge-side verification round.

Shapes only: no arithmetic of the method lives here.  Both the CPU oracle's
tests and the HIP path's tests/bench read these records, so that the two sides
are driven with byte-identical inputs.

The target is a Llama-style decoder (the paper evaluates Llama-3.x / Qwen2.5
targets, Sec. VI "Experiment Settings"); the decision-head input is
[h^D ; h^T ; c] (Sec. V-A, eq. feature_concat).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple

PROTO_FH = 0  # full-hidden upload      (Sec. III-B, option 1)
PROTO_SH = 1  # selective-hidden upload (Sec. III-B, option 2)

ACT_SILU = 0
ACT_RELU = 1  # the paper's head activation (Sec. V-A, eq. mlp_form)

BASE_SEED = 260417701


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    dtype: str            # "f32" | "bf16"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    d_draft: int = 128
    d_csi: int = 4
    d_head_hidden: int = 64
    head_act: int = ACT_SILU
    weight_std: float = 0.02

    @property
    def d_in(self) -> int:
        return self.d_draft + self.d_model + self.d_csi

    @property
    def d_q(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def layer_params(self) -> int:
        d, f = self.d_model, self.d_ff
        return d * self.d_q + 2 * d * self.d_kv + self.d_q * d + 3 * d * f

    def weight_bytes(self) -> int:
        """Bytes of every matrix one verify round has to read (embedding rows excluded)."""
        e = 4 if self.dtype == "f32" else 2
        return e * (self.n_layers * self.layer_params() + self.vocab * self.d_model)

    def head_bytes(self) -> int:
        e = 4 if self.dtype == "f32" else 2
        return e * (self.d_head_hidden * self.d_in + 2 * self.d_head_hidden + 1)

    def kv_bytes_per_token(self) -> int:
        e = 4 if self.dtype == "f32" else 2
        return e * 2 * self.n_layers * self.d_kv


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    model: ModelShape
    batch: int
    ctx: int              # L: cached tokens per stream at the start of the round
    k: int                # K: drafted tokens per stream
    protos: Tuple[int, ...]            # per stream
    taus: Tuple[float, ...] = (0.5,)   # thresholds the round is evaluated at
    match_rate: Tuple[float, float] = (0.7, 0.7)   # (lo, hi) of U(lo,hi) per stream; equal -> fixed
    uniform_drafts: bool = False       # drafts ~ U(vocab) irrespective of the target
    rayleigh_snr: bool = False         # SNR Rayleigh-faded round a 15 dB mean
    kv_source: str = "synthetic"       # "prefill" | "synthetic"

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.index

    @property
    def m(self) -> int:
        return self.batch * self.k

    def algorithmic_bytes(self) -> int:
        """Bytes one round must move: weights once, the cached K/V once, the head once."""
        ms = self.model
        return (ms.weight_bytes() + ms.head_bytes()
                + self.batch * self.ctx * ms.kv_bytes_per_token())


TINY = ModelShape(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64,
                  d_ff=688, vocab=1024, dtype="f32", rope_theta=10000.0,
                  d_draft=128, d_head_hidden=64)

LLAMA8B = ModelShape(n_layers=32, d_model=4096, n_heads=32, n_kv_heads=8, head_dim=128,
                     d_ff=14336, vocab=128256, dtype="bf16", rope_theta=500000.0,
                     d_draft=2048, d_head_hidden=512)


def _alt(batch):  # even streams FH, odd streams SH
    return tuple(PROTO_FH if (b % 2 == 0) else PROTO_SH for b in range(batch))


CONFIGS = (
    Workload("cfg0_tiny_fp32", 0, TINY, batch=1, ctx=128, k=4, protos=(PROTO_FH,),
             uniform_drafts=True, kv_source="prefill"),
    Workload("cfg1_8b_b1_l512_k4", 1, LLAMA8B, batch=1, ctx=512, k=4, protos=(PROTO_FH,),
             match_rate=(0.7, 0.7)),
    Workload("cfg2_8b_b1_l4096_k8_sh", 2, LLAMA8B, batch=1, ctx=4096, k=8, protos=(PROTO_SH,),
             match_rate=(0.6, 0.6), rayleigh_snr=True),
    Workload("cfg3_8b_b16_l2048_k6", 3, LLAMA8B, batch=16, ctx=2048, k=6,
             protos=(PROTO_FH,) * 16, taus=(0.3, 0.5, 0.7), match_rate=(0.3, 0.9)),
    Workload("cfg4_8b_b64_l8192_k8_mixed", 4, LLAMA8B, batch=64, ctx=8192, k=8,
             protos=_alt(64), match_rate=(0.3, 0.9), rayleigh_snr=True),
)


def get(index: int) -> Workload:
    return CONFIGS[index]


def scaled(w: Workload, **model_overrides) -> Workload:
    """A workload with the same recipe on a different model shape (parity-test mid sizes)."""
    return replace(w, model=replace(w.model, **model_overrides))
