"""Pins of the oracle's target forward (Alg. 1 "Verify"; Sec. III-A step 2).

The cached, block-causal forward is compared with a cache-free float64 forward built from
PyTorch library routines, with closed forms of its building blocks, and with itself under
different block partitions.
"""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import wisv_oracle as wo
from wisv_inputs import configs, gen

from ref_torch import full_forward

W0 = configs.get(0)
GQA = replace(configs.TINY, n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=32,
              d_ff=200, vocab=300, rope_theta=500000.0)


@pytest.fixture(scope="module")
def tiny():
    weights = gen.make_weights(W0.model, W0.seed)
    return weights, wo.Oracle(W0.model, weights)


def _block_vs_full(shape, weights, orc, ctx_len, k, seed):
    toks = gen.randint(seed, "toks", (ctx_len + k,), shape.vocab).to(torch.int32)
    cache = orc.new_cache(ctx_len + k)
    pred_next = orc.prefill(cache, toks[:ctx_len])
    out = orc.forward_block(cache, ctx_len, toks[ctx_len:], want_logits=True)
    ref_logits, ref_h = full_forward(weights, shape, toks)
    assert pred_next == int(ref_logits[ctx_len - 1].argmax())
    np.testing.assert_allclose(out["logits"], ref_logits[ctx_len:].numpy(), rtol=0, atol=1e-5)
    np.testing.assert_allclose(out["h_t"], ref_h[ctx_len:].numpy(), rtol=0, atol=1e-5)
    assert out["argmax"].tolist() == ref_logits[ctx_len:].argmax(-1).tolist()
    top2 = ref_logits[ctx_len:].topk(2, dim=-1).values
    np.testing.assert_allclose(out["gap"], (top2[:, 0] - top2[:, 1]).numpy(), atol=2e-5)


def test_cached_block_equals_cache_free_forward_cfg0(tiny):
    weights, orc = tiny
    _block_vs_full(W0.model, weights, orc, W0.ctx, W0.k, 11)


def test_cached_block_equals_cache_free_forward_gqa():
    # 4 query heads on 2 KV heads, other theta: pins the head -> KV-head grouping
    weights = gen.make_weights(GQA, 77)
    _block_vs_full(GQA, weights, wo.Oracle(GQA, weights), 37, 5, 12)


def test_block_partition_does_not_matter(tiny):
    _, orc = tiny
    toks = gen.randint(5, "toks", (40,), W0.model.vocab).to(torch.int32)
    c1, c2, c3 = (orc.new_cache(40) for _ in range(3))
    a = orc.forward_block(c1, 0, toks, want_logits=True)
    orc.prefill(c2, toks[:33], chunk=7)
    b = orc.forward_block(c2, 33, toks[33:], want_logits=True)
    rows = []
    for i in range(40):
        rows.append(orc.forward_block(c3, i, toks[i:i + 1], want_logits=True)["logits"][0])
    np.testing.assert_allclose(a["logits"][33:], b["logits"], atol=2e-6)
    np.testing.assert_allclose(a["logits"], np.stack(rows), atol=2e-6)
    np.testing.assert_allclose(c1, c2, atol=1e-6)
    np.testing.assert_allclose(c1, c3, atol=1e-6)


def test_forward_rejects_bad_arguments(tiny):
    _, orc = tiny
    cache = orc.new_cache(8)
    with pytest.raises(ValueError):
        orc.forward_block(cache, 6, [1, 2, 3])          # runs past the cache
    with pytest.raises(ValueError):
        orc.forward_block(cache, 0, [W0.model.vocab])   # token out of range


# ------------------------------------------------------------------ building blocks, closed forms

def test_rmsnorm_constant_vector():
    n, c, eps = 64, 3.0, 1e-5
    g = np.linspace(0.5, 2.0, n).astype(np.float32)
    out = wo.rmsnorm(np.full(n, c, np.float32), g, eps)
    np.testing.assert_allclose(out, c / math.sqrt(c * c + eps) * g, rtol=1e-6)


def test_rmsnorm_against_definition():
    x = gen.normal(3, "x", (97,), 2.0, torch.float32).numpy()
    g = gen.normal(3, "g", (97,), 1.0, torch.float32).numpy()
    want = x.astype(np.float64) / np.sqrt((x.astype(np.float64) ** 2).mean() + 1e-5) * g
    np.testing.assert_allclose(wo.rmsnorm(x, g, 1e-5), want, rtol=2e-6, atol=1e-7)


def test_linear_is_x_times_w_transposed():
    x = gen.normal(1, "x", (3, 50), 1.0, torch.float32)
    w = gen.normal(1, "w", (7, 50), 1.0, torch.float32)
    np.testing.assert_allclose(wo.linear(x, w), (x.double() @ w.double().T).numpy(), rtol=1e-6, atol=1e-6)
    # a single one in W picks a single input column: fixes which operand is transposed
    w1 = torch.zeros(7, 50)
    w1[2, 9] = 1.0
    y = wo.linear(x, w1)
    assert np.array_equal(y[:, 2], x[:, 9].numpy()) and np.count_nonzero(y) == 3


def test_rope_closed_forms():
    theta = 10000.0
    v = gen.normal(2, "v", (64,), 1.0, torch.float32).numpy()
    assert np.array_equal(wo.rope(v, 0, theta), v)                      # position 0: identity
    r = wo.rope(v, 17, theta)
    assert abs(np.linalg.norm(r) - np.linalg.norm(v)) < 1e-5            # rotation keeps the norm
    e = np.zeros(4, np.float32)
    e[0] = 1.0                                                          # pair (0, 2), angle = pos
    np.testing.assert_allclose(wo.rope(e, 3, theta), [math.cos(3), 0, math.sin(3), 0], atol=1e-6)
    e = np.zeros(4, np.float32)
    e[1] = 1.0                                                          # pair (1, 3), angle = pos/sqrt(theta)
    a = 3 * theta ** -0.5
    np.testing.assert_allclose(wo.rope(e, 3, theta), [0, math.cos(a), 0, math.sin(a)], atol=1e-6)


def test_rope_inner_product_depends_on_offset_only():
    q = gen.normal(4, "q", (32,), 1.0, torch.float32).numpy()
    k = gen.normal(4, "k", (32,), 1.0, torch.float32).numpy()
    base = float(np.dot(wo.rope(q, 9, 500000.0), wo.rope(k, 4, 500000.0)))
    for shift in (1, 50, 1000):
        other = float(np.dot(wo.rope(q, 9 + shift, 500000.0), wo.rope(k, 4 + shift, 500000.0)))
        assert abs(base - other) < 2e-4


def test_attention_closed_forms():
    hd, n = 16, 9
    k = gen.normal(6, "k", (n, hd), 1.0, torch.float32).numpy()
    v = gen.normal(6, "v", (n, hd), 1.0, torch.float32).numpy()
    np.testing.assert_allclose(wo.attend(np.zeros(hd), k, v), v.mean(0), atol=1e-6)      # q = 0: plain mean
    q = gen.normal(6, "q", (hd,), 1.0, torch.float32).numpy()
    np.testing.assert_allclose(wo.attend(q, k[:1], v[:1]), v[0], atol=1e-7)              # one visible key
    s = (k[:2].astype(np.float64) @ q) / math.sqrt(hd)                                   # two keys: logistic weight
    p0 = 1.0 / (1.0 + math.exp(s[1] - s[0]))
    np.testing.assert_allclose(wo.attend(q, k[:2], v[:2]), p0 * v[0] + (1 - p0) * v[1], atol=1e-6)
    want = torch.softmax(torch.from_numpy(k).double() @ torch.from_numpy(q).double() / math.sqrt(hd), 0)
    np.testing.assert_allclose(wo.attend(q, k, v), (want[:, None] * torch.from_numpy(v).double()).sum(0).numpy(),
                               atol=1e-6)


def test_argmax_planted_and_ties():
    z = gen.normal(8, "z", (1000,), 1.0, torch.float32).numpy()
    z[613] = 9.0
    z[77] = 8.5
    idx, gap = wo.argmax(z)
    assert idx == 613 and abs(gap - 0.5) < 1e-6
    z[900] = 9.0
    z[20] = 9.0                       # exact three-way tie: lowest index wins, lead is zero
    idx, gap = wo.argmax(z)
    assert idx == 20 and gap == 0.0
    assert wo.argmax(np.array([-3.0, -1.0, -2.0], np.float32)) == (1, 1.0)


# ------------------------------------------------------------------ bf16 storage and rounding points

def test_round_bf16_matches_library_conversion():
    vals = gen.normal(9, "r", (20000,), 3.0, torch.float32)
    extra = torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -3.0e38, 1e-40, 65504.0,
                          0.1, 256.5, float("inf")])
    for x in torch.cat([vals, extra]).tolist():
        assert wo.round_bf16(x) == float(torch.tensor(x).to(torch.bfloat16).float())
    # ties go to the even mantissa
    assert wo.round_bf16(1.00390625) == 1.0 and wo.round_bf16(1.01171875) == 1.015625


def _bf16_shape():
    return replace(GQA, dtype="bf16")


def test_bf16_storage_is_exact_widening():
    shape = _bf16_shape()
    wb = gen.make_weights(shape, 31)
    up = lambda t: t.float()
    wf = {k: ([up(x) for x in v] if isinstance(v, list) else up(v)) for k, v in wb.items()}
    toks = gen.randint(31, "t", (20,), shape.vocab).to(torch.int32)
    ob = wo.Oracle(shape, wb, round_bf16=False)
    of = wo.Oracle(replace(shape, dtype="f32"), wf)
    a = ob.forward_block(ob.new_cache(20), 0, toks, want_logits=True)
    b = of.forward_block(of.new_cache(20), 0, toks, want_logits=True)
    assert np.array_equal(a["logits"], b["logits"])


def test_bf16_rounding_points_against_library_forward():
    shape = _bf16_shape()
    wb = gen.make_weights(shape, 32)
    toks = gen.randint(32, "t", (24,), shape.vocab).to(torch.int32)
    orc_r = wo.Oracle(shape, wb, round_bf16=True)
    orc_n = wo.Oracle(shape, wb, round_bf16=False)
    zr = orc_r.forward_block(orc_r.new_cache(24), 0, toks, want_logits=True)["logits"].astype(np.float64)
    zn = orc_n.forward_block(orc_n.new_cache(24), 0, toks, want_logits=True)["logits"].astype(np.float64)
    ref_r, _ = full_forward(wb, shape, toks, round_bf16=True)
    ref_n, _ = full_forward(wb, shape, toks, round_bf16=False)
    np.testing.assert_allclose(zn, ref_n.numpy(), atol=1e-5)
    # same rounding points: what is left are rare one-ulp flips, far below the effect of rounding itself
    d_same = np.sqrt(np.mean((zr - ref_r.numpy()) ** 2))
    d_round = np.sqrt(np.mean((zr - zn) ** 2))
    assert d_round > 0 and d_same < 0.2 * d_round, (d_same, d_round)
    # the cache holds bf16-representable numbers in this mode
    c = orc_r.new_cache(24)
    orc_r.forward_block(c, 0, toks)
    ct = torch.from_numpy(c)
    assert torch.equal(ct.to(torch.bfloat16).float(), ct)


def test_bf16_cache_only_mode_rounds_exactly_the_cached_k_and_v():
    shape = _bf16_shape()
    wb = gen.make_weights(shape, 33)
    toks = gen.randint(33, "t", (12,), shape.vocab).to(torch.int32)
    orc_kv = wo.Oracle(shape, wb)                       # default for bf16 weights: "kv"
    orc_n = wo.Oracle(shape, wb, round_bf16="none")
    ck, cn = orc_kv.new_cache(12), orc_n.new_cache(12)
    # one token: nothing cached is read back yet, so the logits agree and the cache is the rounded float cache
    a = orc_kv.forward_block(ck, 0, toks[:1], want_logits=True)
    b = orc_n.forward_block(cn, 0, toks[:1], want_logits=True)
    layer0 = (slice(0, 1), slice(None), slice(None), slice(0, 1))
    assert np.array_equal(ck[layer0], torch.from_numpy(cn[layer0]).to(torch.bfloat16).float().numpy())
    assert not np.array_equal(ck[layer0], cn[layer0])
    # a single position attends only to itself with weight 1: its output is the cached (rounded) v, so the two
    # modes differ from the first layer on, by about one bf16 rounding of v
    rel = np.abs(a["logits"] - b["logits"]).max() / np.abs(b["logits"]).max()
    assert 0 < rel < 3e-2
    # against the library forward with the same two rounding points
    ref, _ = full_forward(wb, shape, toks, round_bf16="kv")
    z = orc_kv.forward_block(orc_kv.new_cache(12), 0, toks, want_logits=True)["logits"]
    zn = orc_n.forward_block(orc_n.new_cache(12), 0, toks, want_logits=True)["logits"]
    d_same = np.sqrt(np.mean((z - ref.numpy()) ** 2))
    d_round = np.sqrt(np.mean((z.astype(np.float64) - zn) ** 2))
    assert d_round > 0 and d_same < 0.2 * d_round, (d_same, d_round)
