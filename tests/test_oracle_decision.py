"""Pins of the oracle's decision head, localisation and first-reject rule.

Head: Sec. V-A (eqs. feature_concat, head_forward, mlp_form); FLOP count: Sec. IV-B.
Rule: eq. threshold, Alg. 1 (last block), Sec. III-A step 4; accepted length in [0, K] and
prefix property: Sec. II-A and Sec. IV-B.  The library returns accept probabilities
p_acc = 1 - p_rej and accepts when p_acc >= tau.
"""
import itertools
import math
import os
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import wisv_oracle as wo
from wisv_inputs import configs, gen
from wisv_inputs.configs import ACT_RELU, ACT_SILU, PROTO_FH, PROTO_SH

W0 = configs.get(0)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _head_only_oracle(shape, w1, b1, w2, b2):
    w = gen.make_weights(shape, 1)
    w.update(head_w1=torch.as_tensor(w1, dtype=torch.float32).contiguous(),
             head_b1=torch.as_tensor(b1, dtype=torch.float32).contiguous(),
             head_w2=torch.as_tensor(w2, dtype=torch.float32).contiguous(),
             head_b2=torch.as_tensor([b2], dtype=torch.float32))
    return wo.Oracle(shape, w)


SMALL = replace(configs.TINY, n_layers=1, d_model=8, n_heads=2, n_kv_heads=2, head_dim=4, d_ff=8, vocab=16,
                d_draft=6, d_csi=4, d_head_hidden=5)


def _rand(seed, tag, shape, std=1.0):
    return gen.normal(seed, tag, shape, std, torch.float32).numpy()


def test_head_against_float64_definition_both_activations():
    dj, din = SMALL.d_head_hidden, SMALL.d_in
    w1, b1, w2, b2 = _rand(1, "w1", (dj, din)), _rand(1, "b1", (dj,)), _rand(1, "w2", (dj,)), 0.3
    hd, ht, c = _rand(1, "hd", (6,)), _rand(1, "ht", (8,)), _rand(1, "c", (4,), 5.0)
    z = np.concatenate([hd, ht, c]).astype(np.float64)          # [h^D ; h^T ; c]
    u = w1.astype(np.float64) @ z + b1
    for act, f in ((ACT_SILU, lambda t: t / (1 + np.exp(-t))), (ACT_RELU, lambda t: np.maximum(t, 0))):
        orc = _head_only_oracle(replace(SMALL, head_act=act), w1, b1, w2, b2)
        s, p_rej, p_acc = orc.head(hd, ht, c)
        s_ref = float(w2.astype(np.float64) @ f(u) + np.float32(b2))
        assert abs(s - s_ref) < 1e-5
        assert abs(p_rej - 1 / (1 + math.exp(-s_ref))) < 1e-6
        assert abs(p_acc + p_rej - 1.0) < 1e-6


def test_head_column_order_is_draft_target_csi():
    dj, din = SMALL.d_head_hidden, SMALL.d_in
    hd, ht, c = np.arange(1, 7), np.arange(10, 18), np.arange(100, 104)
    z = np.concatenate([hd, ht, c]).astype(np.float64)
    for col in (0, 5, 6, 13, 14, 17):
        w1 = np.zeros((dj, din), np.float32)
        w1[2, col] = 1.0
        w2 = np.zeros(dj, np.float32)
        w2[2] = 1.0
        orc = _head_only_oracle(replace(SMALL, head_act=ACT_RELU), w1, np.zeros(dj), w2, 0.0)
        s, _, _ = orc.head(hd, ht, c)
        assert s == z[col]


def test_head_zero_weights_and_exact_half():
    dj, din = SMALL.d_head_hidden, SMALL.d_in
    hd, ht, c = _rand(2, "hd", (6,)), _rand(2, "ht", (8,)), _rand(2, "c", (4,))
    orc = _head_only_oracle(SMALL, np.zeros((dj, din)), np.zeros(dj), np.zeros(dj), 0.75)
    s, p_rej, _ = orc.head(hd, ht, c)
    assert s == 0.75 and abs(p_rej - 1 / (1 + math.exp(-0.75))) < 1e-7
    orc = _head_only_oracle(SMALL, _rand(2, "w1", (dj, din)), np.zeros(dj), np.zeros(dj), 0.0)
    s, p_rej, p_acc = orc.head(hd, ht, c)
    assert s == 0.0 and p_rej == 0.5 and p_acc == 0.5
    # p_acc == tau is an acceptance
    a, _, _, _ = wo.decide([3], [4, 9], [1], [p_acc], 0.5)
    assert a == 1


def test_head_csi_only_closed_form():
    dj, din = SMALL.d_head_hidden, SMALL.d_in
    w1 = np.zeros((dj, din), np.float32)
    w1[:, 14:] = _rand(3, "wc", (dj, 4))
    b1, w2 = _rand(3, "b1", (dj,)), _rand(3, "w2", (dj,))
    c = np.array([17.5, 20.0, 117.0, 40.0], np.float32)
    orc = _head_only_oracle(replace(SMALL, head_act=ACT_RELU), w1, b1, w2, -0.1)
    s, _, _ = orc.head(_rand(3, "hd", (6,)), _rand(3, "ht", (8,)), c)
    u = w1[:, 14:].astype(np.float64) @ c + b1
    assert abs(s - (w2.astype(np.float64) @ np.maximum(u, 0) + np.float32(-0.1))) < 1e-4


def test_head_flop_count_matches_paper_formula():
    # tests/golden/head_flops.txt: d_in d_J f_J, evaluated by hand from Sec. IV-B
    with open(os.path.join(GOLDEN, "head_flops.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 2
    for d_in, d_j, f_j in rows:
        assert wo.head_flops(int(d_in), int(d_j)) == int(f_j)
    assert wo.head_flops(configs.LLAMA8B.d_in, configs.LLAMA8B.d_head_hidden) == 6297089


# ------------------------------------------------------------------ decision rule, exhaustively

def _definition(k, match, head_ok, scored, gate_all):
    """Accepted length straight from the text: the longest prefix whose every position is kept.
    A matching token is kept (unless every position is gated); a mismatching one is kept only if
    the head was evaluated there and did not reject."""
    a = 0
    for j in range(k):
        gated = gate_all or not match[j]
        ok = (not gated) or (scored[j] and head_ok[j])
        if not ok:
            break
        a += 1
    return a


@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_rule_exhaustive(k):
    t = np.arange(100, 100 + k + 1, dtype=np.int32)
    tau = 0.5
    for match in itertools.product([0, 1], repeat=k):
        draft = np.where(np.array(match) == 1, t[:k], t[:k] + 1000).astype(np.int32)
        for head_ok in itertools.product([0, 1], repeat=k):
            p = np.where(np.array(head_ok) == 1, 0.8, 0.2).astype(np.float32)
            for scored in (np.ones(k, np.int32), np.array(match[::-1], np.int32)):
                for gate_all in (False, True):
                    a, y, mask, status = wo.decide(draft, t, scored, p, tau, gate_all)
                    want = _definition(k, match, head_ok, scored, gate_all)
                    assert a == want and 0 <= a <= k
                    assert y == t[a]
                    assert mask == sum((1 - m) << j for j, m in enumerate(match))
                    missing = any((gate_all or not match[j]) and not scored[j] for j in range(k))
                    assert status == (1 if missing else 0)
                    if a < k and not gate_all:
                        assert y != draft[a]        # a correction differs from the rejected draft


def test_rule_threshold_extremes_and_monotonicity():
    k = 6
    t = np.arange(k + 1, dtype=np.int32)
    p = np.array([0.0, 1.0, 0.37, 0.5, 0.99, 0.01], np.float32)
    ones = np.ones(k, np.int32)
    for bits in range(1 << k):
        draft = np.array([t[j] if (bits >> j) & 1 else t[j] + 50 for j in range(k)], np.int32)
        first_mismatch = next((j for j in range(k) if not (bits >> j) & 1), k)
        assert wo.decide(draft, t, ones, p, 0.0)[0] == k                    # tau = 0: everything passes
        assert wo.decide(draft, t, ones, p, 1.5)[0] == first_mismatch       # tau > 1: greedy token rule
        assert wo.decide(draft, t, ones, p, 1.5, gate_all=True)[0] == 0     # ... and nothing if all gated
        prev = k
        for tau in (0.0, 0.2, 0.37, 0.5, 0.7, 1.0, 1.01):
            a = wo.decide(draft, t, ones, p, tau)[0]
            assert a <= prev
            prev = a


# ------------------------------------------------------------------ the whole round on config 0

@pytest.fixture(scope="module")
def tiny_round():
    weights = gen.make_weights(W0.model, W0.seed)
    orc = wo.Oracle(W0.model, weights)
    cache = orc.new_cache(W0.ctx + W0.k)
    pred_next = orc.prefill(cache, gen.context_tokens(W0, 0))
    return orc, cache, pred_next


def _chain(orc, cache, pred_next):
    def next_token(prefix):
        if not prefix:
            return pred_next
        return int(orc.forward_block(cache, W0.ctx, prefix)["argmax"][-1])
    return next_token


def _round(orc, cache, pred_next, draft, tau, proto=PROTO_FH, hd_row=None, gate_all=False):
    hd = gen.draft_hidden(W0, 0)
    if hd_row is None:
        hd_row = np.arange(W0.k)
    return orc.verify_round(cache, W0.ctx, pred_next, draft, proto, hd, hd_row, gen.csi_features(W0)[0],
                            tau, gate_all)


def test_round_drafter_equal_to_target_is_fully_accepted(tiny_round):
    orc, cache, pn = tiny_round
    nt = _chain(orc, cache, pn)
    draft = []
    for _ in range(W0.k):
        draft.append(nt(draft))
    for tau in (0.0, 0.5, 1.5):
        r = _round(orc, cache, pn, draft, tau)
        assert r["accepted_len"] == W0.k and r["mismatch_mask"] == 0
        assert r["correction_token"] == r["t"][W0.k]                 # the bonus token
    r = _round(orc, cache, pn, draft, 0.5, proto=PROTO_SH, hd_row=np.full(W0.k, -1))
    assert r["accepted_len"] == W0.k and r["status"] == 0            # nothing requested, nothing missing


def test_round_threshold_extremes(tiny_round):
    orc, cache, pn = tiny_round
    nt = _chain(orc, cache, pn)
    draft = []
    for j in range(W0.k):                                            # every position off the chain
        draft.append((nt(draft) + 1 + j) % W0.model.vocab)
    r0 = _round(orc, cache, pn, draft, 0.0)
    assert r0["accepted_len"] == W0.k and r0["mismatch_mask"] == (1 << W0.k) - 1
    r1 = _round(orc, cache, pn, draft, 1.5)
    assert r1["accepted_len"] == 0 and r1["correction_token"] == pn
    assert np.all((r0["p_accept"] > 0) & (r0["p_accept"] < 1))
    np.testing.assert_allclose(r0["p_accept"] + r0["p_reject"], 1.0, atol=1e-6)
    # mixed block: match, match, mismatch, ... -> tau > 1 stops at the first mismatch
    draft2 = []
    for j in range(W0.k):
        t = nt(draft2)
        draft2.append(t if j < 2 else (t + 3) % W0.model.vocab)
    r2 = _round(orc, cache, pn, draft2, 1.5)
    assert r2["accepted_len"] == 2 and r2["correction_token"] == r2["t"][2] != draft2[2]
    assert _round(orc, cache, pn, draft2, 1.5, gate_all=True)["accepted_len"] == 0


def test_round_selective_upload_equals_full_upload(tiny_round):
    orc, cache, pn = tiny_round
    draft = gen.build_drafts(W0, 0, None)
    hd = gen.draft_hidden(W0, 0)
    csi = gen.csi_features(W0)[0]
    for tau in (0.3, 0.44, 0.45, 0.46, 0.7):
        fh = orc.verify_round(cache, W0.ctx, pn, draft, PROTO_FH, hd, np.arange(W0.k), csi, tau)
        s = [j for j in range(W0.k) if (fh["mismatch_mask"] >> j) & 1]
        rows = np.full(W0.k, -1, np.int32)
        rows[s] = np.arange(len(s))
        sh = orc.verify_round(cache, W0.ctx, pn, draft, PROTO_SH, hd[s], rows, csi, tau)
        assert (sh["accepted_len"], sh["correction_token"]) == (fh["accepted_len"], fh["correction_token"])
        assert sh["status"] == 0
        np.testing.assert_array_equal(sh["p_accept"][s], fh["p_accept"][s])
        if s:                                                        # a withheld hidden state rejects there
            rows[s[0]] = -1
            miss = orc.verify_round(cache, W0.ctx, pn, draft, PROTO_SH, hd[s], rows, csi, 0.0)
            assert miss["accepted_len"] == s[0] and miss["status"] == 1


def test_round_accepted_length_is_monotone_in_tau(tiny_round):
    orc, cache, pn = tiny_round
    draft = gen.build_drafts(W0, 0, None)
    prev = W0.k
    for tau in np.linspace(0.0, 1.1, 23):
        a = _round(orc, cache, pn, draft, float(tau))["accepted_len"]
        assert 0 <= a <= prev
        prev = a
