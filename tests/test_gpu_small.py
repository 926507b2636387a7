"""GPU parity on the sizes the oracle finishes in seconds: config 0 (tiny fp32, real prefill on both
sides) and small bf16 decoders spanning several tiles and ragged tails.  Everything goes through the
C ABI (paper_2604_17701_amd.binding)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from conftest import have_gpu
from parity import (OracleSide, StreamInputs, record, TOL_BF16, TOL_BF16_MANY, TOL_F32, check_invariants, compare_stream, row_rel_err, to_host_weights)
from paper_2604_17701_amd import binding
from wisv_inputs import configs, gen
from wisv_inputs.configs import PROTO_FH, PROTO_SH

pytestmark = pytest.mark.gpu

W0 = configs.get(0)


def _ctx(w, weights_dev, max_batch=None, extra_ctx=0):
    return binding.Context(w.model, weights_dev, max_batch or w.batch, w.ctx + w.k + extra_ctx, w.k)


def _run_workload(w, tol, kv="prefill", taus=None, keep_logits=True, sampled=None, print_tag="", one_term=None):
    """Builds workload w on both sides, runs one round per tau, compares the sampled streams element by
    element and checks the value-free invariants on all streams.  one_term: mask of product classes that take
    one half-precision term in rounds of more than 16 rows (None: the library's default); tol TOL_BF16 is
    widened to TOL_BF16_MANY when such products run (round or prefill chunks of more than 16 rows)."""
    dev = torch.device("cuda:0")
    wd = gen.make_weights(w.model, w.seed, dev)
    side = OracleSide(w, to_host_weights(wd))
    ctx = _ctx(w, wd)
    if one_term is not None:
        ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, one_term)
    if tol is TOL_BF16 and w.m > 16 and ctx.wisv_get_option(binding.WISV_OPT_ONE_TERM_CLASSES) != 0:
        tol = TOL_BF16_MANY
    sampled = list(range(w.batch)) if sampled is None else sampled
    for b in range(w.batch):
        if kv == "prefill":
            ctx.wisv_prefill(b, gen.context_tokens(w, b))
            if b in sampled:
                side.prefill(b)
        else:
            for l in range(w.model.n_layers):
                k, v = gen.synthetic_kv(w, b, l, dev)
                ctx.wisv_kv_import(b, l, k, v)
            ctx.wisv_set_state(b, w.ctx, gen.synthetic_pred_next(w, b))
            if b in sampled:
                side.load_synthetic_kv(b, dev)
    assert sampled == list(range(w.batch)), "small workloads sample every stream"
    if kv == "prefill":
        for b in sampled:
            assert ctx.wisv_get_state(b) == (w.ctx, side.pred_next[b])
    ins = [side.stream_inputs(b) for b in range(w.batch)]
    hd, row_map = gen.pack_hidden(w, [s.hd for s in ins], [s.mismatch for s in ins])
    drafts = np.concatenate([s.draft for s in ins])
    csi = gen.csi_features(w)
    stats = {}
    for tau in (taus or w.taus):
        flags = binding.WISV_FLAG_NO_COMMIT | (binding.WISV_FLAG_KEEP_LOGITS if keep_logits else 0)
        g = ctx.wisv_verify_round(np.arange(w.batch), drafts, w.protos, hd, row_map, csi, np.full(w.batch, tau),
                                  w.k, flags)
        check_invariants(g, drafts, w.k)
        logits = ctx.wisv_debug_copy(binding.WISV_DBG_LOGITS, w.m) if keep_logits else None
        hidden = ctx.wisv_debug_copy(binding.WISV_DBG_HIDDEN, w.m)
        for b in sampled:
            rows = row_map[b * w.k:(b + 1) * w.k]
            o = side.round(b, ins[b], w.protos[b], hd, rows, csi[b], tau, want_logits=keep_logits)
            if keep_logits:
                err = row_rel_err(logits[b * w.k:(b + 1) * w.k], o["logits"])
                stats["logit_rel"] = max(stats.get("logit_rel", 0.0), err)
                assert err <= tol.logit_rel, f"logits rel err {err}"
            herr = row_rel_err(hidden[b * w.k:(b + 1) * w.k], o["h_t"])
            stats["hidden_rel"] = max(stats.get("hidden_rel", 0.0), herr)
            assert herr <= tol.hidden_rel, f"h^T rel err {herr}"
            compare_stream(g, b, o, w.k, tau, tol, stats, logits[b * w.k:(b + 1) * w.k] if keep_logits else None)
    record(print_tag or w.name, stats)
    ctx.wisv_destroy()
    return stats


def test_generator_is_bit_identical_on_cpu_and_gpu():
    a = gen.normal(5, "x", (100003,), 0.02, torch.bfloat16, "cpu")
    b = gen.normal(5, "x", (100003,), 0.02, torch.bfloat16, "cuda:0").cpu()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    c = gen.normal(5, "y", (4099,), 1.0, torch.float32, "cuda:0", start=77).cpu()
    assert torch.equal(c, gen.normal(5, "y", (4099,), 1.0, torch.float32, "cpu", start=77))


def test_config0_tiny_fp32_full_hidden():
    stats = _run_workload(W0, TOL_F32)
    assert stats.get("exact", 0) + stats.get("exempt_tie", 0) + stats.get("exempt_tau", 0) == 1


def test_config0_threshold_extremes_and_chain_draft():
    dev = torch.device("cuda:0")
    w = W0
    wd = gen.make_weights(w.model, w.seed, dev)
    ctx = _ctx(w, wd)
    ctx.wisv_prefill(0, gen.context_tokens(w, 0))
    _, pn = ctx.wisv_get_state(0)
    hd, csi = gen.draft_hidden(w, 0), gen.csi_features(w)
    nc = binding.WISV_FLAG_NO_COMMIT

    def rnd(draft, tau, proto=PROTO_FH, rows=None, flags=nc, hidden=hd):
        return ctx.wisv_verify_round([0], draft, [proto], hidden, rows, csi, [tau], w.k, flags)

    # a drafter that follows the target's greedy chain is accepted in full at any threshold
    chain = []
    for j in range(w.k):
        probe = chain + [0] * (w.k - j)
        chain.append(int(rnd(probe, 0.0)["target_argmax"][0, j]))
    for tau in (0.0, 0.5, 1.5):
        r = rnd(chain, tau)
        assert r["accepted_len"][0] == w.k and r["mismatch_mask"][0] == 0
        assert r["correction_token"][0] == r["target_argmax"][0, w.k]
    r = rnd(chain, 0.5, proto=PROTO_SH, rows=np.full(w.k, -1), hidden=None)
    assert r["accepted_len"][0] == w.k and r["status"][0] == 0
    # every position off the chain: tau = 0 accepts all, tau > 1 leaves only the correction token
    off = []
    for j in range(w.k):
        t = int(rnd(off + [0] * (w.k - j), 0.0)["target_argmax"][0, j])
        off.append((t + 1 + j) % w.model.vocab)
    r0, r1 = rnd(off, 0.0), rnd(off, 1.5)
    assert r0["accepted_len"][0] == w.k and r0["mismatch_mask"][0] == (1 << w.k) - 1
    assert r1["accepted_len"][0] == 0 and r1["correction_token"][0] == pn
    assert rnd(chain, 1.5, flags=nc | binding.WISV_FLAG_GATE_ALL)["accepted_len"][0] == 0
    # selective upload with exactly the mismatch rows reproduces the full upload
    mixed = [chain[0], off[1] if off[1] != chain[1] else (off[1] + 1) % w.model.vocab] + chain[2:]
    full = rnd(mixed, 0.45)
    s = [j for j in range(w.k) if (int(full["mismatch_mask"][0]) >> j) & 1]
    rows = np.full(w.k, -1, np.int32)
    rows[s] = np.arange(len(s))
    sel = rnd(mixed, 0.45, proto=PROTO_SH, rows=rows, hidden=hd[s])
    assert (sel["accepted_len"][0], sel["correction_token"][0]) == (full["accepted_len"][0], full["correction_token"][0])
    np.testing.assert_array_equal(sel["p_accept"][0, s], full["p_accept"][0, s])
    rows[s[0]] = -1
    miss = rnd(mixed, 0.0, proto=PROTO_SH, rows=rows, hidden=hd[s])
    assert miss["accepted_len"][0] == s[0] and miss["status"][0] == binding.WISV_STATUS_MISSING_HIDDEN
    # same inputs, same bits
    again = rnd(mixed, 0.45)
    for key in full:
        assert np.array_equal(full[key], again[key])
    ctx.wisv_destroy()


def test_selective_hidden_protocol_in_two_calls():
    """Alg. 1 as the wire protocol runs it: Verify + Localize (the mask is the request message), then the
    head on exactly the requested rows.  The second call must give what the one-shot round gives, which
    the oracle checks in the parity tests; the first call's accepted length is plain greedy verification."""
    dev = torch.device("cuda:0")
    w = replace(W0, protos=(PROTO_SH,))
    wd = gen.make_weights(w.model, w.seed, dev)
    side = OracleSide(w, to_host_weights(wd))
    ctx = _ctx(w, wd)
    ctx.wisv_prefill(0, gen.context_tokens(w, 0))
    side.prefill(0)
    ins = side.stream_inputs(0)
    hd_all, csi, k = gen.draft_hidden(w, 0), gen.csi_features(w), w.k
    tau, nc = 0.5, binding.WISV_FLAG_NO_COMMIT
    want_s = list(ins.mismatch)
    # one-shot reference (device already knows S) and the oracle
    rows = np.full(k, -1, np.int32)
    rows[want_s] = np.arange(len(want_s))
    one = ctx.wisv_verify_round([0], ins.draft, [PROTO_SH], hd_all[want_s] if want_s else None, rows, csi, [tau], k, nc)
    o = side.round(0, ins, PROTO_SH, hd_all[want_s], rows, csi[0], tau, want_logits=False)
    compare_stream(one, 0, o, k, tau, TOL_F32, {}, None)
    state0 = ctx.wisv_get_state(0)
    # call 1: forward + localisation, nothing uploaded, nothing committed
    first = ctx.wisv_verify_round([0], ins.draft, [PROTO_SH], None, np.full(k, -1), csi, [tau], k, binding.WISV_FLAG_VERIFY_ONLY)
    got_s = [j for j in range(k) if (int(first["mismatch_mask"][0]) >> j) & 1]
    assert got_s == want_s
    np.testing.assert_array_equal(first["target_argmax"], one["target_argmax"])
    assert first["accepted_len"][0] == (want_s[0] if want_s else k)          # greedy verification
    assert ctx.wisv_get_state(0) == state0
    # call 2: the requested rows arrive; no forward; commit
    second = ctx.wisv_verify_round([0], ins.draft, [PROTO_SH], hd_all[got_s] if got_s else None, rows, csi, [tau], k,
                                   binding.WISV_FLAG_DECIDE_ONLY)
    for key in ("accepted_len", "correction_token", "p_accept", "target_argmax", "mismatch_mask", "status"):
        assert np.array_equal(second[key], one[key]), key
    assert ctx.wisv_get_state(0) == (state0[0] + int(one["accepted_len"][0]), int(one["correction_token"][0]))
    # the pending round is consumed; a decide call for another round is refused
    with pytest.raises(binding.WisvError):
        ctx.wisv_verify_round([0], ins.draft, [PROTO_SH], None, np.full(k, -1), csi, [tau], k, binding.WISV_FLAG_DECIDE_ONLY)
    with pytest.raises(binding.WisvError):
        ctx.wisv_verify_round([0], ins.draft, [PROTO_SH], None, np.full(k, -1), csi, [tau], k,
                              binding.WISV_FLAG_DECIDE_ONLY | binding.WISV_FLAG_VERIFY_ONLY)
    ctx.wisv_destroy()


@pytest.mark.parametrize("between", ["prefill", "set_state", "kv_import"])
def test_two_call_protocol_refuses_a_decide_after_the_state_moved(between):
    """Between the two calls of the selective-hidden protocol (Alg. 1: RequestHidden(S) is a network round trip)
    a server may admit another stream.  A prefill runs the forward over the scratch the pending round left
    (h^T, greedy tokens, row map); set_state / kv_import change what the round was verified against.  The
    decide call must then be refused instead of deciding from another forward's values."""
    dev = torch.device("cuda:0")
    w = replace(W0, protos=(PROTO_SH,))
    wd = gen.make_weights(w.model, w.seed, dev)
    ctx = _ctx(w, wd, max_batch=2)
    ctx.wisv_prefill(0, gen.context_tokens(w, 0))
    k, csi = w.k, gen.csi_features(w)
    draft = gen.build_drafts(w, 0, None)
    first = ctx.wisv_verify_round([0], draft, [PROTO_SH], None, np.full(k, -1), csi, [0.5], k, binding.WISV_FLAG_VERIFY_ONLY)
    state0 = ctx.wisv_get_state(0)                      # reading the state does not disturb the pending round
    if between == "prefill":
        ctx.wisv_prefill(1, gen.context_tokens(w, 0)[:9])
    elif between == "set_state":
        ctx.wisv_set_state(1, 0, 3)
    else:
        kk, vv = ctx.wisv_kv_export(0, 0, 4)
        ctx.wisv_kv_import(1, 0, kk, vv)
    s = [j for j in range(k) if (int(first["mismatch_mask"][0]) >> j) & 1]
    rows = np.full(k, -1, np.int32)
    rows[s] = np.arange(len(s))
    hd = gen.draft_hidden(w, 0)
    with pytest.raises(binding.WisvError) as e:
        ctx.wisv_verify_round([0], draft, [PROTO_SH], hd[s] if s else None, rows, csi, [0.5], k, binding.WISV_FLAG_DECIDE_ONLY)
    assert e.value.code == binding.WISV_ESTATE
    assert ctx.wisv_get_state(0) == state0              # nothing was committed
    ctx.wisv_destroy()


def test_commit_advances_the_stream_state():
    dev = torch.device("cuda:0")
    w = W0
    wd = gen.make_weights(w.model, w.seed, dev)
    side = OracleSide(w, to_host_weights(wd))
    ctx = _ctx(w, wd, extra_ctx=8)
    ctx.wisv_prefill(0, gen.context_tokens(w, 0))
    side.prefill(0)
    si = side.stream_inputs(0)
    csi = gen.csi_features(w)
    r = ctx.wisv_verify_round([0], si.draft, [PROTO_FH], si.hd, None, csi, [0.45], w.k, 0)
    a = int(r["accepted_len"][0])
    assert ctx.wisv_get_state(0) == (w.ctx + a, int(r["correction_token"][0]))   # L' = L + A; the correction token
    # the K/V rows the round appended equal the oracle's
    side.orc.forward_block(side.cache[0], w.ctx, si.draft)
    for l in range(w.model.n_layers):
        k, v = ctx.wisv_kv_export(0, l, w.ctx + w.k)
        np.testing.assert_allclose(k.numpy(), side.cache[0][l, 0], atol=2e-5)
        np.testing.assert_allclose(v.numpy(), side.cache[0][l, 1], atol=2e-5)
    ctx.wisv_destroy()


def test_steady_state_rounds_commit_and_roll_back_like_the_oracle():
    """Six committed rounds in a row (Sec. IV-B state recursion L' = L + A): every round forwards the not yet
    cached correction token of the round before as its first "draft" (it matches pred_next by construction)
    followed by K - 1 tokens of a synthetic drafter that follows the target's greedy chain half of the time.
    Rejected rows are dead and must be overwritten; lengths, correction tokens, masks and probabilities of
    every round, the accepted length statistics and the final cache must equal the oracle's."""
    dev = torch.device("cuda:0")
    w = W0
    k, rounds, tau = w.k, 6, 0.5
    wd = gen.make_weights(w.model, w.seed, dev)
    side = OracleSide(w, to_host_weights(wd))
    ctx = _ctx(w, wd, extra_ctx=rounds * k)
    ctx.wisv_prefill(0, gen.context_tokens(w, 0))
    side.prefill(0)
    orc, csi = side.orc, gen.csi_features(w)
    big = orc.new_cache(w.ctx + k + rounds * k)
    big[:, :, :, :w.ctx] = side.cache[0][:, :, :, :w.ctx]
    L, pn = w.ctx, side.pred_next[0]
    rng = np.random.default_rng(11)
    accepted = []
    for r in range(rounds):
        # the drafter: first the pending token, then the greedy chain or a random token
        draft = [int(pn)]
        for j in range(1, k):
            nxt = int(orc.forward_block(big.copy(), L, draft)["argmax"][-1])
            draft.append(nxt if rng.random() < 0.5 else int(rng.integers(0, w.model.vocab)))
        hd = gen.normal(w.seed + r, "steady_hd", (k, w.model.d_draft), 1.0, torch.float32, "cpu")
        o = orc.verify_round(big, L, pn, draft, PROTO_FH, hd.numpy(), np.arange(k), csi[0], tau)
        g = ctx.wisv_verify_round([0], draft, [PROTO_FH], hd, None, csi, [tau], k, 0)
        assert not (int(g["mismatch_mask"][0]) & 1), "the pending token is the target's own"
        compare_stream(g, 0, o, k, tau, TOL_F32, {}, None)
        a, y = int(g["accepted_len"][0]), int(g["correction_token"][0])
        assert a >= 1 and (a, y) == (o["accepted_len"], o["correction_token"])
        L, pn = L + a, y
        assert ctx.wisv_get_state(0) == (L, pn)
        accepted.append(a)
    assert 1.0 <= sum(accepted) / rounds <= k                     # average accepted length per round
    for l in range(w.model.n_layers):
        kk, vv = ctx.wisv_kv_export(0, l, L)
        np.testing.assert_allclose(kk.numpy(), big[l, 0][:, :L], atol=2e-5)
        np.testing.assert_allclose(vv.numpy(), big[l, 1][:, :L], atol=2e-5)
    ctx.wisv_destroy()


def test_round_argument_errors_leave_outputs_untouched():
    dev = torch.device("cuda:0")
    w = W0
    ctx = _ctx(w, gen.make_weights(w.model, w.seed, dev))
    ctx.wisv_set_state(0, w.ctx, 1)
    hd, csi = gen.draft_hidden(w, 0), gen.csi_features(w)
    good = dict(stream_ids=[0], draft_tokens=[1, 2, 3, 4], proto=[0], hd=hd, hd_row=None, csi=csi, tau=[0.5], k=w.k)
    for change, needle in (({"stream_ids": [3]}, "stream_ids"), ({"draft_tokens": [1, 2, 3, w.model.vocab]}, "vocabulary"),
                           ({"proto": [2]}, "proto"), ({"hd_row": [0, 1, 2, 9]}, "hd_row"),
                           ({"hd": hd[:2]}, "identity")):
        with pytest.raises(binding.WisvError) as e:
            ctx.wisv_verify_round(**{**good, **change})
        assert e.value.code == binding.WISV_EINVAL and needle in str(e.value)
    ctx.wisv_set_state(0, w.ctx + w.k, 1)                       # no room for another block
    with pytest.raises(binding.WisvError) as e:
        ctx.wisv_verify_round(**good)
    assert e.value.code == binding.WISV_ESTATE
    ctx.wisv_destroy()


def test_generic_attention_refuses_contexts_its_workgroup_cannot_hold():
    """The generic attention kernel (float targets, unusual head sizes) keeps one score per visible position in LDS.
    Up to a CU's LDS it runs (beyond 64 KiB after opting in); a longer context is refused with WISV_EUNSUPPORTED and
    nothing is decided or committed - it must not be launched with more LDS than exists."""
    dev = torch.device("cuda:0")
    wd = gen.make_weights(W0.model, W0.seed, dev)
    ctx = binding.Context(W0.model, wd, 1, 50000, W0.k)
    k, csi, hd = W0.k, gen.csi_features(W0), gen.draft_hidden(W0, 0)
    draft = gen.build_drafts(W0, 0, None)
    ctx.wisv_set_state(0, 20000, 5)                      # 80 KiB of scores: needs the opt-in, then runs
    g = ctx.wisv_verify_round([0], draft, [PROTO_FH], hd, None, csi, [0.5], k, binding.WISV_FLAG_NO_COMMIT)
    check_invariants(g, draft, k)
    ctx.wisv_set_state(0, 45000, 5)                      # 180 KiB: more than a workgroup can have
    with pytest.raises(binding.WisvError) as e:
        ctx.wisv_verify_round([0], draft, [PROTO_FH], hd, None, csi, [0.5], k, 0)
    assert e.value.code == binding.WISV_EUNSUPPORTED and "LDS" in str(e.value)
    assert ctx.wisv_get_state(0) == (45000, 5)
    with pytest.raises(binding.WisvError) as e:          # prefill takes the same kernels: the state stays where it was
        ctx.wisv_prefill(0, np.arange(8) % W0.model.vocab)
    assert e.value.code == binding.WISV_EUNSUPPORTED
    assert ctx.wisv_get_state(0) == (45000, 5)
    ctx.wisv_destroy()


# ---------------------------------------------------------------- small bf16 decoders (GQA, ragged sizes)

MID = replace(configs.LLAMA8B, n_layers=3, d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, d_ff=1376, vocab=5003,
              d_draft=192, d_head_hidden=96)


@pytest.mark.parametrize("batch,ctx_len,k,protos", [
    (1, 200, 4, (PROTO_FH,)),
    (3, 333, 7, (PROTO_FH, PROTO_SH, PROTO_SH)),
])
def test_small_bf16_decoder_prefill(batch, ctx_len, k, protos):
    w = replace(configs.get(1), model=MID, batch=batch, ctx=ctx_len, k=k, protos=protos, kv_source="prefill",
                name=f"mid_bf16_b{batch}_l{ctx_len}_k{k}", index=7, match_rate=(0.5, 0.5))
    _run_workload(w, TOL_BF16, kv="prefill")


MID128 = replace(MID, head_dim=128, n_heads=4, n_kv_heads=1)     # the MFMA attention kernel needs head_dim 128


@pytest.mark.parametrize("batch,ctx_len,k,kv", [
    (1, 77, 1, "prefill"),      # one query row; a context that ends inside a 32-key step
    (1, 130, 12, "prefill"),    # 48 query rows per KV head: three query tiles
    (1, 95, 16, "synthetic"),   # 64 query rows: four query tiles, the largest block
    (5, 61, 9, "synthetic"),    # 45 rows: the many-rows GEMM with one 64-row tile
    (9, 40, 8, "prefill"),      # 72 rows: a ragged 128-row tile met by 4 x 2 waves
])
def test_small_bf16_decoder_kernel_variants(batch, ctx_len, k, kv):
    """Shapes that reach the kernel variants the five workloads do not: query tile counts 1 to 4, row counts
    on both sides of the GEMM kernels' switch-over points, contexts that are not multiples of 32."""
    protos = tuple(PROTO_FH if b % 2 == 0 else PROTO_SH for b in range(batch))
    w = replace(configs.get(3), model=MID128, batch=batch, ctx=ctx_len, k=k, protos=protos, kv_source=kv,
                name=f"mid128_b{batch}_l{ctx_len}_k{k}_{kv}", index=10 + k, taus=(0.5,))
    _run_workload(w, TOL_BF16, kv=kv)


@pytest.mark.parametrize("one_term", [0, binding.WISV_TERM_ALL, binding.WISV_TERM_QKV | binding.WISV_TERM_O])
def test_many_rows_precision_classes(one_term):
    """72 rows with every product on two bf16 terms (held to the tight tolerance), with all five classes on one
    half-precision term, and with only the two classes the default leaves on two terms."""
    protos = tuple(PROTO_FH if b % 2 == 0 else PROTO_SH for b in range(9))
    w = replace(configs.get(3), model=MID128, batch=9, ctx=40, k=8, protos=protos, kv_source="prefill",
                name=f"mid128_b9_l40_k8_terms{one_term}", index=18, taus=(0.5,))
    _run_workload(w, TOL_BF16, kv="prefill", one_term=one_term)


def test_precision_classes_and_row_counts_switch_on_one_ctx():
    """Beyond 16 rows every activation buffer is written only in the representation its consumer reads, and which
    one that is follows the precision option.  On one ctx, rounds with fresh random drafts alternate between option
    values and between 72 and 16 rows; a product that read a plane left behind by an earlier round would miss the
    oracle, which recomputes every round from that round's drafts."""
    protos = (PROTO_FH,) * 9
    w = replace(configs.get(3), model=MID128, batch=9, ctx=40, k=8, protos=protos, kv_source="prefill",
                name="mid128_b9_l40_k8_switching", index=19, taus=(0.5,))
    dev = torch.device("cuda:0")
    wd = gen.make_weights(w.model, w.seed, dev)
    side = OracleSide(w, to_host_weights(wd))
    ctx = _ctx(w, wd)
    for b in range(w.batch):
        ctx.wisv_prefill(b, gen.context_tokens(w, b))
        side.prefill(b)
    default = ctx.wisv_get_option(binding.WISV_OPT_ONE_TERM_CLASSES)
    csi = gen.csi_features(w)
    hds = [gen.draft_hidden(w, b) for b in range(w.batch)]
    rng = np.random.default_rng(19)
    steps = [(default, 9), (0, 9), (binding.WISV_TERM_ALL, 9), (default, 2), (binding.WISV_TERM_QKV | binding.WISV_TERM_O, 9),
             (default, 9)]
    flags = binding.WISV_FLAG_NO_COMMIT | binding.WISV_FLAG_KEEP_LOGITS
    stats = {}
    for step, (mask, nb) in enumerate(steps):
        ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, mask)
        tol = TOL_BF16 if mask == 0 or nb * w.k <= 16 else TOL_BF16_MANY
        drafts = rng.integers(0, w.model.vocab, (nb, w.k)).astype(np.int32)
        drafts[:, 0] = [side.pred_next[b] for b in range(nb)]          # a block starts at the pending token
        sub = replace(w, batch=nb, protos=protos[:nb])
        hd, row_map = gen.pack_hidden(sub, hds[:nb], [list(range(w.k))] * nb)
        g = ctx.wisv_verify_round(np.arange(nb), drafts.reshape(-1), protos[:nb], hd, row_map, csi[:nb], np.full(nb, 0.5),
                                  w.k, flags)
        check_invariants(g, drafts.reshape(-1), w.k)
        logits = ctx.wisv_debug_copy(binding.WISV_DBG_LOGITS, nb * w.k)
        for b in range(nb):
            si = StreamInputs(drafts[b], hds[b], side.pred_next[b], list(range(w.k)))
            o = side.round(b, si, PROTO_FH, hd, row_map[b * w.k:(b + 1) * w.k], csi[b], 0.5, want_logits=True)
            err = row_rel_err(logits[b * w.k:(b + 1) * w.k], o["logits"])
            stats[f"logit_rel_step{step}"] = max(stats.get(f"logit_rel_step{step}", 0.0), err)
            assert err <= tol.logit_rel, f"step {step} (classes {mask}, {nb} streams): logits rel err {err}"
            compare_stream(g, b, o, w.k, 0.5, tol, stats, logits[b * w.k:(b + 1) * w.k])
    record(w.name, stats)
    ctx.wisv_destroy()


def test_precision_option_is_refused_where_it_cannot_apply():
    dev = torch.device("cuda:0")
    wd = gen.make_weights(W0.model, W0.seed, dev)
    ctx = _ctx(W0, wd)                                   # fp32 target: no half-precision tiles
    assert ctx.wisv_get_option(binding.WISV_OPT_ONE_TERM_CLASSES) == 0
    with pytest.raises(binding.WisvError) as e:
        ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, binding.WISV_TERM_DOWN)
    assert e.value.code == binding.WISV_EUNSUPPORTED
    with pytest.raises(binding.WisvError):
        ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, 64)
    with pytest.raises(binding.WisvError):
        ctx.wisv_set_option(77, 0)
    ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, 0)
    ctx.wisv_destroy()


@pytest.mark.parametrize("batch,k", [(1, 4), (2, 2), (1, 3), (4, 1), (2, 4), (1, 7)])
def test_small_bf16_decoder_folded_norms(batch, k):
    """At most 4 rows and few attention splits: both RMSNorms of a layer are folded into the products around them
    (QKV with the attention prologue; the O projection with gate/up), on a decoder with a power-of-two FFN width;
    the same decoder with 8 and 7 rows takes the norm kernels."""
    model = replace(MID128, d_ff=2048)
    protos = tuple(PROTO_FH if b % 2 == 0 else PROTO_SH for b in range(batch))
    w = replace(configs.get(1), model=model, batch=batch, ctx=150, k=k, protos=protos, kv_source="prefill",
                name=f"mid128_ffn2048_b{batch}_k{k}", index=20 + k, match_rate=(0.5, 0.5))
    _run_workload(w, TOL_BF16, kv="prefill")


def test_small_bf16_decoder_synthetic_kv():
    w = replace(configs.get(2), model=replace(MID, head_dim=128, n_heads=4, n_kv_heads=1), batch=2, ctx=1100, k=8,
                protos=(PROTO_SH, PROTO_FH), name="mid_bf16_synthkv", index=8)
    _run_workload(w, TOL_BF16, kv="synthetic")


def test_repeated_device_round_replays_match_the_eager_round():
    """A device-I/O round repeated with the same buffers is replayed from a captured graph: every replay,
    with other GPU work and synchronisations in between and with the buffers' contents changed in place,
    must give exactly what the eager host-I/O round gives for the same inputs."""
    w = replace(configs.get(2), model=replace(MID, head_dim=128, n_heads=4, n_kv_heads=1), batch=2, ctx=700, k=5,
                protos=(PROTO_SH, PROTO_FH), name="mid_bf16_replay", index=9)
    dev = torch.device("cuda:0")
    wd = gen.make_weights(w.model, w.seed, dev)
    ctx = _ctx(w, wd)
    for b in range(w.batch):
        for l in range(w.model.n_layers):
            k, v = gen.synthetic_kv(w, b, l, dev)
            ctx.wisv_kv_import(b, l, k, v)
        ctx.wisv_set_state(b, w.ctx, gen.synthetic_pred_next(w, b))
    sid = np.arange(w.batch)
    csi = gen.csi_features(w)
    hds = [gen.draft_hidden(w, b) for b in range(w.batch)]
    hd, row_map = gen.pack_hidden(w, hds, [list(range(w.k))] * w.batch)
    nc = binding.WISV_FLAG_NO_COMMIT
    rng = np.random.default_rng(3)
    drafts = rng.integers(0, w.model.vocab, (w.batch, w.k)).astype(np.int32)
    tau = np.full(w.batch, 0.5, np.float32)
    rnd = ctx.device_round(sid, drafts, w.protos, hd, row_map, csi, tau, w.k, nc)
    junk = torch.zeros(1 << 20, device=dev)
    for it in range(6):
        if it >= 2:   # new drafts and thresholds, written into the same device buffers
            drafts = rng.integers(0, w.model.vocab, (w.batch, w.k)).astype(np.int32)
            tau = np.full(w.batch, 0.2 + 0.1 * it, np.float32)
            rnd.toks.copy_(torch.from_numpy(drafts.reshape(-1)))
            rnd.tau.copy_(torch.from_numpy(tau))
        rnd.run()
        got = rnd.results()
        junk.add_(1.0).sum().item()
        want = ctx.wisv_verify_round(sid, drafts, w.protos, hd, row_map, csi, tau, w.k, nc)
        for name in ("accepted_len", "correction_token", "target_argmax", "mismatch_mask", "status", "p_accept"):
            assert np.array_equal(np.asarray(got[name]).reshape(-1), np.asarray(want[name]).reshape(-1)), (it, name)
    ctx.wisv_destroy()


@pytest.mark.parametrize("lengths,k", [
    ((7, 300, 45), 4), ((520, 31, 33, 64), 3), ((1000, 2), 8),          # at most 16 rows
    ((300, 200, 77), 7),                  # 21 rows, two splits, two query tiles
    ((700, 20, 333), 6),                  # 18 rows, three splits
    ((700, 300, 45, 1000, 64), 6),        # 30 rows, four splits
    ((500, 31, 260), 12),                 # 36 rows, four splits, three query tiles (four waves per workgroup)
    ((400, 90), 16),                      # 32 rows, four splits, four query tiles
    ((2000, 130, 64, 999), 5),            # 20 rows, eight splits: RoPE and the append in a kernel of their own
])
def test_mixed_context_lengths_in_one_round(lengths, k):
    """Streams of very different cached lengths in one round on the MFMA attention path: the k-split attention
    (which does RoPE and the append itself at up to 16 rows, and with up to four splits beyond) gives the tail of
    every stream to its last split, leaves splits of short streams empty, and the O projection (or the combine
    kernel) merges what is there.  Every stream is prefilled for real on both sides and compared with the oracle."""
    batch = len(lengths)
    tol = TOL_BF16 if batch * k <= 16 else TOL_BF16_MANY
    base = replace(configs.get(3), model=MID128, batch=batch, ctx=max(lengths), k=k, protos=(PROTO_FH,) * batch,
                   kv_source="prefill", name=f"mid128_mixed_{'_'.join(map(str, lengths))}_k{k}", index=23, taus=(0.5,))
    dev = torch.device("cuda:0")
    wd = gen.make_weights(base.model, base.seed, dev)
    ctx = _ctx(base, wd)
    sides = []
    for b, n in enumerate(lengths):
        wb = replace(base, ctx=n)                      # the oracle side of stream b, with its own context length
        side = OracleSide(wb, to_host_weights(wd))
        toks = gen.context_tokens(base, b)[:n]
        ctx.wisv_prefill(b, toks)
        c = side.orc.new_cache(n + k)
        side.cache[b] = c
        side.pred_next[b] = side.orc.prefill(c, toks)
        assert ctx.wisv_get_state(b) == (n, side.pred_next[b])
        sides.append(side)
    ins = [sides[b].stream_inputs(b) for b in range(batch)]
    hd, row_map = gen.pack_hidden(base, [s.hd for s in ins], [s.mismatch for s in ins])
    drafts = np.concatenate([s.draft for s in ins])
    csi = gen.csi_features(base)
    flags = binding.WISV_FLAG_NO_COMMIT | binding.WISV_FLAG_KEEP_LOGITS
    g = ctx.wisv_verify_round(np.arange(batch), drafts, base.protos, hd, row_map, csi, np.full(batch, 0.5), k, flags)
    check_invariants(g, drafts, k)
    logits = ctx.wisv_debug_copy(binding.WISV_DBG_LOGITS, batch * k)
    stats = {}
    for b in range(batch):
        rows = slice(b * k, (b + 1) * k)
        o = sides[b].round(b, ins[b], PROTO_FH, hd, row_map[rows], csi[b], 0.5, want_logits=True)
        err = row_rel_err(logits[rows], o["logits"])
        stats["logit_rel"] = max(stats.get("logit_rel", 0.0), err)
        assert err <= tol.logit_rel, (b, err)
        compare_stream(g, b, o, k, 0.5, tol, stats, logits[rows])
    record(base.name, stats)
    ctx.wisv_destroy()
