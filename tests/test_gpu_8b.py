"""GPU parity at the full sizes of configs 1-4 (Llama-3-8B-shaped bf16 target), in the launch
configuration bench.py times.  The KV cache contents and pred_next are seeded synthetic inputs generated
identically for both sides; the oracle recomputes sampled streams in full (every row, every logit), the
value-free invariants are checked on all streams."""
import time
from dataclasses import replace

import numpy as np
import pytest
import torch

from parity import OracleSide, record, TOL_BF16, TOL_BF16_MANY, TOL_BF16_PREFILL, check_invariants, check_ss_stream as check_stream, compare_stream, row_rel_err, to_host_weights
from paper_2604_17701_amd import binding
from wisv_inputs import configs, gen
from wisv_inputs.configs import PROTO_FH, PROTO_SH

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def target8b():
    t0 = time.time()
    w1 = configs.get(1)
    wd = gen.make_weights(w1.model, w1.seed, DEV)      # the same target serves configs 1-4
    wh = to_host_weights(wd)
    print(f"\n[8b weights] generated + copied to host in {time.time() - t0:.1f}s", flush=True)
    return wd, wh


def _gpu_chain_drafts(ctx, w, pred_next):
    """Drafts of every stream built against the HIP path's own greedy chain (input construction for the
    streams the oracle does not look at): position j needs the target token after drafts 0..j-1."""
    drafts = np.zeros((w.batch, w.k), np.int32)
    plans = [gen.draft_plan(w, b) for b in range(w.batch)]
    csi = gen.csi_features(w)
    for j in range(w.k):
        if j == 0:
            t = np.asarray(pred_next)
        else:
            r = ctx.wisv_verify_round(np.arange(w.batch), drafts, w.protos, None, np.full(w.m, -1), csi,
                                      np.zeros(w.batch), w.k, binding.WISV_FLAG_NO_COMMIT)
            t = r["target_argmax"][:, j]
        for b in range(w.batch):
            keep, alt = plans[b]
            a = int(alt[j])
            drafts[b, j] = int(t[b]) if keep[j] else (a if a != int(t[b]) else (a + 1) % w.model.vocab)
    return drafts


def _run(w, target8b, sampled, tol=None, one_term=None):
    """one_term: mask of product classes that take one half-precision term (None: the library's default)."""
    wd, wh = target8b
    t0 = time.time()
    m = w.model
    max_ctx = w.ctx + w.k
    kv = binding.new_kv_cache(m, w.batch, max_ctx, DEV)
    ctx = binding.Context(m, wd, w.batch, max_ctx, w.k, kv_cache=kv)
    if one_term is not None:
        ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, one_term)
    if tol is None:     # rounds of more than 16 rows run the one-term products unless the mask is empty
        many = w.m > 16 and ctx.wisv_get_option(binding.WISV_OPT_ONE_TERM_CLASSES) != 0
        tol = TOL_BF16_MANY if many else TOL_BF16
    side = OracleSide(w, wh)
    pred_next = []
    for b in range(w.batch):
        for l in range(m.n_layers):
            k, v = gen.synthetic_kv(w, b, l, DEV)
            binding.kv_fill(kv, m, l, b, k, v)
        pn = gen.synthetic_pred_next(w, b)
        pred_next.append(pn)
        ctx.wisv_set_state(b, w.ctx, pn)
    torch.cuda.synchronize()
    print(f"\n[{w.name}] cache filled at {time.time() - t0:.1f}s", flush=True)
    for b in sampled:
        side.load_synthetic_kv(b, DEV)
    drafts = _gpu_chain_drafts(ctx, w, pred_next) if len(sampled) < w.batch else np.zeros((w.batch, w.k), np.int32)
    ins = {b: side.stream_inputs(b) for b in sampled}     # the oracle's chain decides the sampled streams
    for b in sampled:
        drafts[b] = ins[b].draft
    print(f"[{w.name}] drafts built at {time.time() - t0:.1f}s", flush=True)
    hds = [ins[b].hd if b in ins else gen.draft_hidden(w, b) for b in range(w.batch)]
    # mismatch sets for the SH upload: the oracle's for sampled streams, the HIP path's own for the rest
    probe = ctx.wisv_verify_round(np.arange(w.batch), drafts, w.protos, None, np.full(w.m, -1), gen.csi_features(w),
                                  np.zeros(w.batch), w.k, binding.WISV_FLAG_NO_COMMIT)
    mism = [ins[b].mismatch if b in ins else [j for j in range(w.k) if (int(probe["mismatch_mask"][b]) >> j) & 1]
            for b in range(w.batch)]
    hd, row_map = gen.pack_hidden(w, hds, mism)
    csi = gen.csi_features(w)
    stats, prev_a = {}, None
    for tau in w.taus:
        g = ctx.wisv_verify_round(np.arange(w.batch), drafts.reshape(-1), w.protos, hd, row_map, csi,
                                  np.full(w.batch, tau), w.k, binding.WISV_FLAG_NO_COMMIT | binding.WISV_FLAG_KEEP_LOGITS)
        check_invariants(g, drafts, w.k)
        if prev_a is not None:
            assert np.all(g["accepted_len"] <= prev_a), "accepted length must not grow with tau"
        prev_a = g["accepted_len"].copy()
        logits = ctx.wisv_debug_copy(binding.WISV_DBG_LOGITS, w.m)
        hidden = ctx.wisv_debug_copy(binding.WISV_DBG_HIDDEN, w.m)
        for b in sampled:
            rows = slice(b * w.k, (b + 1) * w.k)
            o = side.round(b, ins[b], w.protos[b], hd, row_map[rows], csi[b], tau, want_logits=True)
            err, herr = row_rel_err(logits[rows], o["logits"]), row_rel_err(hidden[rows], o["h_t"])
            stats["logit_rel"] = max(stats.get("logit_rel", 0.0), err)
            stats["hidden_rel"] = max(stats.get("hidden_rel", 0.0), herr)
            assert err <= tol.logit_rel and herr <= tol.hidden_rel, (err, herr)
            compare_stream(g, b, o, w.k, tau, tol, stats, logits[rows])
        stats[f"mean_A@{tau}"] = float(np.mean(g["accepted_len"]))
        print(f"[{w.name}] tau={tau} compared at {time.time() - t0:.1f}s", flush=True)
    record(w.name + ("" if one_term is None else f" one_term={one_term}"), stats)
    ctx.wisv_destroy()
    del kv
    torch.cuda.empty_cache()
    return stats


def test_config1_batch1_ctx512_k4_full_hidden(target8b):
    _run(configs.get(1), target8b, sampled=[0])


def test_config2_batch1_ctx4096_k8_selective_hidden(target8b):
    _run(configs.get(2), target8b, sampled=[0])


def test_config3_batch16_ctx2048_k6_tau_sweep(target8b):
    _run(configs.get(3), target8b, sampled=[0, 5, 11, 15])


def test_config3_with_two_bf16_terms_everywhere(target8b):
    """The many-rows kernels in their two-term form (what a ctx falls back to when a weight does not fit a half),
    held to the tolerance of the memory-bound path."""
    _run(replace(configs.get(3), taus=(0.5,)), target8b, sampled=[0, 11], tol=TOL_BF16, one_term=0)


def test_config4_batch64_ctx8192_k8_mixed_protocols(target8b):
    _run(configs.get(4), target8b, sampled=[0, 5, 38, 63])     # two FH (even) and two SH (odd) streams, first and last included


def test_8b_shape_real_prefill_then_round(target8b):
    """The cache of the headline shape filled by the library's own prefill (the round's kernels in K-row chunks)
    instead of synthetic contents: the oracle prefills the same 64 tokens itself, and the two sides are compared
    cache to cache (three layers, every head and position), by the greedy token after the context, and then on
    a K = 4 round against those caches.  Cached k, v are bf16 values: an entry differs by a bf16 step wherever the two
    float results straddle a rounding boundary, and deep layers inherit the steps of the layers before them, so the
    cache bound is one bf16 step of the largest entry of the plane and the round is held to TOL_BF16_PREFILL."""
    wd, wh = target8b
    w = replace(configs.get(1), name="cfg1_shape_real_prefill_l64", ctx=64, kv_source="prefill")
    m = w.model
    t0 = time.time()
    ctx = binding.Context(m, wd, 1, w.ctx + w.k, w.k)
    toks = gen.context_tokens(w, 0)
    ctx.wisv_prefill(0, toks)
    side = OracleSide(w, wh)
    c = side.orc.new_cache(w.ctx + w.k)
    side.pred_next[0] = side.orc.prefill(c, toks, chunk=32)
    side.cache[0] = c
    print(f"\n[{w.name}] both prefills done at {time.time() - t0:.1f}s", flush=True)
    stats = {}
    assert ctx.wisv_get_state(0) == (w.ctx, side.pred_next[0])
    for layer in (0, m.n_layers // 2, m.n_layers - 1):
        kg, vg = ctx.wisv_kv_export(0, layer, w.ctx)
        for name, got, want in (("k", kg, c[layer, 0, :, :w.ctx]), ("v", vg, c[layer, 1, :, :w.ctx])):
            err = float(np.max(np.abs(got.float().numpy() - want)) / np.max(np.abs(want)))
            stats[f"kv_rel_l{layer}"] = max(stats.get(f"kv_rel_l{layer}", 0.0), err)
            assert err <= 2.0 ** -7, (layer, name, err)        # at most one bf16 step of the largest entry
            frac_equal = float(np.mean(got.float().numpy() == want))
            stats[f"{name}_equal_l{layer}"] = frac_equal
            d = np.abs(got.float().numpy() - want)
            ulp = np.maximum(np.abs(want), 1e-30) * 2.0 ** -7      # at least one bf16 step of the entry itself
            stats[f"{name}_within_1step_l{layer}"] = float(np.mean(d <= ulp))
    assert stats["k_equal_l0"] > 0.99 and stats["v_equal_l0"] > 0.99      # the first layer sees identical inputs
    ins = side.stream_inputs(0)
    hd, csi = ins.hd, gen.csi_features(w)
    g = ctx.wisv_verify_round([0], ins.draft, [PROTO_FH], hd, None, csi, [0.5], w.k,
                              binding.WISV_FLAG_NO_COMMIT | binding.WISV_FLAG_KEEP_LOGITS)
    check_invariants(g, ins.draft, w.k)
    logits, hidden = ctx.wisv_debug_copy(binding.WISV_DBG_LOGITS, w.k), ctx.wisv_debug_copy(binding.WISV_DBG_HIDDEN, w.k)
    o = side.round(0, ins, PROTO_FH, hd, np.arange(w.k), csi[0], 0.5, want_logits=True)
    stats["logit_rel"], stats["hidden_rel"] = row_rel_err(logits, o["logits"]), row_rel_err(hidden, o["h_t"])
    tol = TOL_BF16_PREFILL
    assert stats["logit_rel"] <= tol.logit_rel and stats["hidden_rel"] <= tol.hidden_rel, stats
    compare_stream(g, 0, o, w.k, 0.5, tol, stats, logits)
    record(w.name, stats)
    ctx.wisv_destroy()
    torch.cuda.empty_cache()


def test_config1_shape_speculative_sampling_round(target8b):
    """The stochastic verifier of Sec. II-A at the 8B shape (two streams, L = 512, K = 4): alpha, A and the
    emitted token against the oracle's forward + rule.  The two forwards differ by the bf16 path's rounding
    (logits to about 1e-4 relative), so the margin inside which an integer may differ is 3e-4 (measured alpha error: 7e-5)."""
    from oracle import spec_sampling as ss
    wd, wh = target8b
    w1 = configs.get(1)
    w = configs.Workload("ss_8b_b2_l512_k4", 1, w1.model, batch=2, ctx=512, k=4, protos=(PROTO_FH,) * 2)
    m, k, batch = w.model, w.k, w.batch
    kv = binding.new_kv_cache(m, batch, w.ctx + k, DEV)
    ctx = binding.Context(m, wd, batch, w.ctx + k, k, kv_cache=kv)
    side = OracleSide(w, wh)
    pending = []
    for b in range(batch):
        for l in range(m.n_layers):
            kk, vv = gen.synthetic_kv(w, b, l, DEV)
            binding.kv_fill(kv, m, l, b, kk, vv)
        side.load_synthetic_kv(b, DEV)
        pending.append(gen.synthetic_pred_next(w, b))
        ctx.wisv_set_state(b, w.ctx, pending[b])
    tokens = gen.randint(77, "ss_tok", (batch, k), m.vocab).numpy().astype(np.int32)
    tokens[:, 0] = pending
    olog = []
    for b in range(batch):
        for j in range(1, k):                               # drafts follow the oracle's greedy chain except the last of stream 1
            if not (b == 1 and j == k - 1):
                tokens[b, j] = side.next_token_fn(b)([int(t) for t in tokens[b, :j]])
        olog.append(side.orc.forward_block(side.cache[b], w.ctx, tokens[b], want_logits=True)["logits"])
    # drafter mass on the drafted token around the target's own probability of it, so that alpha lands on both sides of 1
    p_tok = np.array([[1.0] + [float(ss.softmax(olog[b][j - 1])[tokens[b, j]]) for j in range(1, k)] for b in range(batch)])
    mass = np.clip(p_tok * np.array([[1.0, 0.5, 3.0, 1.5], [1.0, 4.0, 0.8, 2.0]]), 0.0, 0.9)
    q = gen.draft_distributions(77, batch * k, m.vocab, tokens.reshape(-1), mass.reshape(-1)).reshape(batch, k, -1)
    v = gen.unit_uniforms(77, "ss_v", batch)
    stats = {}
    for trial, uscale in enumerate((0.2, 0.6, 1.0)):
        u = gen.unit_uniforms(77 + trial, "ss_u", batch * k).reshape(batch, k) * np.float32(uscale)
        g = ctx.wisv_ss_verify_round(np.arange(batch), tokens, q, u, v, k, binding.WISV_FLAG_NO_COMMIT)
        for b in range(batch):
            check_stream(olog[b], pending[b], tokens[b], q[b], u[b], float(v[b]), int(g["accepted_len"][b]),
                         int(g["correction_token"][b]), g["alpha"][b], 3e-4, stats)
        stats[f"A@{uscale}"] = g["accepted_len"].tolist()
    record(w.name, stats)
    assert stats.get("a_inside_margin", 0) <= 1
    ctx.wisv_destroy()
    del kv
    torch.cuda.empty_cache()


@pytest.mark.parametrize("batch,k", [(8, 4), (8, 8), (1, 16), (1, 12), (2, 8), (20, 8), (37, 8)])
def test_8b_shape_mid_row_counts(target8b, batch, k):
    """32 and 64 rows at the 8B shape: the row counts between the weight-streaming kernel (at most 16 rows) and the
    128-row tiles, where gate/up runs in the k-slice layout of the many-rows kernel.  12 and 16 rows: the
    weight-streaming kernel at its largest row counts (no folded norms) with three and four query tiles per KV head
    in the attention kernel, and two streams of eight drafts.  160 and 296 rows: the 128-row tiles with a ragged last
    tile, in the 4 x 2-wave and in the wide workgroup shape."""
    w = configs.Workload(f"mid_8b_b{batch}_l256_k{k}", 1, configs.get(1).model, batch=batch, ctx=256, k=k,
                         protos=tuple(PROTO_FH if b % 2 == 0 else PROTO_SH for b in range(batch)), match_rate=(0.4, 0.9))
    _run(w, target8b, sampled=[min(3, batch - 1)])
