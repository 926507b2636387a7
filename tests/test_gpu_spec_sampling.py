"""GPU parity of the speculative-sampling verifier (Sec. II-A) against oracle/spec_sampling.py.

alpha is compared element by element.  A and the emitted token are integers decided by floating point: they
must be the oracle's wherever the oracle's own margin (|u - alpha|, distance of v * total from the cumulative
weights on either side of the oracle's token) exceeds the stated tolerance; inside the margin the HIP result must
still be a valid outcome of the rule (a neighbouring position / a token whose cumulative interval, widened by
the tolerance, contains v * total, and never a token of zero weight)."""
import numpy as np
import pytest
import torch

from oracle import spec_sampling as ss
from parity import OracleSide, record, check_ss_stream as check_stream, to_host_weights
from paper_2604_17701_amd import binding
from wisv_inputs import configs, gen

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def tiny_ctx():
    w = configs.get(0)
    wd = gen.make_weights(w.model, w.seed, DEV)
    ctx = binding.Context(w.model, wd, 8, 64, 16)
    yield ctx
    ctx.wisv_destroy()


@pytest.fixture(scope="module")
def wide_vocab_ctx():
    # a two-layer target with the 8B vocabulary: the decision kernels at their real row length (63 chunks, ragged tail)
    w = configs.scaled(configs.get(0), vocab=128256, d_model=128, n_heads=2, n_kv_heads=2, d_ff=256)
    wd = gen.make_weights(w.model, w.seed, DEV)
    ctx = binding.Context(w.model, wd, 16, 64, 8)
    yield ctx
    ctx.wisv_destroy()


def _decide_case(ctx, seed, batch, k, vocab, scale, tol=2e-6):
    rows = batch * k
    rng = np.random.default_rng(seed)                     # test-side choices only (which rows get which recipe)
    logits = gen.target_logits(seed, rows, vocab, scale)
    tokens = gen.randint(seed, "ss_tok", (rows,), vocab).numpy().astype(np.int32)
    top = np.argmax(logits, axis=1).astype(np.int32)      # drafts that hit a likely token: rows shifted by one position
    likely = rng.random(rows) < 0.6
    tokens[1:][likely[1:]] = top[:-1][likely[1:]]
    pending = gen.randint(seed, "ss_pending", (batch,), vocab).numpy().astype(np.int32)
    start_ok = rng.random(batch) < 0.85
    tokens[::k][start_ok] = pending[start_ok]             # most blocks start at their pending token
    mass = rng.choice([1e-4, 1e-3, 1e-2, 0.1, 0.6], size=rows)
    q = gen.draft_distributions(seed, rows, vocab, tokens, mass)
    identical = rng.random(rows) < 0.15                   # rows where the drafter equals the target: alpha = 1
    for r in np.nonzero(identical)[0]:
        if r % k:
            q[r] = ss.softmax(logits[r - 1]).astype(np.float32)
    u = gen.unit_uniforms(seed, "ss_u", rows)
    u[rng.random(rows) < 0.4] *= np.float32(0.05)         # more accepted prefixes
    v = gen.unit_uniforms(seed, "ss_v", batch)
    v[:2] = [0.0, np.float32(1.0) - np.float32(2.0 ** -24)][:min(2, batch)]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    alen, tok, alpha = ctx.wisv_ss_decide(dev(logits), dev(pending), dev(tokens), dev(q), dev(u), dev(v), k)
    torch.cuda.synchronize()
    alen, tok, alpha = alen.cpu().numpy(), tok.cpu().numpy(), alpha.cpu().numpy()
    stats = {}
    for b in range(batch):
        s = slice(b * k, (b + 1) * k)
        check_stream(logits[s], int(pending[b]), tokens[s], q[s], u[s], float(v[b]), int(alen[b]), int(tok[b]),
                     alpha[b], tol, stats)
    record(f"ss_decide b={batch} k={k} V={vocab}", {**stats, "A_histogram": np.bincount(alen, minlength=k + 1).tolist()})
    assert stats.get("a_inside_margin", 0) <= max(1, batch // 10)
    if stats.get("tokens", 0) >= 8:
        assert stats["tokens_equal"] >= 0.85 * stats["tokens"]
    return stats


@pytest.mark.parametrize("batch,k,vocab,scale", [(1, 1, 1024, 3.0), (8, 16, 1024, 3.0), (5, 7, 997, 4.0), (8, 3, 5, 1.0),
                                                (3, 4, 1000, 0.5)])
def test_ss_decide_small_vocabularies(tiny_ctx, batch, k, vocab, scale):
    _decide_case(tiny_ctx, 100 + batch * k + vocab, batch, k, vocab, scale)


@pytest.mark.parametrize("batch,k,scale", [(16, 8, 3.5), (4, 5, 0.7), (6, 2, 3.5)])
def test_ss_decide_full_vocabulary(wide_vocab_ctx, batch, k, scale):
    _decide_case(wide_vocab_ctx, 7 + batch, batch, k, 128256, scale)


def test_ss_decide_rejects_bad_arguments(tiny_ctx):
    z = torch.zeros(4 * 2048, device=DEV)
    zi = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.WisvError):                # vocabulary larger than the ctx's
        tiny_ctx.wisv_ss_decide(z.view(4, 2048), zi[:1], zi, z.view(4, 2048), z[:4], z[:1], 4)
    with pytest.raises(binding.WisvError):                # k beyond max_k
        tiny_ctx.wisv_ss_decide(z[:17 * 8].view(17, 8), zi[:1], torch.zeros(17, dtype=torch.int32, device=DEV),
                                z[:17 * 8].view(17, 8), z[:17], z[:1], 17)


def test_ss_round_tiny_target_chain_of_rounds():
    """Three committed rounds on the fp32 target: forward, rule, commit of length and pending token, each round
    checked against the oracle's forward and rule, both sides carrying their own state."""
    w = configs.get(0)
    m, k, batch = w.model, 5, 3
    wd = gen.make_weights(m, w.seed, DEV)
    ctx = binding.Context(m, wd, batch, w.ctx + 3 * k + 1, k)
    side = OracleSide(configs.scaled(w), to_host_weights(wd))
    caches, length, pending = [], [], []
    for b in range(batch):
        toks = gen.context_tokens(w, b)[:40 + 13 * b]
        ctx.wisv_prefill(b, toks)
        c = side.orc.new_cache(w.ctx + 3 * k + 1)
        pending.append(side.orc.prefill(c, toks))
        caches.append(c)
        length.append(len(toks))
        assert ctx.wisv_get_state(b) == (length[b], pending[b])
    stats = {}
    for rnd in range(3):
        seed = 900 + rnd
        tokens = gen.randint(seed, "ss_tok", (batch, k), m.vocab).numpy().astype(np.int32)
        tokens[:, 0] = pending
        if rnd == 1:
            tokens[1, 0] = (pending[1] + 1) % m.vocab       # one block that does not start at its pending token
        olog = [side.orc.forward_block(caches[b], length[b], tokens[b], want_logits=True)["logits"] for b in range(batch)]
        for b in range(batch):                              # drafts 1.. follow the oracle's likely tokens half of the time
            for j in range(1, k):
                if (b + j + rnd) % 2:
                    tokens[b, j] = int(np.argmax(olog[b][j - 1]))
            olog[b] = side.orc.forward_block(caches[b], length[b], tokens[b], want_logits=True)["logits"]
        mass = np.full(batch * k, 0.02)
        q = gen.draft_distributions(seed, batch * k, m.vocab, tokens.reshape(-1), mass).reshape(batch, k, -1)
        u = gen.unit_uniforms(seed, "ss_u", batch * k).reshape(batch, k) * np.float32(0.6)
        v = gen.unit_uniforms(seed, "ss_v", batch)
        g = ctx.wisv_ss_verify_round(np.arange(batch), tokens, q, u, v, k)
        for b in range(batch):
            check_stream(olog[b], pending[b], tokens[b], q[b], u[b], float(v[b]), int(g["accepted_len"][b]),
                         int(g["correction_token"][b]), g["alpha"][b], 2e-5, stats)
            # both sides commit their own result; they agree unless a decision fell inside the margin
            a, tok, _ = ss.verify_block(olog[b], pending[b], tokens[b], q[b], u[b], float(v[b]))
            assert (int(g["accepted_len"][b]), int(g["correction_token"][b])) == (a, tok)
            length[b] += a
            pending[b] = tok
            assert ctx.wisv_get_state(b) == (length[b], pending[b])
    record("ss_round tiny", stats)
    assert stats.get("a_inside_margin", 0) == 0
    ctx.wisv_destroy()


def test_ss_round_no_commit_and_device_io_agree():
    w = configs.get(0)
    m, k, batch = w.model, 4, 2
    wd = gen.make_weights(m, w.seed, DEV)
    ctx = binding.Context(m, wd, batch, 64, k)
    for b in range(batch):
        ctx.wisv_prefill(b, gen.context_tokens(w, b)[:20 + b])
    state = [ctx.wisv_get_state(b) for b in range(batch)]
    tokens = gen.randint(5, "ss_tok", (batch, k), m.vocab).numpy().astype(np.int32)
    tokens[:, 0] = [s[1] for s in state]
    q = gen.draft_distributions(5, batch * k, m.vocab, tokens.reshape(-1), np.full(batch * k, 1e-3))
    u = gen.unit_uniforms(5, "ss_u", batch * k) * np.float32(0.3)
    v = gen.unit_uniforms(5, "ss_v", batch)
    host = ctx.wisv_ss_verify_round(np.arange(batch), tokens, q, u, v, k, binding.WISV_FLAG_NO_COMMIT)
    assert [ctx.wisv_get_state(b) for b in range(batch)] == state
    dr = ctx.ss_device_round(np.arange(batch), tokens, q, u, v, k, binding.WISV_FLAG_NO_COMMIT)
    dr.run()
    dev = dr.results()
    for name in ("accepted_len", "correction_token", "alpha"):
        np.testing.assert_array_equal(host[name], dev[name])
    dr2 = ctx.ss_device_round(np.arange(batch), tokens, q, u, v, k, 0)
    dr2.run()
    dr2.results()
    for b in range(batch):
        assert ctx.wisv_get_state(b) == (state[b][0] + int(host["accepted_len"][b]), int(host["correction_token"][b]))
    with pytest.raises(binding.WisvError):
        ctx.wisv_ss_verify_round(np.arange(batch), tokens, q, np.ones(batch * k, np.float32), v, k)   # u = 1 is outside [0, 1)
    ctx.wisv_destroy()


def test_ss_round_bf16_decoder_many_rows_odd_vocabulary():
    """A small bf16 decoder, 5 streams x 5 positions (25 rows: the many-rows GEMM writes the logits) and a
    vocabulary of 5003 tokens (rows of the logits are not 16-byte aligned: the scalar load path of the rule's
    kernels), checked against the oracle's forward + rule."""
    from dataclasses import replace
    model = replace(configs.LLAMA8B, n_layers=2, d_model=256, n_heads=2, n_kv_heads=1, head_dim=128, d_ff=688, vocab=5003,
                    d_draft=64, d_head_hidden=32)
    w = replace(configs.get(3), model=model, batch=5, ctx=70, k=5, protos=(0,) * 5, kv_source="prefill", index=31)
    m, k, batch = w.model, w.k, w.batch
    wd = gen.make_weights(m, w.seed, DEV)
    ctx = binding.Context(m, wd, batch, w.ctx + k, k)
    side = OracleSide(w, to_host_weights(wd))
    pending, caches, olog = [], [], []
    tokens = gen.randint(41, "ss_tok", (batch, k), m.vocab).numpy().astype(np.int32)
    for b in range(batch):
        toks = gen.context_tokens(w, b)[:w.ctx - 9 * b]
        ctx.wisv_prefill(b, toks)
        c = side.orc.new_cache(w.ctx + k)
        pending.append(side.orc.prefill(c, toks))
        caches.append(c)
        tokens[b, 0] = pending[b]
        for j in range(1, k):                                # drafts follow the oracle's greedy chain except one position
            lg = side.orc.forward_block(c, len(toks), tokens[b, :j], want_logits=True)["logits"]
            if j != 1 + b % (k - 1):
                tokens[b, j] = int(np.argmax(lg[-1]))
        olog.append(side.orc.forward_block(c, len(toks), tokens[b], want_logits=True)["logits"])
    p_tok = np.array([[1.0] + [float(ss.softmax(olog[b][j - 1])[tokens[b, j]]) for j in range(1, k)] for b in range(batch)])
    mass = np.clip(p_tok * (0.5 + 2.5 * gen.uniform01(41, "ss_mass", batch * k).reshape(batch, k)), 1e-9, 0.9)
    q = gen.draft_distributions(41, batch * k, m.vocab, tokens.reshape(-1), mass.reshape(-1)).reshape(batch, k, -1)
    u = gen.unit_uniforms(41, "ss_u", batch * k).reshape(batch, k)
    v = gen.unit_uniforms(41, "ss_v", batch)
    g = ctx.wisv_ss_verify_round(np.arange(batch), tokens, q, u, v, k, binding.WISV_FLAG_NO_COMMIT)
    stats = {}
    for b in range(batch):
        check_stream(olog[b], pending[b], tokens[b], q[b], u[b], float(v[b]), int(g["accepted_len"][b]),
                     int(g["correction_token"][b]), g["alpha"][b], 1e-3, stats)
    stats["A"] = g["accepted_len"].tolist()
    record("ss_round bf16 25 rows", stats)
    assert stats.get("a_inside_margin", 0) <= 1
    ctx.wisv_destroy()
