"""The entry point that allocates nothing (wisv_ss_decide_static) against the one it is a variant of
(wisv_ss_decide): same kernels, scratch in the library's static array instead of the ctx's memory.  Two calls in
a row, the second with a smaller input, must both give exactly what wisv_ss_decide gives on the same inputs
(integers equal, alpha bit-equal), which the speculative-sampling parity tests in turn hold to the oracle."""
import numpy as np
import pytest
import torch

from paper_2604_17701_amd import binding
from wisv_inputs import configs, gen

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(seed, batch, k, vocab, scale):
    rows = batch * k
    logits = gen.target_logits(seed, rows, vocab, scale)
    tokens = gen.randint(seed, "ss_tok", (rows,), vocab).numpy().astype(np.int32)
    top = np.argmax(logits, axis=1).astype(np.int32)
    tokens[1:] = np.where(np.arange(1, rows) % 3 != 0, top[:-1], tokens[1:])       # most drafts hit a likely token
    pending = gen.randint(seed, "ss_pending", (batch,), vocab).numpy().astype(np.int32)
    tokens[::k] = np.where(np.arange(batch) % 5 != 4, pending, tokens[::k])       # most blocks start at their pending token
    q = gen.draft_distributions(seed, rows, vocab, tokens, np.full(rows, 0.05))
    u = gen.unit_uniforms(seed, "ss_u", rows) * np.float32(0.5)
    v = gen.unit_uniforms(seed, "ss_v", batch)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return [dev(x) for x in (logits, pending, tokens, q, u, v)]


def test_static_scratch_entry_point_matches_the_allocating_one_on_two_calls_in_a_row():
    w = configs.get(0)
    wd = gen.make_weights(w.model, w.seed, DEV)
    ctx = binding.Context(w.model, wd, 16, 64, 8)
    # the static entry point is sized by the library's array, not by this ctx: the first case exceeds the ctx's
    # vocabulary (1024) and batch (16) where only the static one may be called, so compare on a second ctx that fits it
    big = configs.scaled(w, vocab=128256, d_model=128, n_heads=2, n_kv_heads=2, d_ff=256)
    wd_big = gen.make_weights(big.model, big.seed, DEV)
    ref_ctx = binding.Context(big.model, wd_big, 24, 64, 8)
    cases = [(24, 8, 128256, 3.5), (5, 3, 997, 4.0)]       # 192 rows x 63 chunks, then 15 rows x 1 ragged chunk
    ins = [_inputs(900 + i, *c) for i, c in enumerate(cases)]
    outs = [(torch.full((b,), -7, dtype=torch.int32, device=DEV), torch.full((b,), -7, dtype=torch.int32, device=DEV),
             torch.full((b * k,), -7.0, dtype=torch.float32, device=DEV)) for b, k, _, _ in cases]
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    got = []
    for (b, k, vocab, _), x, o in zip(cases, ins, outs):   # two calls in a row on one GPU, the second smaller
        got.append(ctx.wisv_ss_decide_static(*x, k, out=o))
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "device memory was allocated or freed during the calls"
    for (b, k, vocab, _), x, g in zip(cases, ins, got):
        want = ref_ctx.wisv_ss_decide(*x, k)
        torch.cuda.synchronize()
        assert torch.equal(g[0], want[0]) and torch.equal(g[1], want[1])
        assert torch.equal(g[2].view(torch.int32), want[2].view(torch.int32))     # alpha bit for bit
        assert int(g[0].min()) >= 0 and int(g[0].max()) <= k
    # sizes beyond the static array are refused, with a message, before anything is enqueued
    z = torch.zeros(1025 * 8, device=DEV)
    zi = torch.zeros(1025, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.WisvError) as e:
        ctx.wisv_ss_decide_static(z.view(1025, 8), zi, zi, z.view(1025, 8), z[:1025], z[:1025], 1)
    assert e.value.code == binding.WISV_EUNSUPPORTED and "1024" in str(e.value)
    ctx.wisv_destroy()
    ref_ctx.wisv_destroy()
