"""A cache-free target forward composed from PyTorch CPU library routines in float64.

Used only to pin the oracle: it recomputes every position from scratch over the whole
sequence (no KV cache, no block structure), with `scaled_dot_product_attention`,
`linear`, `embedding` and `silu` as the library steps.  It shares nothing with the oracle
or the HIP path.
"""
import torch
import torch.nn.functional as F


def _bf(x, on):
    return x.to(torch.bfloat16).double() if on else x


def _modes(round_bf16):
    """(round every matrix-product operand, round k and v as cached)."""
    if round_bf16 == "kv":
        return False, True
    return bool(round_bf16), bool(round_bf16)


def full_forward(weights, shape, tokens, round_bf16=False):
    """tokens: 1-D int tensor of the whole sequence.  Returns (logits [n, V], h_t [n, d]) float64."""
    d64 = lambda t: t.double()
    round_bf16, round_kv = _modes(round_bf16)
    n = tokens.numel()
    H, G, hd = shape.n_heads, shape.n_kv_heads, shape.head_dim
    half = hd // 2

    def norm(x, g):
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + shape.rms_eps) * d64(g)

    dev = tokens.device
    pos = torch.arange(n, dtype=torch.float64, device=dev)
    inv_freq = shape.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64, device=dev) / hd)
    ang = pos[:, None] * inv_freq[None, :]                    # [n, hd/2]
    cos, sin = ang.cos(), ang.sin()

    def rope(t):                                              # t [heads, n, hd]
        t1, t2 = t[..., :half], t[..., half:]
        return torch.cat([t1 * cos - t2 * sin, t2 * cos + t1 * sin], dim=-1)

    x = F.embedding(tokens.long(), d64(weights["embed"]))
    for l in range(shape.n_layers):
        a = _bf(norm(x, weights["attn_norm"][l]), round_bf16)
        q = F.linear(a, d64(weights["wq"][l])).view(n, H, hd).transpose(0, 1)
        k = F.linear(a, d64(weights["wk"][l])).view(n, G, hd).transpose(0, 1)
        v = F.linear(a, d64(weights["wv"][l])).view(n, G, hd).transpose(0, 1)
        q, k, v = _bf(rope(q), round_bf16), _bf(rope(k), round_kv), _bf(v, round_kv)
        k = k.repeat_interleave(H // G, dim=0)
        v = v.repeat_interleave(H // G, dim=0)
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
        o = _bf(o.transpose(0, 1).reshape(n, H * hd), round_bf16)
        x = x + F.linear(o, d64(weights["wo"][l]))
        a2 = _bf(norm(x, weights["ffn_norm"][l]), round_bf16)
        h = F.silu(F.linear(a2, d64(weights["w_gate"][l]))) * F.linear(a2, d64(weights["w_up"][l]))
        x = x + F.linear(_bf(h, round_bf16), d64(weights["w_down"][l]))
    h_t = norm(x, weights["final_norm"])
    logits = F.linear(_bf(h_t, round_bf16), d64(weights["lm_head"]))
    return logits, h_t
