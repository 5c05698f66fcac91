"""Pins for the oracle's decoder, KV cache and self-speculative round.

The paper fixes the token stream (greedy self-speculative output equals the target
model's greedy output: Section 2, greedy special case; Section 5.2 on exact token
matches) and the definitions of u_r and c_r^l (Section 4.2).  The decoder block is
pinned against a composition of torch library routines and closed forms.
"""
import math

import pytest
import torch
import torch.nn.functional as F

from oracle.del_oracle import (Oracle, empirical_tpl, generate_del, generate_fixed,
                               generate_vanilla, rmsnorm, rope_rotate, silu)


# ---------------------------------------------------------------- closed forms
def test_rope_closed_forms():
    torch.manual_seed(0)
    x = torch.randn(5, 3, 64, dtype=torch.float64)
    # position 0 is the identity
    assert torch.equal(rope_rotate(x, torch.zeros(5, dtype=torch.long), 1e4), x)
    pos = torch.tensor([0, 1, 7, 100, 1023])
    y = rope_rotate(x, pos, 1e4)
    # each pair (j, j + hd/2) is rotated: its norm is preserved
    n_in = x[..., :32] ** 2 + x[..., 32:] ** 2
    n_out = y[..., :32] ** 2 + y[..., 32:] ** 2
    assert torch.allclose(n_in, n_out, rtol=1e-12, atol=1e-12)
    # first pair rotates by exactly `pos` radians (frequency theta^0 = 1)
    ang = torch.atan2(y[..., 32], y[..., 0]) - torch.atan2(x[..., 32], x[..., 0])
    want = pos.to(torch.float64)[:, None].expand(5, 3)
    assert torch.allclose(torch.remainder(ang - want + math.pi, 2 * math.pi) - math.pi,
                          torch.zeros(5, 3, dtype=torch.float64), atol=1e-9)
    # scores depend on the position difference only
    q = torch.randn(1, 1, 64, dtype=torch.float64)
    k = torch.randn(1, 1, 64, dtype=torch.float64)
    s1 = (rope_rotate(q, torch.tensor([9]), 5e5) * rope_rotate(k, torch.tensor([4]), 5e5)).sum()
    s2 = (rope_rotate(q, torch.tensor([105]), 5e5) * rope_rotate(k, torch.tensor([100]), 5e5)).sum()
    assert s1.item() == pytest.approx(s2.item(), rel=1e-9)


def test_rope_matches_complex_multiplication():
    torch.manual_seed(1)
    x = torch.randn(4, 2, 32, dtype=torch.float64)
    pos = torch.tensor([3, 4, 50, 51])
    theta = 5e5
    z = torch.complex(x[..., :16], x[..., 16:])
    freqs = theta ** (-torch.arange(16, dtype=torch.float64) * 2 / 32)
    rot = torch.polar(torch.ones(4, 16, dtype=torch.float64), pos[:, None].double() * freqs[None])
    zz = z * rot[:, None, :]
    want = torch.cat([zz.real, zz.imag], dim=-1)
    assert torch.allclose(rope_rotate(x, pos, theta), want, rtol=1e-12, atol=1e-12)


def test_rmsnorm_and_silu_match_library():
    torch.manual_seed(2)
    x = torch.randn(7, 96, dtype=torch.float64)
    g = torch.randn(96, dtype=torch.float64)
    assert torch.allclose(rmsnorm(x, g, 1e-5), F.rms_norm(x, (96,), g, 1e-5), rtol=1e-12, atol=1e-12)
    assert torch.allclose(silu(x), F.silu(x), rtol=1e-12, atol=1e-12)
    # unit gain: rows come out with mean square ~1
    y = rmsnorm(x, torch.ones(96, dtype=torch.float64), 0.0)
    assert torch.allclose((y * y).mean(-1), torch.ones(7, dtype=torch.float64))


# ---------------------------------------------------------------- block vs torch composition
def _block_with_library(o, l, h):
    """One decoder block over a whole sequence from position 0 using torch routines."""
    c = o.cfg
    li = l - 1
    m = h.shape[0]
    W = lambda k: o.w[(li, k)].to(h.dtype)
    a = F.rms_norm(h, (c.d_model,), W("attn_norm").reshape(-1), c.rms_eps)
    q = F.linear(a, W("wq")).view(m, c.n_q_heads, c.head_dim).transpose(0, 1)
    k = F.linear(a, W("wk")).view(m, c.n_kv_heads, c.head_dim).transpose(0, 1)
    v = F.linear(a, W("wv")).view(m, c.n_kv_heads, c.head_dim).transpose(0, 1)
    half = c.head_dim // 2
    freqs = c.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2 / c.head_dim)
    rot = torch.polar(torch.ones(m, half, dtype=torch.float64),
                      torch.arange(m, dtype=torch.float64)[:, None] * freqs[None])

    def rope(t):
        z = torch.complex(t[..., :half].double(), t[..., half:].double()) * rot[None]
        return torch.cat([z.real, z.imag], dim=-1).to(t.dtype)
    q, k = rope(q), rope(k)
    attn = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True,
                                          enable_gqa=True)[0]
    o_ = attn.transpose(0, 1).reshape(m, c.n_q_heads * c.head_dim)
    h1 = h + F.linear(o_, W("wo"))
    b = F.rms_norm(h1, (c.d_model,), W("ffn_norm").reshape(-1), c.rms_eps)
    return h1 + F.linear(F.silu(F.linear(b, W("wg"))) * F.linear(b, W("wu")), W("wd"))


@pytest.mark.parametrize("name", ["tiny", "mini_fp32"])
def test_block_and_head_match_library_composition(name):
    from synthdata import get_config, gen_prompt
    from oracle.del_oracle import load_weights
    cfg = get_config(name)
    w = load_weights(cfg)
    o = Oracle(cfg, w, kv_dtype="fp32")      # fp32-stored KV from fp64 values: rounding ~6e-8
    toks = gen_prompt(cfg, length=19).tolist()
    h = torch.stack([o.embed(t) for t in toks])
    for l in range(1, cfg.n_layers + 1):
        want = _block_with_library(o, l, h)
        got = o.layer(l, h, 0)
        scale = want.abs().max().item()
        assert (got - want).abs().max().item() <= 2e-6 * scale
        h = got
    lg = o.logits(h)
    want = F.linear(F.rms_norm(h, (cfg.d_model,), o.w[(-1, "final_norm")].reshape(-1).double(),
                               cfg.rms_eps), o.w[(-1, "lm_head")].double())
    assert torch.allclose(lg, want, rtol=1e-10, atol=1e-12)
    ids, gaps = o.head(h)
    assert ids == want.float().argmax(-1).tolist()
    assert all(g >= 0 for g in gaps)


def test_single_token_context_attention_returns_value(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w, kv_dtype="fp32")
    h = o.embed(prompt[0])[None, :]
    out = o.layer(1, h, 0)
    a = rmsnorm(h, o.W(0, "attn_norm"), cfg.rms_eps)
    v = (a @ o.W(0, "wv").T).float().double()      # what the cache holds
    h1 = h + v @ o.W(0, "wo").T                    # softmax over one key is 1 (MHA: head j reads kv j)
    b = rmsnorm(h1, o.W(0, "ffn_norm"), cfg.rms_eps)
    want = h1 + (F.silu(b @ o.W(0, "wg").T) * (b @ o.W(0, "wu").T)) @ o.W(0, "wd").T
    assert torch.allclose(out, want, rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- cache reuse (reading R3)
def test_cached_rounds_equal_uncached_forward(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w, kv_dtype="fp32")
    pre = o.prefill(prompt, keep_hidden=True)
    seq = list(prompt) + [pre.first_token]
    for E, g in ((1, 3), (2, 4), (3, 2), (2, 0), (4, 1)):
        T = o.T
        r = o.round(E, g, keep_hidden=True)
        # inputs of the gamma+1 rows: pending token then the drafts
        rows_in = [seq[-1]] + r.draft_ids
        full = o.forward_nocache(seq[:-1] + rows_in)       # [L+1, T+g+1, d]
        got = r.hidden                                     # [L+1, g+1, d]
        want = full[:, T:T + g + 1]
        scale = want.abs().max().item()
        assert (got - want).abs().max().item() <= 1e-5 * scale
        seq.extend(r.out_tokens)
    assert o.T == len(seq) - 1


# ---------------------------------------------------------------- token stream
def test_speculative_tokens_equal_vanilla_tokens(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    van = generate_vanilla(o, prompt, cfg.gen_len)
    assert len(van) == cfg.gen_len
    for E in (1, 2, 3):
        for g in (1, 2, 3, 4):
            toks, recs = generate_fixed(o, prompt, cfg.gen_len, E, g)
            assert toks == van, (E, g)
            for r in recs:
                assert 1 <= len(r.out_tokens) <= r.gamma + 1        # Section 2
                assert len(r.out_tokens) == r.u + 1 == r.n
    toks, pre, recs = generate_del(o, prompt, cfg.gen_len)
    assert toks == van
    assert all(1 <= r.E < cfg.n_layers and 0 <= r.gamma <= cfg.d_max for r in recs)


def test_degenerate_rounds(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    van = generate_vanilla(o, prompt, 24)
    # E = L, gamma = 1: the draft is the full model, always accepted, two tokens a round
    toks, recs = generate_fixed(o, prompt, 24, cfg.n_layers, 1)
    assert toks == van
    assert all(r.u == r.gamma for r in recs)
    # gamma = 0: a round is one vanilla step; eTPL is exactly 1/L (Appendix B.4)
    toks, recs = generate_fixed(o, prompt, 24, 2, 0)
    assert toks == van
    assert all(len(r.out_tokens) == 1 for r in recs)
    assert empirical_tpl(recs, cfg.n_layers) == pytest.approx(1.0 / cfg.n_layers)


# ---------------------------------------------------------------- u and c by brute force
@pytest.mark.parametrize("name", ["tiny", "mini_fp32"])
def test_counts_match_brute_force_per_layer_argmax(name):
    from synthdata import get_config, gen_prompt
    from oracle.del_oracle import load_weights
    cfg = get_config(name)
    w = load_weights(cfg)
    prompt = gen_prompt(cfg).tolist()
    o = Oracle(cfg, w, kv_dtype="fp32")
    pre = o.prefill(prompt)
    L = cfg.n_layers
    # prefill pseudo-round (reading R6): brute force over the last window positions
    full = o.forward_nocache(prompt)
    per_layer = [None] + [o.head(full[l, -pre.window:])[0] for l in range(1, L + 1)]
    assert pre.shadow[1:] == per_layer[1:]
    assert pre.c[1:] == [sum(int(a == b) for a, b in zip(per_layer[l], per_layer[L]))
                         for l in range(1, L + 1)]
    seq = list(prompt) + [pre.first_token]
    E, g = pre.next_E, pre.next_gamma
    for _ in range(12):
        g = max(g, 1)
        r = o.round(E, g)
        rows_in = [seq[-1]] + r.draft_ids
        T = len(seq) - 1
        full = o.forward_nocache(seq[:-1] + rows_in)
        per_layer = [None] + [o.head(full[l, T:])[0] for l in range(1, L + 1)]
        # the draft tokens are layer E's greedy tokens
        assert per_layer[E][:g] == r.draft_ids
        u = next((i for i in range(g) if per_layer[E][i] != per_layer[L][i]), g)
        assert u == r.u
        c = [sum(int(per_layer[l][i] == per_layer[L][i]) for i in range(u + 1))
             for l in range(1, L + 1)]
        assert c == r.c[1:]
        assert r.c[L] == r.n and all(0 <= x <= r.n for x in r.c[1:])
        assert r.out_tokens == per_layer[L][:u + 1]
        seq.extend(r.out_tokens)
        E, g = r.next_E, r.next_gamma


def test_stats_recurrence_and_selection_consistency(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    _, pre, recs = generate_del(o, prompt, 40)
    sc = [float(x) for x in pre.c]
    sn = float(pre.window)
    for r in recs:
        sc = [cfg.omega * a + b for a, b in zip(sc, r.c)]
        sn = cfg.omega * sn + r.n
        for l in range(1, cfg.n_layers + 1):
            assert r.S_c[l] == pytest.approx(sc[l], rel=1e-12)
            assert r.alpha[l] == pytest.approx(sc[l] / sn, rel=1e-12)
        assert r.S_n == pytest.approx(sn, rel=1e-12)
        assert r.alpha[cfg.n_layers] == pytest.approx(1.0)


def test_kv_store_rounding_is_rne_bf16():
    from synthdata import get_config
    cfg = get_config("mini_gqa")
    o = Oracle.__new__(Oracle)
    o.kv_dtype, o.dtype = "bf16", torch.float64
    x = torch.tensor([1.0, 1.00390625, 1.005859375, 1.001953125, -3.1415926, 1e-3], dtype=torch.float64)
    y = o._store_round(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 1.5*2^-8 -> 1 + 2^-7
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.0078125 and y[3] == 1.0
    bits = x.float().view(torch.int32)
    rne = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    assert torch.equal(y.float().view(torch.int32), rne)
