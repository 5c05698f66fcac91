"""Speculative sampling through the C ABI against the oracle (Section 2, "Speculative decoding").

Two levels.  The sampling arithmetic alone (nucleus, draws, acceptance, residual) on logits both sides
receive bit-identically: every decision must be equal.  Whole rounds in lock-step with the oracle on
the reduced shapes: equal except for near-boundary decisions (tests/gpu_harness.py)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle.del_oracle import Oracle, inverse_cdf, load_weights, speculative_accept, tempered_nucleus
from synthdata import gen_prompt, gen_uniforms, get_config

pytestmark = pytest.mark.gpu


def _ctx_for_vocab(vocab, d_max=8):
    """A context whose model is never loaded: only its sampling buffers are used."""
    from paper_2504_05598_amd.binding import DelContext
    cfg = dataclasses.replace(get_config("tiny"), name=f"vocab{vocab}", vocab=vocab, d_max=d_max, n_layers=1,
                              d_model=64, n_q_heads=1, n_kv_heads=1, head_dim=64, d_ffn=64, prompt_len=4, gen_len=4)
    return DelContext(cfg), cfg


def _oracle_decisions(q_logits, p_logits, gamma, T, top_p, un):
    q = [tempered_nucleus(torch.from_numpy(q_logits[i]), T, top_p) for i in range(gamma)]
    p = [tempered_nucleus(torch.from_numpy(p_logits[i]), T, top_p) for i in range(gamma + 1)]
    drafts = [inverse_cdf(q[i], un[i]) for i in range(gamma)]
    u, last, _ = speculative_accept(drafts, q, p, un[gamma:2 * gamma], un[2 * gamma])
    return drafts, u, last


def _logit_rows(rng, rows, vocab, kind):
    if kind == "peaked":
        z = rng.standard_normal((rows, vocab)) * 4.0
    elif kind == "flat":
        z = rng.standard_normal((rows, vocab)) * 0.4
    elif kind == "ties":            # few distinct values: the nucleus cut falls inside a run of equal logits
        z = np.round(rng.standard_normal((rows, vocab)) * 2.0) * 0.5
    else:                           # signs mixed, with exact zeros of both signs
        z = rng.standard_normal((rows, vocab)) * 2.0
        z[:, ::7] = 0.0
        z[:, 3::11] = -0.0
    return np.ascontiguousarray(z, dtype=np.float32)


@pytest.mark.parametrize("vocab", [3000, 3001, 32000, 128256])
def test_sampling_arithmetic_is_exact_on_given_logits(vocab):
    ctx, cfg = _ctx_for_vocab(vocab)
    rng = np.random.default_rng(vocab)
    cases = 0
    for kind in ("peaked", "flat", "ties", "zeros"):
        for (T, top_p) in [(1.0, 1.0), (0.6, 0.95), (0.25, 0.5), (1.3, 0.37), (0.6, 1e-6)]:
            for gamma in (0, 1, 3, 8):
                if vocab == 128256 and gamma == 3:
                    continue
                pl = _logit_rows(rng, gamma + 1, vocab, kind)
                # drafts near the target (so that acceptances and rejections both occur), one row identical
                ql = (pl[:gamma] + _logit_rows(rng, gamma, vocab, "flat") * (0.5 if kind != "ties" else 0.0)).astype(np.float32)
                if kind == "ties" and gamma:
                    ql = np.ascontiguousarray(np.roll(pl[:gamma], 1, axis=1))
                if gamma >= 3:
                    ql[1] = pl[1]
                un = gen_uniforms(cfg, 1000 * cases + gamma, 2 * gamma + 1).tolist()
                want = _oracle_decisions(ql, pl, gamma, T, top_p, un)
                got = ctx.spec_sample(ql, pl, gamma, T, top_p, un)
                assert (got[0], got[1], got[2]) == want, (vocab, kind, T, top_p, gamma, got, want)
                cases += 1
    assert cases >= 60


def test_acceptance_extremes_on_given_logits():
    ctx, cfg = _ctx_for_vocab(5000, d_max=4)
    rng = np.random.default_rng(7)
    pl = _logit_rows(rng, 5, 5000, "peaked")
    # identical rows: everything accepted, whatever the uniform numbers
    un = [0.3, 0.99, 0.0, 0.5, 0.99999994, 0.0, 0.5, 0.99999994, 0.25]
    drafts, u, last = ctx.spec_sample(pl[:4].copy(), pl, 4, 0.7, 0.9, un)
    assert u == 4 and (drafts, u, last) == _oracle_decisions(pl[:4].copy(), pl, 4, 0.7, 0.9, un)
    # disjoint nuclei: the first draft has target probability 0 and is rejected even at r = 0
    ql = pl[:4].copy()
    ql[0] = -pl[0]
    un = [0.5, 0.5, 0.5, 0.5, 0.0, 0.0, 0.0, 0.0, 0.6]
    got = ctx.spec_sample(ql, pl, 4, 0.3, 0.5, un)
    assert got[1] == 0 and got == _oracle_decisions(ql, pl, 4, 0.3, 0.5, un)


def test_argument_checks():
    from paper_2504_05598_amd.binding import DelError
    ctx, cfg = _ctx_for_vocab(3000, d_max=4)
    pl = np.zeros((2, 3000), dtype=np.float32)
    for (T, top_p, un) in [(0.0, 0.9, [0.1, 0.1, 0.1]), (1.0, 0.0, [0.1, 0.1, 0.1]), (1.0, 1.5, [0.1, 0.1, 0.1]),
                           (1.0, 0.9, [0.1, 1.0, 0.1]), (1.0, 0.9, [-0.1, 0.1, 0.1])]:
        with pytest.raises(DelError):
            ctx.spec_sample(pl[:1].copy(), pl, 1, T, top_p, un)
    with pytest.raises(DelError):           # no prefill yet
        ctx.round_sample(1, 1, 1.0, 0.9, [0.1, 0.1, 0.1])
    with pytest.raises(DelError):
        ctx.sample_first(1.0, 0.9, 0.5)


# ---- whole rounds ---------------------------------------------------------------------------

def _setup(name):
    from gpu_harness import gpu_context
    cfg = get_config(name)
    weights = load_weights(cfg)
    prompt = gen_prompt(cfg).tolist()
    ctx, _ = gpu_context(cfg)
    return cfg, Oracle(cfg, weights), ctx, prompt


# temperature 0.6 and top_p 0.95 are the paper's sampling settings (appendix, inference setup); the
# low-temperature cases give peaked distributions.  Tolerances: fp32 shapes differ from the oracle by
# ~1e-6 in the logits, bf16 shapes by ~1e-3.
CASES = [("tiny", 0.6, 0.95, 2e-4, 2e-3), ("mini_fp32", 0.6, 0.95, 2e-4, 2e-3),
         ("mini_gqa", 0.6, 0.95, 5e-3, 3e-2), ("mini_mha", 0.6, 0.95, 5e-3, 3e-2), ("mini_g8", 0.6, 0.95, 5e-3, 3e-2),
         ("mini_gqa", 0.15, 0.9, 5e-3, 3e-2), ("mini_fp32", 0.05, 0.8, 2e-4, 2e-3)]


@pytest.mark.parametrize("name,T,top_p,stol,rtol", CASES)
def test_sampled_rounds_in_lockstep_del_driven(name, T, top_p, stol, rtol):
    from gpu_harness import lockstep_sample, log
    cfg, oracle, ctx, prompt = _setup(name)
    rep = lockstep_sample(cfg, oracle, ctx, prompt, cfg.gen_len, T, top_p, stol, rtol)
    log(f"{name}: {rep.rounds} rounds, {rep.decisions} sampled decisions, {rep.flips} near-boundary, "
        f"{rep.resyncs} resyncs, hidden err {rep.max_hidden_err:.2e}")
    assert len(rep.tokens) >= cfg.gen_len
    assert rep.flips <= max(2, rep.decisions // 5)


@pytest.mark.parametrize("name,T,top_p,stol,rtol", [CASES[0], CASES[2], CASES[5]])
def test_sampled_rounds_in_lockstep_fixed_schedules(name, T, top_p, stol, rtol):
    from gpu_harness import lockstep_sample, log
    cfg, oracle, ctx, prompt = _setup(name)
    L = cfg.n_layers
    for k, sched in enumerate([(1, cfg.d_max), (L // 2, 2), (L, 3), (2, 0)]):
        rep = lockstep_sample(cfg, oracle, ctx, prompt, min(16, cfg.gen_len), T, top_p, stol, rtol, schedule=sched, stream0=100 * (k + 1))
        log(f"{name} {sched}: {rep.rounds} rounds, {rep.decisions} decisions, {rep.flips} near-boundary")
        assert rep.flips <= max(2, rep.decisions // 5)


def test_one_token_nucleus_is_the_greedy_round():
    """top_p -> 0 keeps the arg-max alone: the sampled round must emit what the greedy round emits."""
    from gpu_harness import gpu_context
    cfg = get_config("mini_gqa")
    prompt = gen_prompt(cfg).tolist()
    a, _ = gpu_context(cfg)
    b, _ = gpu_context(cfg)
    fa, E, g = a.prefill(prompt)
    fb, _, _ = b.prefill(prompt)
    assert b.sample_first(0.7, 1e-9, 0.83) == fa == fb
    for k in range(12):
        E, g = 1 + k % cfg.n_layers, k % (cfg.d_max + 1)
        un = gen_uniforms(cfg, 500 + k, 2 * g + 1).tolist()
        assert b.round_sample(E, g, 0.7, 1e-9, un) == a.round(E, g), (k, E, g)
        sa, sb = a.stats(), b.stats()
        assert sa["last_c"] == sb["last_c"] and sa["alpha"] == sb["alpha"]
        assert (sa["next_E"], sa["next_gamma"]) == (sb["next_E"], sb["next_gamma"])
        assert a.state() == b.state()


def test_sampled_generation_is_reproducible():
    from gpu_harness import gpu_context
    cfg = get_config("mini_mha")
    prompt = gen_prompt(cfg).tolist()
    runs = []
    for _ in range(2):
        ctx, _ = gpu_context(cfg)
        _, E, g = ctx.prefill(prompt)
        toks = [ctx.sample_first(0.9, 0.95, 0.123)]
        k = 0
        while len(toks) < cfg.gen_len:
            g = min(g, cfg.gen_len - len(toks) - 1)
            un = gen_uniforms(cfg, 900 + k, 2 * g + 1).tolist()
            toks += ctx.round_sample(E, g, 0.9, 0.95, un)
            st = ctx.stats()
            E, g = st["next_E"], st["next_gamma"]
            k += 1
        runs.append(toks)
    assert runs[0] == runs[1]
    assert len(set(runs[0])) > 8


@pytest.mark.parametrize("name,T,top_p,stol,rtol", [CASES[0], CASES[2], CASES[4], CASES[5]])
def test_sampled_rounds_with_draft_exiting_in_lockstep(name, T, top_p, stol, rtol):
    """Algorithm 1 in full under sampling: E from the statistics, the draft loop stops on tau_E."""
    from gpu_harness import lockstep_sample, log
    cfg, oracle, ctx, prompt = _setup(name)
    rep = lockstep_sample(cfg, oracle, ctx, prompt, cfg.gen_len, T, top_p, stol, rtol, dynamic=True, stream0=7000)
    log(f"{name} draft-exiting: {rep.rounds} rounds, {rep.decisions} sampled decisions, {rep.flips} near-boundary, "
        f"{rep.resyncs} resyncs")
    assert len(rep.tokens) >= cfg.gen_len
    assert rep.flips <= max(2, rep.decisions // 5)


def test_draft_exiting_threshold_extremes_under_sampling():
    from gpu_harness import gpu_context
    cfg = get_config("mini_mha")
    prompt = gen_prompt(cfg).tolist()
    a, _ = gpu_context(cfg)
    b, _ = gpu_context(cfg)
    for ctx in (a, b):
        ctx.prefill(prompt)
        ctx.sample_first(0.8, 0.9, 0.4)
    for k in range(6):
        E, cap = 1 + k % 4, 1 + k % cfg.d_max
        un = gen_uniforms(cfg, 8000 + k, 2 * cap + 1).tolist()
        # tau = 0 never stops: the plain sampled round with the same uniform numbers
        out_b, g, stopped = b.round_sample_dynamic(E, 0.0, cap, 0.8, 0.9, un)
        assert out_b == a.round_sample(E, cap, 0.8, 0.9, un) and g == cap and not stopped
        assert a.state() == b.state()
    # tau above 1 stops before the first draft: one token a round, drawn with the last uniform number
    T0 = b.state()[0]
    out, g, stopped = b.round_sample_dynamic(2, 1.5, 4, 0.8, 0.9, gen_uniforms(cfg, 8100, 9).tolist())
    assert len(out) == 1 and g == 0 and stopped and b.state() == (T0 + 1, out[0])
