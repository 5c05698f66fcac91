"""Pins of the oracle's speculative-sampling arithmetic (Section 2, "Speculative decoding") against
things other than itself: a hand-worked example, brute force over subsets, library soft-max, the
exactness of the output distribution, and the greedy round as the low-temperature limit."""
import itertools
import math

import pytest
import torch

from oracle.del_oracle import (Oracle, inverse_cdf, residual_distribution, speculative_accept,
                               tempered_nucleus)
from conftest import read_golden


def _vals(gold, key):
    return [float(x) for x in next(row for row in gold if row[0] == key)[1:]]


def test_hand_worked_acceptance_and_residual():
    g = read_golden("spec_sampling_worked.txt")
    p = torch.tensor(_vals(g, "p"), dtype=torch.float64)
    q = torch.tensor(_vals(g, "q"), dtype=torch.float64)
    acc = _vals(g, "accept")
    # acceptance probability of token x = measure of the r for which the rule accepts
    N = 2000
    for x in range(3):
        hits = sum(speculative_accept([x], [q], [p, p], [(k + 0.5) / N], 0.0)[0] == 1 for k in range(N))
        assert hits / N == pytest.approx(acc[x], abs=1.0 / N)
    assert residual_distribution(p, q).tolist() == pytest.approx(_vals(g, "residual"), abs=1e-15)
    reject = sum(float(q[x]) * (1 - acc[x]) for x in range(3))
    assert reject == pytest.approx(_vals(g, "reject_mass")[0], abs=1e-15)


def test_hand_worked_nucleus():
    g = read_golden("spec_sampling_worked.txt")
    probs = torch.tensor(_vals(g, "nucleus_in"), dtype=torch.float64)
    out = tempered_nucleus(torch.log(probs), 1.0, _vals(g, "nucleus_top_p")[0])
    assert out.tolist() == pytest.approx(_vals(g, "nucleus_out"), abs=1e-7)


def test_top_p_one_is_the_library_softmax_of_scaled_logits():
    z = torch.randn(1000, generator=torch.Generator().manual_seed(1)) * 3
    for T in (1.0, 0.6, 2.5):
        ref = torch.nn.functional.softmax(z.to(torch.float64) / T, dim=-1)
        assert torch.allclose(tempered_nucleus(z, T, 1.0), ref, rtol=1e-12, atol=0)


@pytest.mark.parametrize("seed", range(6))
def test_nucleus_is_the_smallest_heaviest_set_reaching_top_p(seed):
    gen = torch.Generator().manual_seed(100 + seed)
    V = 7
    z = torch.randn(V, generator=gen) * 1.5
    T = 0.8
    top_p = [0.3, 0.5, 0.7, 0.9, 0.95, 0.999][seed]
    p = torch.softmax(z.to(torch.float64) / T, dim=0)
    best = None
    for k in range(1, V + 1):
        sets = [(float(sum(p[i] for i in S)), S) for S in itertools.combinations(range(V), k)]
        ok = [s for s in sets if s[0] >= top_p]
        if ok:
            best = max(ok)[1]
            break
    out = tempered_nucleus(z, T, top_p)
    assert set(torch.nonzero(out).flatten().tolist()) == set(best)
    assert float(out.sum()) == pytest.approx(1.0, abs=1e-14)
    kept = list(best)
    assert torch.allclose(out[kept], p[kept] / p[kept].sum(), rtol=1e-13)


def test_equal_logits_at_the_cut_keep_the_lower_id():
    z = torch.tensor([0.0, 1.0, 1.0, 1.0, -5.0])
    out = tempered_nucleus(z, 1.0, 0.5)       # each of ids 1..3 has mass ~0.30: two are needed
    assert torch.nonzero(out).flatten().tolist() == [1, 2]


def test_low_temperature_and_tiny_top_p_reduce_to_the_argmax():
    z = torch.randn(500, generator=torch.Generator().manual_seed(3))
    a = int(torch.argmax(z))
    assert int(torch.argmax(tempered_nucleus(z, 1e-4, 1.0))) == a
    assert float(tempered_nucleus(z, 1e-4, 1.0)[a]) == pytest.approx(1.0, abs=1e-12)
    one = tempered_nucleus(z, 1.0, 1e-6)
    assert torch.nonzero(one).flatten().tolist() == [a] and float(one[a]) == 1.0


def test_inverse_cdf_gives_every_token_its_probability():
    p = torch.tensor([0.0, 0.25, 0.0, 0.125, 0.5, 0.125, 0.0], dtype=torch.float64)
    N = 4096
    counts = [0] * len(p)
    for k in range(N):
        counts[inverse_cdf(p, (k + 0.5) / N)] += 1
    assert [c / N for c in counts] == pytest.approx(p.tolist(), abs=1.0 / N)
    assert inverse_cdf(p, 0.0) == 1 and inverse_cdf(p, 0.25) == 3 and inverse_cdf(p, 0.999999) == 5
    # unnormalised masses are allowed: r scales with the total
    assert inverse_cdf(p * 7.0, 0.3) == inverse_cdf(p, 0.3)


@pytest.mark.parametrize("seed", range(3))
def test_one_drafted_token_reproduces_the_target_distribution(seed):
    """The rule's defining property (Section 2 cites its proof): drafting from q, accepting with
    min(1, p/q) and resampling from the residual yields exactly p.  Integrated over a lattice of the
    three uniform numbers; a swapped ratio, a missing clamp or a residual from q fails it."""
    gen = torch.Generator().manual_seed(200 + seed)
    V = 4
    p = torch.softmax(torch.randn(V, generator=gen, dtype=torch.float64) * 1.5, dim=0)
    q = torch.softmax(torch.randn(V, generator=gen, dtype=torch.float64) * 1.5, dim=0)
    bonus = torch.softmax(torch.randn(V, generator=gen, dtype=torch.float64), dim=0)
    N1, N2, N3 = 64, 24, 24
    first = torch.zeros(V, dtype=torch.float64)
    second = torch.zeros(V, dtype=torch.float64)
    for a in range(N1):
        x = inverse_cdf(q, (a + 0.5) / N1)
        for b in range(N2):
            for c in range(N3):
                u, tok, _ = speculative_accept([x], [q], [p, bonus], [(b + 0.5) / N2], (c + 0.5) / N3)
                if u == 1:
                    first[x] += 1
                    second[tok] += 1
                else:
                    first[tok] += 1
    total = N1 * N2 * N3
    assert (first / total).tolist() == pytest.approx(p.tolist(), abs=0.03)
    n_acc = float(second.sum())
    assert (second / n_acc).tolist() == pytest.approx(bonus.tolist(), abs=0.03)
    # closed form of the same statement from the rule's pieces
    acc = torch.minimum(torch.ones_like(p), p / q)
    closed = q * acc + (1 - float((q * acc).sum())) * residual_distribution(p, q)
    assert torch.allclose(closed, p, atol=1e-14)


def test_identical_distributions_accept_everything():
    gen = torch.Generator().manual_seed(9)
    ps = [torch.softmax(torch.randn(50, generator=gen, dtype=torch.float64), dim=0) for _ in range(5)]
    drafts = [inverse_cdf(ps[i], 0.37 + 0.1 * i) for i in range(4)]
    u, tok, dist = speculative_accept(drafts, ps[:4], ps, [0.999999, 0.5, 0.0, 0.73], 0.42)
    assert u == 4 and tok == inverse_cdf(ps[4], 0.42) and dist is ps[4]


def test_first_rejection_discards_the_rest():
    p = torch.tensor([0.5, 0.5, 0.0], dtype=torch.float64)
    q = torch.tensor([0.0, 0.5, 0.5], dtype=torch.float64)
    # token 2 has p = 0: rejected for every r; the residual is token 0 alone
    u, tok, _ = speculative_accept([1, 2, 1], [q, q, q], [p, p, p, p], [0.3, 0.0, 0.0], 0.9)
    assert (u, tok) == (1, 0)


# ---- the whole round ----------------------------------------------------------------------

def test_low_temperature_round_is_the_greedy_round(tiny_model):
    cfg, weights, prompt = tiny_model
    a, b = Oracle(cfg, weights), Oracle(cfg, weights)
    pa, pb = a.prefill(prompt), b.prefill(prompt)
    tok, _ = b.sample_first(1e-5, 1.0, 0.77)
    assert tok == pa.first_token
    gen = torch.Generator().manual_seed(5)
    for (E, g) in [(2, 3), (1, 4), (3, 2), (4, 2), (2, 0)]:
        ra = a.round(E, g)
        rb = b.round_sample(E, g, 1e-5, 1.0, torch.rand(2 * g + 1, generator=gen).tolist())
        assert rb.out_tokens == ra.out_tokens and rb.u == ra.u and rb.c == ra.c
        assert rb.draft_ids == ra.draft_ids
        assert rb.alpha == ra.alpha and (rb.next_E, rb.next_gamma) == (ra.next_E, ra.next_gamma)
    assert (a.T, a.pending) == (b.T, b.pending)


def test_exit_at_the_last_layer_accepts_every_draft(tiny_model):
    cfg, weights, prompt = tiny_model
    o = Oracle(cfg, weights)
    o.prefill(prompt)
    o.sample_first(0.9, 0.9, 0.5)
    gen = torch.Generator().manual_seed(6)
    for g in (1, 3, 4):
        T0 = o.T
        r = o.round_sample(cfg.n_layers, g, 0.9, 0.9, torch.rand(2 * g + 1, generator=gen).tolist())
        assert r.u == g and len(r.out_tokens) == g + 1 and o.T == T0 + g + 1
        assert r.out_tokens[:g] == r.draft_ids


def test_sampled_round_bookkeeping(tiny_model):
    """Emitted tokens are the accepted drafts plus one; the cache grows by as many; the statistics
    count greedy shadow matches over rows 0..u; every emitted token has target probability > 0 in
    the nucleus it was judged against."""
    cfg, weights, prompt = tiny_model
    o = Oracle(cfg, weights)
    o.prefill(prompt)
    o.sample_first(0.8, 0.9, 0.1)
    gen = torch.Generator().manual_seed(7)
    rejected = 0
    for k in range(12):
        E, g = 1 + k % 3, 1 + k % 4
        T0 = o.T
        r = o.round_sample(E, g, 0.8, 0.9, torch.rand(2 * g + 1, generator=gen).tolist())
        assert r.out_tokens[:r.u] == r.draft_ids[:r.u] and len(r.out_tokens) == r.u + 1
        assert o.T == T0 + r.u + 1 and o.pending == r.out_tokens[-1]
        for l in range(1, cfg.n_layers + 1):
            assert r.c[l] == sum(r.shadow[l][i] == r.shadow[cfg.n_layers][i] for i in range(r.u + 1))
        assert r.c[cfg.n_layers] == r.n == r.u + 1
        for i in range(r.u):
            assert float(r.p_dists[i][r.draft_ids[i]]) > 0.0
        assert float(r.last_dist[r.out_tokens[-1]]) > 0.0
        if r.u < g:
            rejected += 1
            x = r.draft_ids[r.u]
            assert float(r.last_dist[x]) == 0.0 or float(r.p_dists[r.u][x]) > float(r.q_dists[r.u][x])
    assert rejected > 0


def test_draft_exiting_under_sampling_limits(tiny_model):
    """tau = 0 never stops (the plain sampled round); tau > 1 stops at once (a round of one token drawn
    from the target with the last uniform number); at low temperature it is the greedy round with
    draft-exiting."""
    cfg, weights, prompt = tiny_model
    gen = torch.Generator().manual_seed(11)
    a, b, c, d, e = (Oracle(cfg, weights) for _ in range(5))
    for o in (a, b, c, d, e):
        o.prefill(prompt)
    for o in (a, b, c):
        o.sample_first(0.8, 0.9, 0.3)
    for (E, cap) in [(2, 4), (1, 3), (3, 4), (2, 1)]:
        un = torch.rand(2 * cap + 1, generator=gen).tolist()
        ra = a.round_sample(E, cap, 0.8, 0.9, un)
        rb = b.round_sample(E, cap, 0.8, 0.9, un, tau=0.0)
        assert rb.out_tokens == ra.out_tokens and rb.u == ra.u and not rb.stopped_early
        assert len(rb.draft_conf) == cap and rb.gamma == cap
        rc = c.round_sample(E, cap, 0.8, 0.9, un, tau=1.5)
        assert rc.stopped_early and rc.gamma == 0 and rc.u == 0 and len(rc.out_tokens) == 1
        assert rc.out_tokens[0] == int(inverse_cdf(rc.p_dists[0], un[2 * cap])) and len(rc.draft_conf) == 1
        tau = 0.5 * (max(rb.draft_conf) + min(rb.draft_conf))
        rd = d.round(E, cap, tau=tau)
        re_ = e.round_sample(E, cap, 1e-5, 1.0, un, tau=tau)
        assert re_.out_tokens == rd.out_tokens and re_.stopped_early == rd.stopped_early and re_.gamma == rd.gamma
        assert re_.draft_conf == rd.draft_conf and re_.c == rd.c
        # keep the three sampled contexts on the same tokens
        for o in (b, c):
            o.T, o.pending = a.T, a.pending
            for l in range(1, cfg.n_layers + 1):
                o.K[l], o.V[l] = a.K[l].clone(), a.V[l].clone()
