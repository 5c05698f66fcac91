"""Pins for the oracle's dynamic draft-exiting (Section 4.4, Eq. 3, Algorithm 1 loop)."""
import pytest
import torch

from conftest import read_golden
from oracle.del_oracle import (DelStats, Oracle, confidence_sums, generate_del_full, generate_fixed,
                               generate_vanilla)


def test_tau_worked_values_eq3():
    for row in read_golden("tau_eq3_worked.txt"):
        omega, want = float(row[0]), float(row[1])
        rounds = [row[2 + 4 * i: 6 + 4 * i] for i in range((len(row) - 2) // 4)]
        st = DelStats(2, omega, 4)
        for tcs, c, fcs, n in rounds:
            st.append([0, int(c), int(n)], int(n), int(n) - 1, [0.0, float(tcs), 0.0], [0.0, float(fcs), 0.0])
        assert st.tau()[1] == pytest.approx(want, rel=1e-12)


def test_tau_zero_denominators_count_as_zero():
    st = DelStats(2, 0.95, 4)
    st.append([0, 3, 3], 3, 2, [0.0, 2.4, 3.0], [0.0, 0.0, 0.0])     # layer 1 always matched
    assert st.tau()[1] == pytest.approx(0.5 * (2.4 / 3))
    st = DelStats(2, 0.95, 4)
    st.append([0, 0, 3], 3, 2, [0.0, 0.0, 3.0], [0.0, 0.9, 0.0])     # layer 1 never matched
    assert st.tau()[1] == pytest.approx(0.5 * (0.9 / 3))


def test_confidence_sums_by_hand():
    target = [5, 6, 7, 8]
    shadow = [[0] * 4, [5, 0, 7, 8], [5, 6, 7, 8]]
    conf = [[0.0] * 4, [0.5, 0.25, 0.125, 0.0625], [1.0, 1.0, 1.0, 1.0]]
    tcs, fcs = confidence_sums(shadow, conf, target, 2)
    assert tcs[1] == 0.625 and fcs[1] == 0.25 and tcs[2] == 3.0 and fcs[2] == 0.0
    tcs, fcs = confidence_sums(shadow, conf, target, 0)
    assert tcs[1] == 0.5 and fcs[1] == 0.0


def test_confidence_is_softmax_probability_of_the_greedy_token(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    h = torch.stack([o.embed(t) for t in prompt[:5]])
    for l in range(1, cfg.n_layers + 1):
        h = o.layer(l, h, 0)
    ids, gaps, conf = o.head_conf(h)
    probs = torch.softmax(o.logits(h), dim=-1)
    for r in range(5):
        assert ids[r] == int(probs[r].argmax())
        assert conf[r] == pytest.approx(float(probs[r].max()), rel=1e-12)
        assert 1.0 / cfg.vocab <= conf[r] <= 1.0


def test_full_del_tokens_equal_vanilla_and_break_semantics(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    van = generate_vanilla(o, prompt, cfg.gen_len)
    toks, pre, recs = generate_del_full(o, prompt, cfg.gen_len)
    assert toks == van                                    # Section 2: greedy verification is lossless
    tau_used = pre.tau[pre.next_E]
    assert any(r.stopped_early for r in recs)
    for r in recs:
        assert len(r.draft_conf) == r.gamma + (1 if r.stopped_early else 0)
        assert all(cf >= tau_used for cf in r.draft_conf[:r.gamma])       # appended tokens were confident
        if r.stopped_early:
            assert r.draft_conf[-1] < tau_used and r.gamma < cfg.d_max    # the stopping token is not appended
        assert 1 <= len(r.out_tokens) <= r.gamma + 1
        # draft confidences are layer E's shadow confidences at the same rows
        for i, cf in enumerate(r.draft_conf):
            assert cf == pytest.approx(r.conf[r.E][i], rel=1e-12)
        # tcs + fcs = all confidence inside the valid context; tau is the midpoint of the two means
        for l in range(1, cfg.n_layers + 1):
            assert r.tcs[l] + r.fcs[l] == pytest.approx(sum(r.conf[l][:r.u + 1]), rel=1e-12)
        tau_used = r.tau[r.next_E]


def test_threshold_extremes_reduce_to_fixed_schedules(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    o.prefill(prompt)
    a = [o.round(2, cfg.d_max, tau=0.0) for _ in range(6)]          # never stops: LS(E, d_max)
    assert all(not r.stopped_early and r.gamma == cfg.d_max for r in a)
    _, fixed = generate_fixed(o, prompt, sum(len(r.out_tokens) for r in a) + 1, 2, cfg.d_max)
    assert [r.out_tokens for r in a] == [r.out_tokens for r in fixed[:6]]
    o.prefill(prompt)
    b = [o.round(2, cfg.d_max, tau=1.5) for _ in range(6)]          # always stops at once: vanilla steps
    assert all(r.stopped_early and r.gamma == 0 and len(r.out_tokens) == 1 for r in b)


def test_running_confidence_sums_match_their_definition(tiny_model):
    cfg, w, prompt = tiny_model
    o = Oracle(cfg, w)
    _, pre, recs = generate_del_full(o, prompt, 32)
    L = cfg.n_layers
    w_ = pre.window
    target = pre.shadow[L]
    st, sf = [0.0] * (L + 1), [0.0] * (L + 1)
    for l in range(1, L + 1):
        for i in range(w_):
            if pre.shadow[l][i] == target[i]:
                st[l] += pre.conf[l][i]
            else:
                sf[l] += pre.conf[l][i]
    for r in recs:
        for l in range(1, L + 1):
            st[l] = cfg.omega * st[l] + r.tcs[l]
            sf[l] = cfg.omega * sf[l] + r.fcs[l]
            assert r.S_tcs[l] == pytest.approx(st[l], rel=1e-11, abs=1e-15)
            assert r.S_fcs[l] == pytest.approx(sf[l], rel=1e-11, abs=1e-15)
