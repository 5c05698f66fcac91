"""Pins for the oracle's DEL policy arithmetic (Sections 4.1-4.3, Eq. 1-2, Appendix B)."""
import itertools
import random

import pytest

from conftest import read_golden
from oracle.del_oracle import (DelStats, decayed_sum, first_mismatch, matched_counts,
                               select_exit_and_length, tpl)


def test_tpl_worked_values_eq1():
    for a, l, d, L, want in read_golden("tpl_eq1_worked.txt"):
        got = tpl(float(a), int(l), int(d), int(L))
        assert got == pytest.approx(float(want), rel=1e-12)


def test_tpl_sum_equals_closed_form():
    # the paper states the sum and the closed form are the same quantity (below Eq. 1)
    rng = random.Random(1)
    for _ in range(300):
        a = rng.uniform(0.0, 0.999)
        l, d, L = rng.randint(1, 79), rng.randint(0, 18), 80
        closed = (1 - a ** (d + 1)) / ((1 - a) * (d * l + L))
        assert tpl(a, l, d, L) == pytest.approx(closed, rel=1e-11)


def test_tpl_special_cases():
    for L in (4, 16, 32, 40, 80):
        for l in range(1, L):
            assert tpl(0.37, l, 0, L) == pytest.approx(1.0 / L, rel=1e-15)   # d = 0: vanilla step
            for d in (1, 5, 12):
                assert tpl(0.0, l, d, L) == pytest.approx(1.0 / (d * l + L))
                assert tpl(1.0, l, d, L) == pytest.approx((d + 1) / (d * l + L))


def test_vanilla_etpl_printed_in_tables():
    for _, L, printed in read_golden("vanilla_etpl_table1.txt"):
        assert tpl(0.5, 3, 0, int(L)) == pytest.approx(float(printed), abs=5.1e-4)   # printed to 3 decimals


def test_ls_rows_imply_tokens_per_round_in_range():
    # cost model gamma*E + L (Section 4.1) against Table 1's LS rows
    for row in read_golden("ls_etpl_table1.txt"):
        L, E, g = int(row[1]), int(row[2]), int(row[3])
        for e in row[4:]:
            per_round = float(e) * (g * E + L)
            assert 1.0 <= per_round <= g + 1
            # the expected tokens of Eq. 1 must be able to reach it for some alpha in [0,1]
            assert tpl(1.0, E, g, L) * (g * E + L) >= per_round


def test_decayed_sum_definition():
    omega, back, centre, tol = (float(x) for x in read_golden("decay_half_life.txt")[0])
    back = int(back)
    # unit impulse `back` rounds ago followed by zeros: weight must be ~0.5; newest has weight 1
    a = [0.0] * (back + 1)
    a[0] = 1.0
    assert decayed_sum(a, omega) == pytest.approx(centre, abs=tol)
    a = [0.0] * (back + 1)
    a[-1] = 1.0
    assert decayed_sum(a, omega) == 1.0
    # omega = 1: plain sum; omega = 0: last element only
    xs = [3, 1, 4, 1, 5, 9, 2, 6]
    assert decayed_sum(xs, 1.0) == sum(xs)
    assert decayed_sum(xs, 0.0) == xs[-1]
    # recurrence S_r = omega * S_{r-1} + a[r-1]
    s = 0.0
    for i, x in enumerate(xs):
        s = 0.95 * s + x
        assert decayed_sum(xs[:i + 1], 0.95) == pytest.approx(s, rel=1e-13)


def test_figure2_round_counts():
    rows = {r[0]: [int(x) for x in r[1:]] for r in read_golden("figure2_round.txt")}
    gamma = rows["gamma"][0]
    u = first_mismatch(rows["draft"], rows["target"], gamma)
    assert u == rows["u"][0]
    assert rows["target"][:u + 1] == rows["emitted"]
    # all drafts right: u = gamma, gamma + 1 tokens emitted (Section 2)
    assert first_mismatch(rows["target"][:gamma], rows["target"], gamma) == gamma
    # first draft wrong: one token
    assert first_mismatch([0] * gamma, rows["target"], gamma) == 0
    assert first_mismatch([], [7], 0) == 0


def test_matched_counts_by_hand():
    target = [5, 6, 7, 8]
    shadow = [[0] * 4,          # index 0 unused
              [5, 0, 7, 8],     # layer 1
              [5, 6, 0, 8],     # layer 2
              [5, 6, 7, 8]]     # layer L
    assert matched_counts(shadow, target, 3) == [0, 3, 3, 4]
    assert matched_counts(shadow, target, 1) == [0, 1, 2, 2]
    assert matched_counts(shadow, target, 0) == [0, 1, 1, 1]


def test_alpha_ratio_of_decayed_sums():
    st = DelStats(3, 0.5, 4)
    st.append([0, 1, 2, 2], 2, 1)
    st.append([0, 0, 3, 4], 4, 3)
    # S(c^1) = 0.5*1 + 0 = 0.5 ; S(c^2) = 0.5*2 + 3 = 4 ; S(n) = 0.5*2 + 4 = 5
    al = st.alpha()
    assert al[1] == pytest.approx(0.1) and al[2] == pytest.approx(0.8) and al[3] == pytest.approx(1.0)
    # alpha stays in [0, 1] and alpha_L == 1 when c^L == n (reading R1)
    assert all(0.0 <= a <= 1.0 for a in al)


def _select_other_order(alpha, L, d_max):
    """Second scan, d-major and from the top, with the tie rule applied explicitly."""
    cands = []
    for d in range(d_max, -1, -1):
        for l in range(L - 1, 0, -1):
            cands.append((tpl(alpha[l], l, d, L), l, d))
    best = max(c[0] for c in cands)
    ties = [(l, d) for v, l, d in cands if v == best]
    return min(ties)          # smallest layer, then smallest d


def test_selection_exhaustive_and_ties():
    rng = random.Random(7)
    for L, d_max in ((4, 4), (16, 8), (32, 8), (80, 12)):
        for _ in range(40):
            alpha = [0.0] + sorted(rng.random() for _ in range(L - 1)) + [1.0]
            assert select_exit_and_length(alpha, L, d_max) == _select_other_order(alpha, L, d_max)
        # all-zero alpha: every (l, d=0) ties at 1/L and is the maximum -> (1, 0)
        assert select_exit_and_length([0.0] * (L + 1), L, d_max) == (1, 0)
        # perfect first layer: cheapest drafts, longest speculation
        assert select_exit_and_length([0.0] + [1.0] * L, L, d_max) == (1, d_max)


def test_selection_monotone_in_alpha_of_choice():
    rng = random.Random(11)
    L, d_max = 16, 8
    for _ in range(50):
        alpha = [0.0] + [rng.random() for _ in range(L - 1)] + [1.0]
        l0, d0 = select_exit_and_length(alpha, L, d_max)
        alpha2 = list(alpha)
        alpha2[l0] = min(1.0, alpha[l0] + 0.1)
        l1, _ = select_exit_and_length(alpha2, L, d_max)
        if d0 > 0:
            assert l1 == l0
