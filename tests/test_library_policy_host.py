"""The library's host-side policy arithmetic (statistics, alpha, tau, TPL arg-max) against the oracle's,
on random round histories.  No GPU: del_policy_step needs no context."""
import random

import pytest

from oracle.del_oracle import DelStats
from paper_2504_05598_amd.binding import del_policy_step


@pytest.mark.parametrize("L,d_max,omega", [(4, 4, 0.95), (16, 8, 0.95), (32, 8, 0.5), (80, 12, 1.0), (6, 6, 0.0)])
def test_running_sums_alpha_tau_and_selection_match_the_oracle(L, d_max, omega):
    rng = random.Random(L * 131 + d_max)
    ora = DelStats(L, omega, d_max)
    state = {"S_c": [0.0] * (L + 1), "S_n": 0.0, "S_tcs": [0.0] * (L + 1), "S_fcs": [0.0] * (L + 1)}
    for r in range(40):
        n = rng.randint(1, d_max + 1)
        # agreement rises with depth, layer L always matches itself
        c = [0] + [min(n, sum(rng.random() < (l / L) ** 0.7 for _ in range(n))) for l in range(1, L)] + [n]
        tcs = [0.0] + [sum(rng.uniform(0.3, 1.0) for _ in range(c[l])) for l in range(1, L + 1)]
        fcs = [0.0] + [sum(rng.uniform(0.0, 0.5) for _ in range(n - c[l])) for l in range(1, L + 1)]
        ora.append(c, n, n - 1, tcs, fcs)
        state = del_policy_step(L, d_max, omega, c, n, tcs, fcs, state)
        a, t = ora.alpha(), ora.tau()
        assert state["S_n"] == pytest.approx(ora.S_n(), rel=1e-12)
        for l in range(1, L + 1):
            assert state["S_c"][l] == pytest.approx(ora.S_c(l), rel=1e-12, abs=1e-300)
            assert state["alpha"][l] == pytest.approx(a[l], rel=1e-12, abs=1e-15)
            assert state["tau"][l] == pytest.approx(t[l], rel=1e-11, abs=1e-15)
        # selection: evaluate with the library's own alpha so that a last-bit difference of the
        # running sums cannot pick another maximum
        from oracle.del_oracle import select_exit_and_length
        assert (state["next_E"], state["next_gamma"]) == select_exit_and_length(state["alpha"], L, d_max)
    assert 1 <= state["next_E"] < max(L, 2) and 0 <= state["next_gamma"] <= d_max


def test_all_tie_at_zero_alpha_picks_first_layer_and_no_drafts():
    L, d_max = 8, 4
    state = {"S_c": [0.0] * (L + 1), "S_n": 0.0, "S_tcs": [0.0] * (L + 1), "S_fcs": [0.0] * (L + 1)}
    out = del_policy_step(L, d_max, 0.95, [0] * L + [3], 3, [0.0] * (L + 1), [0.0] * (L + 1), state)
    assert (out["next_E"], out["next_gamma"]) == (1, 0)
    assert out["alpha"][L] == 1.0 and out["tau"][1] == 0.0


def test_policy_step_properties_random_histories():
    """Properties that hold for any history: alpha in [0, 1] and alpha_L = 1; tau in [0, 1]; the choice is
    an arg-max of Eq. 1 over the grid (no grid point is strictly better); omega = 1 gives plain ratios."""
    from hypothesis import given, settings, strategies as st
    from oracle.del_oracle import tpl

    @settings(max_examples=40, deadline=None)
    @given(st.integers(2, 24), st.integers(0, 10), st.sampled_from([0.0, 0.5, 0.95, 1.0]), st.integers(0, 2**31 - 1),
           st.integers(1, 12))
    def run(L, d_max, omega, seed, n_rounds):
        rng = random.Random(seed)
        state = {"S_c": [0.0] * (L + 1), "S_n": 0.0, "S_tcs": [0.0] * (L + 1), "S_fcs": [0.0] * (L + 1)}
        tot_c, tot_n = [0] * (L + 1), 0
        for _ in range(n_rounds):
            n = rng.randint(1, d_max + 1)
            c = [0] + [rng.randint(0, n) for _ in range(1, L)] + [n]
            tcs = [0.0] + [rng.uniform(0, 1) * c[l] for l in range(1, L + 1)]
            fcs = [0.0] + [rng.uniform(0, 1) * (n - c[l]) for l in range(1, L + 1)]
            state = del_policy_step(L, d_max, omega, c, n, tcs, fcs, state)
            tot_c = [a + b for a, b in zip(tot_c, c)]
            tot_n += n
            a = state["alpha"]
            assert all(0.0 <= a[l] <= 1.0 + 1e-12 for l in range(1, L + 1)) and abs(a[L] - 1.0) < 1e-12
            assert all(0.0 <= state["tau"][l] <= 1.0 + 1e-12 for l in range(1, L + 1))
            E, g = state["next_E"], state["next_gamma"]
            assert 1 <= E <= max(1, L - 1) and 0 <= g <= d_max
            best = tpl(a[E], E, g, L)
            for l in range(1, L):
                for d in range(d_max + 1):
                    assert tpl(a[l], l, d, L) <= best * (1 + 1e-12) + 1e-15
        if omega == 1.0:
            for l in range(1, L + 1):
                assert state["alpha"][l] == pytest.approx(tot_c[l] / tot_n, rel=1e-12)

    run()
