"""Host-side round controllers (no GPU): the finite-state rule and the loop's bookkeeping."""
from paper_2504_05598_amd.controllers import empirical_tpl, fs_next_gamma, generate


def test_finite_state_rule():
    # Section 5.1: +1 after a fully accepted round, -1 after any rejection
    assert fs_next_gamma(3, True, 8) == 4 and fs_next_gamma(3, False, 8) == 2
    assert fs_next_gamma(8, True, 8) == 8 and fs_next_gamma(1, False, 8) == 1


class _FakeCfg:
    n_layers, d_max = 8, 4


class _FakeCtx:
    """Stands in for DelContext: accepts every draft of a round iff gamma is odd."""
    cfg = _FakeCfg()

    def __init__(self):
        self.calls = []

    def prefill(self, prompt):
        return 7, 2, 3

    def round(self, E, g):
        self.calls.append((E, g))
        return [1] * (g + 1 if g % 2 else 1)

    def sample_first(self, temperature, top_p, r):
        self.first_r = r
        return 9

    def round_sample(self, E, g, temperature, top_p, un):
        assert len(un) == 2 * g + 1 and all(0.0 <= x < 1.0 for x in un)
        self.calls.append((E, g))
        return [2] * (g + 1 if g % 2 else 1)

    def stats(self):
        return {"next_E": 2, "next_gamma": 3, "tau": [0.0] * 9}


def test_generate_bookkeeping_and_fs_trajectory():
    ctx = _FakeCtx()
    toks, log = generate(ctx, [1, 2, 3], 12, "fs", E=3, gamma=2)
    assert len(toks) == 12 and toks[0] == 7
    assert [g for _, g in ctx.calls][:4] == [2, 1, 2, 1]       # reject at 2 -> 1, accept at 1 -> 2, ...
    assert all(E == 3 for E, _ in ctx.calls)
    assert sum(n for _, _, n in log) == 11
    ctx = _FakeCtx()
    toks, log = generate(ctx, [1], 9, "vanilla")
    assert all(c == (1, 0) for c in ctx.calls) and empirical_tpl(log, 8) == 1 / 8
    ctx = _FakeCtx()
    toks, log = generate(ctx, [1], 20, "ls", E=2, gamma=3)
    assert all(E == 2 for E, _ in ctx.calls) and ctx.calls[-1][1] <= 3 and len(toks) == 20


def test_generate_with_sampling_draws_the_first_token_and_passes_the_right_number_of_uniforms():
    ctx = _FakeCtx()
    draws = []

    def uniforms(k, count):
        draws.append((k, count))
        return [0.25] * count
    toks, log = generate(ctx, [1, 2], 10, "del", sampling=(0.6, 0.95, uniforms))
    assert toks[0] == 9 and ctx.first_r == 0.25 and len(toks) == 10
    assert draws[0] == (0, 1) and [k for k, _ in draws] == list(range(len(draws)))
    assert all(count == 2 * g + 1 for (_, count), (_, g) in zip(draws[1:], ctx.calls))
