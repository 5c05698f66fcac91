"""The round controllers on the device (run with -m gpu): vanilla, the static LayerSkip schedule (LS), the
finite-state speculation length (FS), DEL's Token-per-Layer selection and full DEL with draft-exiting
(Section 5.1 baselines, Sections 4.3-4.4, Appendix B.4).

controllers.generate drives the library through the C ABI; the CPU oracle then replays the logged
(E, gamma) sequence round by round.  Whatever the controller, greedy self-speculative decoding must
emit the target model's greedy tokens (Section 2), so the oracle's replay must give the same tokens
and the same number of tokens per round (a difference is tolerated only at a position where the
oracle's top-2 logit gap is below 1e-2, and ends the comparison); eTPL of the log must equal the
oracle's; the FS trajectory must follow its rule and DEL's must equal the oracle's own selections.
"""
import pytest
import torch

from synthdata import get_config, gen_prompt

pytestmark = pytest.mark.gpu

GAP_TOL = 1e-2


def _replay(oracle, prompt, log):
    pre = oracle.prefill(prompt)
    toks, gaps, recs = [pre.first_token], [pre.first_gap], []
    for (E, g, n) in log:
        r = oracle.round(E, g)
        recs.append(r)
        toks.extend(r.out_tokens)
        gaps.extend(r.gaps[oracle.L][:r.u + 1])
    return toks, gaps, recs, pre


@pytest.mark.parametrize("name", ["mini_gqa", "mini_mha"])
def test_controllers_on_device_against_oracle_replay(name):
    from gpu_harness import gpu_context, log as say
    from oracle.del_oracle import Oracle, empirical_tpl as oracle_etpl
    from paper_2504_05598_amd.controllers import empirical_tpl, fs_next_gamma, generate
    cfg = get_config(name)
    ctx, host = gpu_context(cfg, keep_host=True)
    oracle = Oracle(cfg, host, dtype=torch.float64)
    prompt = gen_prompt(cfg).tolist()
    n = cfg.gen_len
    L = cfg.n_layers
    for controller, kw in (("vanilla", {}), ("ls", dict(E=2, gamma=3)), ("fs", dict(E=2, gamma=2)), ("del", {}),
                           ("del_full", {})):
        toks, rlog = generate(ctx, prompt, n, controller, **kw)
        assert len(toks) >= n and sum(k for _, _, k in rlog) == len(toks) - 1
        assert all(1 <= k <= g + 1 and 1 <= E <= L and 0 <= g <= cfg.d_max for E, g, k in rlog)
        want, gaps, recs, pre = _replay(oracle, prompt, rlog)
        # tokens: equal up to a first difference, which must sit on an oracle near-tie
        same = next((i for i, (a, b) in enumerate(zip(toks, want)) if a != b), min(len(toks), len(want)))
        if same < min(len(toks), len(want)):
            assert gaps[same] < GAP_TOL, f"{controller}: token {same} gpu {toks[same]} oracle {want[same]} gap {gaps[same]}"
        # rounds wholly inside the common prefix: same number of emitted tokens, hence same acceptance count
        pos, full_rounds = 1, 0
        for (E, g, k), r in zip(rlog, recs):
            if pos + max(k, len(r.out_tokens)) > same:
                break
            assert k == len(r.out_tokens) == r.u + 1, (controller, full_rounds, k, r.u)
            pos += k
            full_rounds += 1
        say(f"[{name} {controller}] {len(rlog)} rounds, {len(toks)} tokens, equal to the oracle's replay for {same} tokens "
            f"({full_rounds} whole rounds), eTPL {empirical_tpl(rlog, L):.4f}")
        assert same >= min(len(toks), len(want)) // 2, "too little of the run could be compared"
        if same == len(toks) == len(want):
            assert abs(empirical_tpl(rlog, L) - oracle_etpl(recs, L)) < 1e-12
        # controller rules on the compared rounds
        if controller == "vanilla":
            assert all((E, g, k) == (1, 0, 1) for E, g, k in rlog)
            assert empirical_tpl(rlog, L) == pytest.approx(1.0 / L)
        if controller == "ls":
            assert all(E == 2 and g == min(3, n - 1 - sum(k for _, _, k in rlog[:i]) - 1) for i, (E, g, _) in enumerate(rlog))
        if controller == "fs":
            g_want = 2
            for i in range(full_rounds):
                E, g, k = rlog[i]
                room = n - 1 - sum(kk for _, _, kk in rlog[:i]) - 1
                assert E == 2 and g == min(g_want, room), (i, g, g_want, room)
                g_want = fs_next_gamma(g_want, recs[i].u == g and k == g + 1, cfg.d_max)
        if controller == "del":
            E_want, g_want = pre.next_E, pre.next_gamma
            for i in range(full_rounds):
                E, g, k = rlog[i]
                room = n - 1 - sum(kk for _, _, kk in rlog[:i]) - 1
                if any(x < GAP_TOL for l in range(1, L + 1) for x in recs[i].gaps[l]) or \
                        (i == 0 and any(x < GAP_TOL for row in pre.gaps[1:] for x in row)):
                    break       # a near-tie shadow token may legitimately move the statistics from here on
                assert (E, g) == (E_want, min(g_want, room)), (i, (E, g), (E_want, g_want))
                E_want, g_want = recs[i].next_E, recs[i].next_gamma
    ctx.close()
