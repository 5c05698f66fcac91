"""Lock-step parity harness: HIP library versus the CPU oracle on the same seeded inputs.

Protocol.  Both sides prefill on the same prompt and then run the same rounds with the
oracle's (E, gamma).  Token ids, acceptance counts and the selected (E, gamma) must be equal,
except where the oracle's top-2 logit gap at that very (layer, row) is below GAP_TOL; hidden
states must agree to HID_TOL (max abs difference over max abs oracle value, per layer).
A tolerated flip makes the two contexts differ, so the harness then re-prefills the GPU
context on prompt + oracle tokens and imports the oracle's statistics, and goes on.
"""
from __future__ import annotations

import sys
from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch

from oracle.del_oracle import Oracle
from paper_2504_05598_amd.binding import DelContext
from synthdata import gen_tensor, iter_tensor_specs

GAP_TOL = 1e-2     # oracle top-2 logit gap below which either of the top two ids is accepted
HID_TOL = 2e-2     # bf16 weights, fp32 accumulation (stated by the benchmark contract)
CONF_RTOL = 5e-3   # confidence = 1 / sum exp(logit - max): a few 1e-4 of logit error over the vocabulary


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gpu_context(cfg, use_mfma=True, max_context=None, keep_host=False):
    """Generate the model on the GPU with the shared generator and load it through the C ABI.
    Returns (ctx, host_weights or None)."""
    ctx = DelContext(cfg, use_mfma=use_mfma, max_context=max_context)
    host = {} if keep_host else None
    for layer, kind in iter_tensor_specs(cfg):
        t = gen_tensor(cfg, layer, kind, device="cuda")
        ctx.load_tensor(layer, kind, t)
        if keep_host:
            host[(layer, kind)] = t.cpu()
        del t
    torch.cuda.synchronize()
    return ctx, host


@dataclass
class ParityReport:
    rounds: int = 0
    compared_ids: int = 0
    flips: int = 0
    resyncs: int = 0
    max_hidden_err: float = 0.0
    tokens: List[int] = field(default_factory=list)
    decisions: int = 0


def _rel_err(got: np.ndarray, want: np.ndarray) -> float:
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))


def _resync(ctx: DelContext, oracle: Oracle, prompt, emitted, rep: ParityReport):
    """GPU context := prefill(prompt + all emitted tokens but the last), pending := last."""
    first, _, _ = ctx.prefill(list(prompt) + emitted[:-1])
    if first != emitted[-1]:
        ctx.set_pending(emitted[-1])
    L = oracle.L
    ctx.set_stats([0.0] + [oracle.stats.S_c(l) for l in range(1, L + 1)], oracle.stats.S_n(),
                  [0.0] + [oracle.stats.S_tcs(l) for l in range(1, L + 1)],
                  [0.0] + [oracle.stats.S_fcs(l) for l in range(1, L + 1)])
    T, pend = ctx.state()
    assert T == oracle.T and pend == oracle.pending
    rep.resyncs += 1


def _close(a, b, rtol):
    return abs(a - b) <= rtol * max(abs(a), abs(b)) + 1e-9


def lockstep(cfg, oracle: Oracle, ctx: DelContext, prompt, n_tokens, schedule=None,
             check_hidden=True, max_rounds=None, dynamic=False) -> ParityReport:
    """schedule: None = DEL-selected (E, gamma) from the oracle; or a fixed (E, gamma).
    dynamic: full DEL (Section 4.4): E from the oracle's selection, the draft loop stops on the
    oracle's tau_E; a stop decision may differ only where the oracle's confidence is within
    CONF_RTOL of the threshold."""
    rep = ParityReport()
    L, d_max = cfg.n_layers, cfg.d_max
    pre = oracle.prefill(prompt, keep_hidden=check_hidden)
    first, gE, gg = ctx.prefill(prompt)
    st = ctx.stats()
    # ---- prefill: first token, window statistics, first (E, gamma)
    near = [[g < GAP_TOL for g in row] for row in pre.gaps]
    if first != pre.first_token:
        assert pre.first_gap < GAP_TOL, f"first token {first} != {pre.first_token}, gap {pre.first_gap}"
        rep.flips += 1
    w = pre.window
    for l in range(1, L + 1):
        slack = sum(1 for i in range(w) if near[l][i] or near[L][i])
        assert abs(st["last_c"][l] - pre.c[l]) <= slack, (l, st["last_c"][l], pre.c[l], slack)
    exact = all(st["last_c"][l] == pre.c[l] for l in range(1, L + 1)) and first == pre.first_token
    if check_hidden:
        for l in (1, L // 2 + 1, L):
            # the last prompt position is the last row of the last prefill pass
            err = _rel_err(ctx.hidden(l, ctx.last_rows() - 1), pre.hidden[l, -1].float().numpy())
            rep.max_hidden_err = max(rep.max_hidden_err, err)
            assert err <= HID_TOL, ("prefill hidden", l, err)
    emitted = [pre.first_token]
    if exact:
        assert (gE, gg) == (pre.next_E, pre.next_gamma)
        for l in range(1, L + 1):
            assert st["alpha"][l] == pre.alpha[l] or abs(st["alpha"][l] - pre.alpha[l]) < 1e-12
            assert _close(st["tau"][l], pre.tau[l], CONF_RTOL), ("prefill tau", l, st["tau"][l], pre.tau[l])
    else:
        _resync(ctx, oracle, prompt, emitted, rep)
    E, gamma = (pre.next_E, pre.next_gamma) if schedule is None else schedule
    tau = pre.tau[E]
    while len(emitted) < n_tokens and (max_rounds is None or rep.rounds < max_rounds):
        stop_flip = False
        if dynamic:
            g = min(cfg.d_max, n_tokens - len(emitted) - 1)
            r = oracle.round(E, g, keep_hidden=check_hidden, tau=tau)
            out, g_gpu, stopped = ctx.round_dynamic(E, tau, g)
            st = ctx.stats()
            if (g_gpu, stopped) != (r.gamma, r.stopped_early):
                # the two sides stopped at different steps: tolerated only on a near-threshold confidence
                k = min(g_gpu, r.gamma)
                assert k < len(r.draft_conf) and _close(r.draft_conf[k], tau, CONF_RTOL), (
                    f"round {rep.rounds + 1}: gpu drafted {g_gpu} (stopped {stopped}), oracle {r.gamma} "
                    f"(stopped {r.stopped_early}), oracle confidences {r.draft_conf}, tau {tau}")
                stop_flip = True
                rep.flips += 1
            g = min(g_gpu, r.gamma)
            for i, cf in enumerate(st["last_draft_conf"][:g]):
                if st["last_draft"][:i] == r.draft_ids[:i]:       # same inputs up to this step
                    assert _close(cf, r.draft_conf[i], CONF_RTOL), ("draft confidence", i, cf, r.draft_conf[i])
        else:
            g = min(gamma, n_tokens - len(emitted) - 1)
            r = oracle.round(E, g, keep_hidden=check_hidden)
            out = ctx.round(E, g)
            st = ctx.stats()
        rep.rounds += 1
        # rows whose inputs are the same on both sides: up to the first differing draft
        same_rows = g + 1
        for i in range(g):
            if st["last_draft"][i] != r.draft_ids[i]:
                same_rows = i + 1
                break
        flipped = False
        for l in range(1, L + 1):
            for i in range(same_rows):
                rep.compared_ids += 1
                if st["last_shadow"][l][i] == r.shadow[l][i]:
                    assert _close(st["last_conf"][l][i], r.conf[l][i], CONF_RTOL), (
                        "confidence", rep.rounds, l, i, st["last_conf"][l][i], r.conf[l][i])
                if st["last_shadow"][l][i] != r.shadow[l][i]:
                    assert r.gaps[l][i] < GAP_TOL, (
                        f"round {rep.rounds} E={E} g={g} layer {l} row {i}: gpu {st['last_shadow'][l][i]} "
                        f"oracle {r.shadow[l][i]} gap {r.gaps[l][i]}")
                    rep.flips += 1
                    flipped = True
        if check_hidden:
            for l in range(1, L + 1):
                want = r.hidden[l, :same_rows].float().numpy()
                got = np.stack([ctx.hidden(l, i) for i in range(same_rows)])
                err = _rel_err(got, want)
                rep.max_hidden_err = max(rep.max_hidden_err, err)
                assert err <= HID_TOL, ("hidden", rep.rounds, l, err)
        emitted.extend(r.out_tokens)
        if not flipped and not stop_flip and same_rows == g + 1:
            # identical ids everywhere: counts, tokens, statistics and selection must be equal
            assert out == r.out_tokens, (out, r.out_tokens)
            assert st["last_u"] == r.u and st["last_n"] == r.n
            assert st["last_c"][1:] == r.c[1:]
            assert st["last_draft"] == r.draft_ids
            for l in range(1, L + 1):
                assert abs(st["S_c"][l] - r.S_c[l]) <= 1e-9 * max(1.0, r.S_c[l])
                assert abs(st["alpha"][l] - r.alpha[l]) <= 1e-9
            assert abs(st["S_n"] - r.S_n) <= 1e-9 * r.S_n
            assert (st["next_E"], st["next_gamma"]) == (r.next_E, r.next_gamma)
            for l in range(1, L + 1):
                assert _close(st["S_tcs"][l], r.S_tcs[l], CONF_RTOL) and _close(st["S_fcs"][l], r.S_fcs[l], CONF_RTOL)
                assert _close(st["tau"][l], r.tau[l], CONF_RTOL), ("tau", l, st["tau"][l], r.tau[l])
            T, pend = ctx.state()
            assert T == oracle.T and pend == oracle.pending
        else:
            _resync(ctx, oracle, prompt, emitted, rep)
        if schedule is None:
            E, gamma = r.next_E, r.next_gamma
        tau = r.tau[E]
    rep.tokens = emitted
    return rep


def gpu_generate(ctx: DelContext, prompt, n_tokens, schedule=None, dynamic=False):
    """Free-running generation through the C ABI with the library's own (E, gamma) choice
    (or a fixed schedule; or, dynamic, the library's E and tau_E with draft-exiting).
    Returns tokens and the per-round log."""
    first, E, gamma = ctx.prefill(prompt)
    if schedule is not None:
        E, gamma = schedule
    toks = [first]
    rounds = []
    while len(toks) < n_tokens:
        g = min(ctx.cfg.d_max if dynamic else gamma, n_tokens - len(toks) - 1)
        if dynamic:
            out, g, _ = ctx.round_dynamic(E, ctx.stats()["tau"][E], g)
        else:
            out = ctx.round(E, g)
        assert 1 <= len(out) <= g + 1
        rounds.append((E, g, len(out)))
        toks.extend(out)
        if schedule is None:
            st = ctx.stats()
            E, gamma = st["next_E"], st["next_gamma"]
    return toks, rounds


# ---- speculative sampling ------------------------------------------------------------------
# A sampled decision is a uniform number against a boundary of a cumulative distribution (a draw) or
# against a probability ratio (an acceptance).  The two sides' logits differ by rounding, so the
# boundaries move by a little: a decision may differ only where the oracle's uniform number lies
# within the tolerance of the boundary that decides for the GPU's outcome.
CUT_TOL = 2e-2     # nucleus: a token may be in or out if the kept mass is this close to top_p


def _interval_distance(dist: torch.Tensor, token: int, r: float) -> float:
    """How far r lies from the interval of `token` in the cumulative distribution (0 inside)."""
    cdf = torch.cumsum(dist, dim=0)
    hi = float(cdf[token])
    lo = float(cdf[token - 1]) if token > 0 else 0.0
    return max(lo - r, r - hi, 0.0)


def _cut_slack(oracle: Oracle, h_row: torch.Tensor, dist: torch.Tensor, temperature: float, top_p: float) -> float:
    """Mass that moves when the token at the nucleus cut flips in or out; 0 if the cut is clear."""
    from oracle.del_oracle import tempered_nucleus
    if top_p >= 1.0:
        return 0.0
    full = tempered_nucleus(oracle.logits(h_row[None, :])[0], temperature, 1.0)
    kept = dist > 0
    mass = float(full[kept].sum())
    last_in = float(full[kept].min())
    out = full[~kept]
    first_out = float(out.max()) if out.numel() else 0.0
    if mass - top_p < CUT_TOL * top_p or top_p - (mass - last_in) < CUT_TOL * top_p:
        return 2.0 * max(last_in, first_out) / mass
    return 0.0


def lockstep_sample(cfg, oracle: Oracle, ctx: DelContext, prompt, n_tokens, temperature, top_p,
                    sample_tol, ratio_tol, schedule=None, stream0=0, dynamic=False) -> ParityReport:
    """Speculative sampling in lock-step: the same uniform numbers on both sides; drafts, acceptance
    count, emitted tokens, greedy shadow tokens, statistics and the next (E, gamma) are compared.
    A differing sampled decision must be a near-boundary one (see above) and is followed by a
    re-prefill of the GPU context on the oracle's tokens.
    dynamic: draft-exiting on top: the cap is d_max, the loop stops on the oracle's tau_E; the stop
    decision may differ only where the oracle's confidence is within CONF_RTOL of the threshold."""
    from synthdata import gen_uniforms
    rep = ParityReport()
    L = cfg.n_layers
    pre = oracle.prefill(prompt, keep_hidden=True)
    first, gE, gg = ctx.prefill(prompt)
    assert first == pre.first_token or pre.first_gap < GAP_TOL
    r0 = float(gen_uniforms(cfg, stream0, 1)[0])
    tok_o, dist0 = oracle.sample_first(temperature, top_p, r0)
    tok_g = ctx.sample_first(temperature, top_p, r0)
    emitted = [tok_o]
    decisions = 1
    if tok_g != tok_o:
        d = _interval_distance(dist0, tok_g, r0)
        slack = _cut_slack(oracle, pre.hidden[L, -1], dist0, temperature, top_p)
        assert d <= sample_tol + slack, f"first token gpu {tok_g} oracle {tok_o} r {r0} distance {d}"
        rep.flips += 1
        ctx.set_pending(tok_o)
    if (gE, gg) != (pre.next_E, pre.next_gamma):
        _resync(ctx, oracle, prompt, emitted, rep)
    E, gamma = (pre.next_E, pre.next_gamma) if schedule is None else schedule
    tau = pre.tau[E]
    while len(emitted) < n_tokens:
        # g: the draft length asked for (the cap, if dynamic); the uniform numbers are laid out by it
        g = min(cfg.d_max if dynamic else gamma, n_tokens - len(emitted) - 1)
        un = gen_uniforms(cfg, stream0 + 1 + rep.rounds, 2 * g + 1).tolist()
        diverged = None
        if dynamic:
            r = oracle.round_sample(E, g, temperature, top_p, un, keep_hidden=True, tau=tau)
            out, g_gpu, stopped = ctx.round_sample_dynamic(E, tau, g, temperature, top_p, un)
            st = ctx.stats()
            n_draft = min(g_gpu, r.gamma)
            for i, cf in enumerate(st["last_draft_conf"][:n_draft]):
                if st["last_draft"][:i] == r.draft_ids[:i]:
                    assert _close(cf, r.draft_conf[i], CONF_RTOL), ("draft confidence", i, cf, r.draft_conf[i])
            if (g_gpu, stopped) != (r.gamma, r.stopped_early) and st["last_draft"][:n_draft] == r.draft_ids[:n_draft]:
                assert n_draft < len(r.draft_conf) and _close(r.draft_conf[n_draft], tau, CONF_RTOL), (
                    f"round {rep.rounds + 1}: gpu drafted {g_gpu} (stopped {stopped}), oracle {r.gamma} "
                    f"(stopped {r.stopped_early}), confidences {r.draft_conf}, tau {tau}")
                diverged = ("stop", n_draft)
        else:
            r = oracle.round_sample(E, g, temperature, top_p, un, keep_hidden=True)
            out = ctx.round_sample(E, g, temperature, top_p, un)
            st = ctx.stats()
            n_draft = g
        rep.rounds += 1
        decisions += 2 * n_draft + 1
        # the drafts, in order; after a differing draft the two sides see different inputs
        same_rows = n_draft + 1
        for i in range(n_draft):
            if st["last_draft"][i] != r.draft_ids[i]:
                d = _interval_distance(r.q_dists[i], st["last_draft"][i], un[i])
                slack = _cut_slack(oracle, r.hidden[E, i], r.q_dists[i], temperature, top_p)
                assert d <= sample_tol + slack, (
                    f"round {rep.rounds} E={E} g={g} draft {i}: gpu {st['last_draft'][i]} oracle {r.draft_ids[i]} "
                    f"r {un[i]} distance {d} slack {slack}")
                diverged = ("draft", i)
                same_rows = i + 1
                break
        # greedy shadow tokens and hidden states of the rows with equal inputs
        flipped = False
        for l in range(1, L + 1):
            for i in range(same_rows):
                rep.compared_ids += 1
                if st["last_shadow"][l][i] != r.shadow[l][i]:
                    assert r.gaps[l][i] < GAP_TOL, ("shadow", rep.rounds, l, i, r.gaps[l][i])
                    flipped = True
                else:
                    assert _close(st["last_conf"][l][i], r.conf[l][i], CONF_RTOL)
            err = _rel_err(np.stack([ctx.hidden(l, i) for i in range(same_rows)]),
                           r.hidden[l, :same_rows].float().numpy())
            rep.max_hidden_err = max(rep.max_hidden_err, err)
            assert err <= HID_TOL, ("hidden", rep.rounds, l, err)
        if diverged is None:
            u_g = len(out) - 1
            gg = r.gamma      # drafts actually taken (equal on both sides here)
            if u_g != r.u:
                # the acceptance at the first position where the two sides differ
                k = min(u_g, r.u)
                x = r.draft_ids[k]
                ratio = float(r.p_dists[k][x]) / float(r.q_dists[k][x])
                slack = (_cut_slack(oracle, r.hidden[L, k], r.p_dists[k], temperature, top_p) +
                         _cut_slack(oracle, r.hidden[E, k], r.q_dists[k], temperature, top_p))
                in_p_cut = float(r.p_dists[k][x]) == 0.0 and slack > 0.0
                assert abs(un[g + k] - min(ratio, 1.0)) <= ratio_tol * max(ratio, 1e-3) + slack or in_p_cut, (
                    f"round {rep.rounds} E={E} g={g}: gpu accepted {u_g}, oracle {r.u}; at {k} r {un[g + k]} ratio {ratio}")
                diverged = ("accept", k)
            elif out[:r.u] != r.out_tokens[:r.u]:
                raise AssertionError(("accepted drafts differ", out, r.out_tokens))
            elif out[-1] != r.out_tokens[-1]:
                d = _interval_distance(r.last_dist, out[-1], un[2 * g])
                slack = _cut_slack(oracle, r.hidden[L, r.u], r.p_dists[r.u], temperature, top_p)
                if r.u < gg:
                    slack += _cut_slack(oracle, r.hidden[E, r.u], r.q_dists[r.u], temperature, top_p)
                    # the residual is renormalised by its own total: boundary shifts scale with 1 / total
                    total = float(torch.clamp(r.p_dists[r.u] - r.q_dists[r.u], min=0).sum())
                    tol = sample_tol / max(total, 1e-6)
                else:
                    tol = sample_tol
                assert d <= tol + slack, (
                    f"round {rep.rounds} E={E} g={g} last token: gpu {out[-1]} oracle {r.out_tokens[-1]} "
                    f"r {un[2 * g]} distance {d} tol {tol} slack {slack}")
                diverged = ("last", r.u)
        emitted.extend(r.out_tokens)
        if diverged is None and not flipped:
            assert out == r.out_tokens and st["last_u"] == r.u and st["last_n"] == r.n
            assert st["last_c"][1:] == r.c[1:]
            for l in range(1, L + 1):
                assert abs(st["alpha"][l] - r.alpha[l]) <= 1e-9
                assert _close(st["tau"][l], r.tau[l], CONF_RTOL)
            assert (st["next_E"], st["next_gamma"]) == (r.next_E, r.next_gamma)
            T, pend = ctx.state()
            assert T == oracle.T and pend == oracle.pending
        else:
            if diverged is not None:
                rep.flips += 1
                log(f"  sampled decision differs within tolerance: round {rep.rounds} {diverged}")
            _resync(ctx, oracle, prompt, emitted, rep)
        if schedule is None:
            E, gamma = r.next_E, r.next_gamma
        tau = r.tau[E]
    rep.tokens = emitted
    rep.decisions = decisions
    return rep


# ---- replay of stored oracle records (full-size shapes) ------------------------------------
# tests/golden/make_fullsize_records.py runs the oracle on the CPU ahead of time and stores what
# lockstep() compares round by round; here the library is driven through the same rounds and held
# to the same rules (exact ids / counts / selection outside near-ties, re-prefill + statistics
# import after a tolerated flip).  Hidden rows are stored for three layers of a few rounds.

def load_records(name):
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"fullsize_{name}.npz")
    z = np.load(path)
    rec = {k: z[k] for k in z.files}
    rec["meta"] = json.loads(str(z["meta"]))
    return rec


def _resync_records(ctx: DelContext, prompt, emitted, S_c, S_n, S_tcs, S_fcs, T, pending, rep):
    first, _, _ = ctx.prefill(list(prompt) + emitted[:-1])
    if first != emitted[-1]:
        ctx.set_pending(emitted[-1])
    ctx.set_stats(list(S_c), float(S_n), list(S_tcs), list(S_fcs))
    assert ctx.state() == (T, pending)
    rep.resyncs += 1


def lockstep_records(cfg, rec, ctx: DelContext, max_rounds=None, conf_rtol=None) -> ParityReport:
    """Drive the library through the rounds of a stored oracle run (DEL-selected (E, gamma)).
    conf_rtol: relative tolerance of confidences and of the sums and thresholds built from them.  A
    confidence is exp(z_top - logsumexp(z)), so its relative error is at most twice the largest absolute
    logit error; at the full-size shapes (d_model 4096-8192, logits of a few units, fp32 oracle) that is
    up to about 1e-2, so the default here is the 2e-2 the logits themselves are held to."""
    CONF_RTOL = HID_TOL if conf_rtol is None else conf_rtol
    rep = ParityReport()
    L = cfg.n_layers
    meta = rec["meta"]
    for k, v in meta["config"].items():        # the record was made for this very configuration
        assert getattr(cfg, k) == v, (k, getattr(cfg, k), v)
    prompt = rec["prompt"].tolist()
    from synthdata import gen_prompt
    assert prompt == gen_prompt(cfg).tolist()
    hid_layers = [int(x) for x in rec["hidden_layers"]]
    first, gE, gg = ctx.prefill(prompt)
    st = ctx.stats()
    w = int(rec["pre_window"])
    pre_first = int(rec["pre_first_token"])
    near = rec["pre_gaps"] < GAP_TOL
    if first != pre_first:
        assert float(rec["pre_first_gap"]) < GAP_TOL, f"first token {first} != {pre_first}"
        rep.flips += 1
    for l in range(1, L + 1):
        slack = int(np.sum(near[l] | near[L]))
        assert abs(st["last_c"][l] - int(rec["pre_c"][l])) <= slack, (l, st["last_c"][l], int(rec["pre_c"][l]), slack)
    for k, l in enumerate(hid_layers):
        err = _rel_err(ctx.hidden(l, ctx.last_rows() - 1), rec["pre_hidden"][k])
        rep.max_hidden_err = max(rep.max_hidden_err, err)
        assert err <= HID_TOL, ("prefill hidden", l, err)
    emitted = [pre_first]
    exact = first == pre_first and all(st["last_c"][l] == int(rec["pre_c"][l]) for l in range(1, L + 1))
    if exact:
        assert (gE, gg) == (int(rec["pre_next_E"]), int(rec["pre_next_gamma"]))
        for l in range(1, L + 1):
            assert abs(st["alpha"][l] - rec["pre_alpha"][l]) < 1e-12
            assert _close(st["tau"][l], rec["pre_tau"][l], CONF_RTOL), ("prefill tau", l)
    else:
        _resync_records(ctx, prompt, emitted, rec["pre_c"].astype(np.float64), float(w), rec["pre_tcs"],
                        rec["pre_fcs"], len(prompt), pre_first, rep)
    R = len(rec["E"]) if max_rounds is None else min(max_rounds, len(rec["E"]))
    hid_at = {int(r): k for k, r in enumerate(rec["hidden_rounds"])}
    for r in range(R):
        E, g, u = int(rec["E"][r]), int(rec["gamma"][r]), int(rec["u"][r])
        assert ctx.state()[0] == int(rec["T_before"][r])
        out = ctx.round(E, g)
        st = ctx.stats()
        rep.rounds += 1
        drafts = rec["draft_ids"][r, :g].tolist()
        target = rec["target_ids"][r, :g + 1].tolist()
        same_rows = g + 1
        for i in range(g):
            if st["last_draft"][i] != drafts[i]:
                same_rows = i + 1
                break
        flipped = False
        for l in range(1, L + 1):
            for i in range(same_rows):
                rep.compared_ids += 1
                want = int(rec["shadow"][r, l, i])
                if st["last_shadow"][l][i] == want:
                    assert _close(st["last_conf"][l][i], rec["conf"][r, l, i], CONF_RTOL), (
                        "confidence", r, l, i, st["last_conf"][l][i], rec["conf"][r, l, i])
                else:
                    assert rec["gaps"][r, l, i] < GAP_TOL, (
                        f"round {r + 1} E={E} g={g} layer {l} row {i}: gpu {st['last_shadow'][l][i]} "
                        f"oracle {want} gap {rec['gaps'][r, l, i]}")
                    rep.flips += 1
                    flipped = True
        if r in hid_at:
            for k, l in enumerate(hid_layers):
                want = rec["hidden"][hid_at[r], k, :same_rows]
                got = np.stack([ctx.hidden(l, i) for i in range(same_rows)])
                err = _rel_err(got, want)
                rep.max_hidden_err = max(rep.max_hidden_err, err)
                assert err <= HID_TOL, ("hidden", r, l, err)
        out_want = target[:u + 1]
        emitted.extend(out_want)
        T_after, pending = int(rec["T_before"][r]) + u + 1, out_want[-1]
        if not flipped and same_rows == g + 1:
            assert out == out_want, (out, out_want)
            assert st["last_u"] == u and st["last_n"] == int(rec["n"][r])
            assert st["last_c"][1:] == rec["c"][r, 1:].tolist()
            assert st["last_draft"][:g] == drafts
            for l in range(1, L + 1):
                assert abs(st["S_c"][l] - rec["S_c"][r, l]) <= 1e-9 * max(1.0, rec["S_c"][r, l])
                assert abs(st["alpha"][l] - rec["alpha"][r, l]) <= 1e-9
                assert _close(st["S_tcs"][l], rec["S_tcs"][r, l], CONF_RTOL)
                assert _close(st["S_fcs"][l], rec["S_fcs"][r, l], CONF_RTOL)
                assert _close(st["tau"][l], rec["tau"][r, l], CONF_RTOL), ("tau", r, l)
            assert abs(st["S_n"] - rec["S_n"][r]) <= 1e-9 * rec["S_n"][r]
            assert (st["next_E"], st["next_gamma"]) == (int(rec["next_E"][r]), int(rec["next_gamma"][r]))
            assert ctx.state() == (T_after, pending)
        else:
            _resync_records(ctx, prompt, emitted, rec["S_c"][r], rec["S_n"][r], rec["S_tcs"][r], rec["S_fcs"][r],
                            T_after, pending, rep)
    rep.tokens = emitted
    return rep
