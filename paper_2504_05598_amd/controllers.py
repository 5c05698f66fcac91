"""Round controllers on top of the C ABI: who picks (E, gamma) for the next round.

* "del"       DEL's Token-per-Layer arg-max picks E and gamma (Sections 4.1-4.3; the paper's DEL-E variant)
* "del_full"  DEL picks E, the draft loop stops on the dynamic threshold tau_E (Section 4.4; Algorithm 1)
* "ls"        static exit layer and speculation length (the LayerSkip baseline, Section 5.1)
* "fs"        static exit layer, finite-state speculation length: +1 after a round in which every
              draft was accepted, -1 otherwise, kept in [1, d_max] (Section 5.1, Appendix B.3)
* "vanilla"   gamma = 0: one auto-regressive step per round

Host logic only; every round still runs through del_round / del_round_dynamic.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def fs_next_gamma(gamma: int, accepted_all: bool, d_max: int) -> int:
    """Finite-state controller: lengthen after a fully accepted round, shorten otherwise."""
    return min(d_max, gamma + 1) if accepted_all else max(1, gamma - 1)


def generate(ctx, prompt: Sequence[int], n_tokens: int, controller: str = "del", E: int = 1, gamma: int = 1,
             sampling=None) -> Tuple[List[int], List[Tuple[int, int, int]]]:
    """Generate n_tokens (the first comes from the prefill).  Returns the tokens and, per round,
    (E, tokens drafted, tokens emitted).
    sampling: None for greedy decoding, or (temperature, top_p, uniforms) for speculative sampling
    (Section 2), where uniforms(k, count) returns the `count` numbers in [0, 1) of draw k: k = 0 is
    the first token, k = r + 1 is round r (2 * gamma + 1 numbers: drafts, acceptances, last token)."""
    cfg = ctx.cfg
    first, dE, dg = ctx.prefill(list(prompt))
    if controller in ("del", "del_full"):
        E, gamma = dE, dg
    elif controller == "vanilla":
        E, gamma = 1, 0
    elif controller not in ("ls", "fs"):
        raise ValueError(controller)
    if sampling is not None:
        temperature, top_p, uniforms = sampling
        first = ctx.sample_first(temperature, top_p, float(uniforms(0, 1)[0]))
    toks = [first]
    log = []
    while len(toks) < n_tokens:
        room = n_tokens - len(toks) - 1
        if controller == "del_full":
            st = ctx.stats()
            E = st["next_E"]
            cap = min(cfg.d_max, room)
            if sampling is not None:
                out, g, _ = ctx.round_sample_dynamic(E, st["tau"][E], cap, temperature, top_p,
                                                     [float(x) for x in uniforms(len(log) + 1, 2 * cap + 1)])
            else:
                out, g, _ = ctx.round_dynamic(E, st["tau"][E], cap)
        else:
            g = min(gamma, room)
            if sampling is not None:
                out = ctx.round_sample(E, g, temperature, top_p, [float(x) for x in uniforms(len(log) + 1, 2 * g + 1)])
            else:
                out = ctx.round(E, g)
        toks.extend(out)
        log.append((E, g, len(out)))
        if controller == "del":
            st = ctx.stats()
            E, gamma = st["next_E"], st["next_gamma"]
        elif controller == "fs":
            gamma = fs_next_gamma(gamma, len(out) == g + 1, cfg.d_max)
    return toks, log


def empirical_tpl(log: Sequence[Tuple[int, int, int]], n_layers: int) -> float:
    """eTPL = generated tokens / loaded layers, gamma*E + L layers per round (Section 4.1, Appendix B.4)."""
    return sum(n for _, _, n in log) / sum(g * E + n_layers for E, g, _ in log)
