"""Synthetic (E, gamma) grid sweep on one GPU: eTPL, tokens/s and ms per round of static schedules
next to DEL, and a check of the paper's cost model (time of a round ~ gamma*E + L loaded layers,
Section 4.1) against measured milliseconds.

    python -m paper_2504_05598_amd.sweep --config llama7b --tokens 96
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="llama7b")
    ap.add_argument("--tokens", type=int, default=96)
    ap.add_argument("--exits", default="")
    ap.add_argument("--gammas", default="")
    args = ap.parse_args()
    import torch
    from synthdata import gen_prompt, gen_tensor, get_config, iter_tensor_specs
    from .binding import DelContext
    from .controllers import empirical_tpl, generate

    cfg = get_config(args.config)
    L = cfg.n_layers
    exits = [int(x) for x in args.exits.split(",")] if args.exits else sorted({1, 2, max(1, L // 8), L // 4, (3 * L) // 8, L // 2})
    gammas = [int(x) for x in args.gammas.split(",")] if args.gammas else [1, 2, 4, min(6, cfg.d_max), cfg.d_max]
    ctx = DelContext(cfg, max_context=cfg.prompt_len + args.tokens + cfg.d_max + 2)
    for layer, kind in iter_tensor_specs(cfg):
        ctx.load_tensor(layer, kind, gen_tensor(cfg, layer, kind, device="cuda"))
    prompt = gen_prompt(cfg).tolist()

    def timed(controller, **kw):
        generate(ctx, prompt, 8, controller, **kw)            # warm-up
        torch.cuda.synchronize()
        ctx.prefill(prompt)                                   # prefill is not part of the decode time
        t0 = time.perf_counter()
        toks, log = generate(ctx, prompt, args.tokens, controller, **kw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # subtract the prefill that generate() runs
        t1 = time.perf_counter(); ctx.prefill(prompt); torch.cuda.synchronize(); pre = time.perf_counter() - t1
        dt -= pre
        return {"controller": controller, **kw, "rounds": len(log), "tokens_per_s": (args.tokens - 1) / dt,
                "ms_per_round": 1e3 * dt / len(log), "eTPL": empirical_tpl(log, L),
                "tokens_per_round": (args.tokens - 1) / len(log),
                "layers_per_round": sum(g * E + L for E, g, _ in log) / len(log),
                "drafts_per_round": sum(g for _, g, _ in log) / len(log)}

    rows = [timed("vanilla"), timed("del"), timed("del_full")]
    for E in exits:
        for g in gammas:
            rows.append(timed("ls", E=E, gamma=g))
    rows.append(timed("fs", E=exits[len(exits) // 2], gamma=min(4, cfg.d_max)))
    # cost model: ms_per_round ~ a * loaded layers + b * (drafts + 1) LM-head passes
    ls = [r for r in rows if r["controller"] in ("ls", "vanilla")]
    A = np.array([[r["layers_per_round"], r["drafts_per_round"] + 1.0] for r in ls])
    y = np.array([r["ms_per_round"] for r in ls])
    coef, res, _, _ = np.linalg.lstsq(A, y, rcond=None)
    pred = A @ coef
    fit = {"ms_per_loaded_layer": float(coef[0]), "ms_per_head_pass": float(coef[1]),
           "max_rel_error": float(np.max(np.abs(pred - y) / y)),
           "layers_only_max_rel_error": float(np.max(np.abs(A[:, 0] * (y @ A[:, 0]) / (A[:, 0] @ A[:, 0]) - y) / y))}
    for r in rows:
        print(json.dumps({k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}))
    print(json.dumps({"cost_model_fit": fit}))


if __name__ == "__main__":
    main()
