#!/usr/bin/env python3
"""Benchmark of the greedy self-speculative decode round with DEL on one MI355X.

A "step" is one round of the whole hot path (draft, verify, shadow head, statistics and
selection of the next (E, gamma)) on the Llama-2-7B-shaped synthetic model after a 1024-token
prefill.  Prints ONE JSON line.  `value` is accepted tokens per second with all inputs resident
in HBM; `roofline` is the dominant weight-streaming kernel against the HBM peak; `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def round_bytes(cfg, E, gamma, T):
    """Algorithmic HBM bytes of one round at KV length T (what the method must move):
    (gamma*E + L) layer loads, gamma draft heads + 1 shadow/verify head, KV rows read by every
    layer pass, KV rows written, hidden buffer written and read once."""
    L = cfg.n_layers
    es = 2 if cfg.weight_dtype == "bf16" else 4
    b_layer = cfg.layer_weight_bytes()
    b_head = cfg.head_weight_bytes()
    kv_row = 2 * cfg.n_kv_heads * cfg.head_dim * es           # K and V of one position, one layer
    kv_read = 0
    for i in range(gamma + 1):                                # draft steps and the last-token pass
        kv_read += E * (T + i + 1) * kv_row
    kv_read += (L - E) * (T + gamma + 1) * kv_row             # verify reads the cache once per layer
    kv_write = (gamma + 1) * L * kv_row
    hidden = 2 * L * (gamma + 1) * cfg.d_model * 4
    return (gamma * E + L) * b_layer + (gamma + 1) * b_head + kv_read + kv_write + hidden


def segment_bytes(cfg, E, gamma, T):
    """Algorithmic HBM bytes of a round's segments at KV length T: (draft layer passes incl. the last-token
    pass, draft heads, verify layer passes, shadow/verify head).  Same accounting as round_bytes."""
    L = cfg.n_layers
    es = 2 if cfg.weight_dtype == "bf16" else 4
    b_layer, b_head = cfg.layer_weight_bytes(), cfg.head_weight_bytes()
    kv_row = 2 * cfg.n_kv_heads * cfg.head_dim * es
    draft = sum(E * (b_layer + (T + i + 1) * kv_row + kv_row) for i in range(gamma + 1))
    heads = gamma * b_head
    m = gamma + 1
    verify = (L - E) * (b_layer + (T + m) * kv_row + m * kv_row)
    shadow = b_head + 2 * L * m * cfg.d_model * 4
    return draft, heads, verify, shadow


def library_source_hash():
    """sha256 over the HIP sources the library is built from (what a stored profile is valid for)."""
    import hashlib
    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2504_05598_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(root)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(root, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(cfg_name, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 PMC summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by a plain copy kernel of known size).  The summary names the sources it
    was measured on (library_source_hash); None if there is no summary or the library has changed since."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        f"bench_{cfg_name}_hbm_traffic.txt")
    value, valid = None, False
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                value = int(float(parts[2]))
            if len(parts) == 2 and parts[0] == "library_source_hash":
                valid = parts[1] == library_source_hash()
    except OSError:
        pass
    return value if valid else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="llama7b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma", action="store_true")
    ap.add_argument("--micro", action="store_true",
                    help="only the GEMV decomposition table (del_bench_gemv_parts) for this config's matrix shapes")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (batch-1 decode on a single MI355X); "
                 "use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from paper_2504_05598_amd.binding import DelContext
    from synthdata import gen_prompt, gen_tensor, get_config, iter_tensor_specs

    cfg = get_config(args.config)
    if args.micro:
        return micro(cfg, DelContext)
    K, W = args.steps, args.warmup
    max_context = cfg.prompt_len + (2 * K + W + 8) * (cfg.d_max + 1) + cfg.d_max + 1
    want_cpu = not args.no_cpu_baseline
    t0 = time.time()
    ctx = DelContext(cfg, use_mfma=not args.no_mfma, max_context=max_context)
    host = {} if want_cpu else None
    for layer, kind in iter_tensor_specs(cfg):
        t = gen_tensor(cfg, layer, kind, device="cuda")
        ctx.load_tensor(layer, kind, t)
        if want_cpu:
            host[(layer, kind)] = t.cpu()
        del t
    torch.cuda.synchronize()
    log(f"[bench] model {cfg.name} generated and loaded in {time.time() - t0:.1f}s")
    prompt = gen_prompt(cfg).tolist()

    def run(n_rounds, collect=None):
        """n_rounds DEL-driven rounds from the current state; returns tokens emitted."""
        st = ctx.stats()
        E, g = st["next_E"], st["next_gamma"]
        tokens = 0
        for _ in range(n_rounds):
            T = ctx.state()[0]
            out = ctx.round(E, g)
            tokens += len(out)
            if collect is not None:
                d, v, s = ctx.timings()
                collect.append((E, g, T, len(out), d, v, s))
            st = ctx.stats()
            E, g = st["next_E"], st["next_gamma"]
        return tokens

    # ---- timed region: prefill (untimed), W warm-up rounds, exactly K timed rounds
    t0 = time.time()
    first, E0, g0 = ctx.prefill(prompt)
    torch.cuda.synchronize()
    prefill_s = time.time() - t0
    run(W)
    torch.cuda.synchronize()
    timed = []
    t0 = time.perf_counter()
    tokens = run(K, timed)      # per round: two host-side reads of state the library already holds
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    value = tokens / dt

    # ---- same K rounds again with per-round splits and per-kernel HIP-event timing
    ctx.prefill(prompt)
    run(W)
    ctx.profile_enable(True)
    run(K, [])
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    by_kernel = {}
    for e in prof:
        k = by_kernel.setdefault(e["kernel"], {"launches": 0, "total_ms": 0.0, "bytes": 0})
        k["launches"] += e["launches"]; k["total_ms"] += e["total_ms"]
        k["bytes"] += e["weight_bytes"] * e["launches"]
    # dominant kernel among the single-shape weight-streaming classes
    dom_name, dom = max(((n, k) for n, k in by_kernel.items() if ",1>" not in n and "<1>" not in n),
                        key=lambda kv: kv[1]["total_ms"])
    dom_bytes = dom["bytes"] / dom["launches"]
    dom_us = 1e3 * dom["total_ms"] / dom["launches"]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    # round split and segment fractions from the TIMED run's own per-round event times
    recs = timed
    alg_bytes = sum(round_bytes(cfg, E, g, T) for (E, g, T, n, d, v, s) in recs)
    seg = [sum(r[i] for r in recs) / len(recs) for i in (4, 5, 6)]
    round_ms_prof = sum(seg)
    layers_loaded = sum(g * E + cfg.n_layers for (E, g, T, n, d, v, s) in recs)
    etpl = sum(r[3] for r in recs) / layers_loaded
    sb = [segment_bytes(cfg, E, g, T) for (E, g, T, n, d, v, s) in recs]
    draft_seg_bytes = sum(b[0] + b[1] for b in sb)
    verify_seg_bytes = sum(b[2] for b in sb)
    shadow_seg_bytes = sum(b[3] for b in sb)
    draft_s = sum(r[4] for r in recs) * 1e-3
    verify_s = sum(r[5] for r in recs) * 1e-3
    shadow_s = sum(r[6] for r in recs) * 1e-3
    verify_layer_passes = sum(cfg.n_layers - E for (E, g, T, n, d, v, s) in recs)

    # ---- vanilla (gamma = 0) rounds with the same library, for the speed-up figure
    ctx.prefill(prompt)
    for _ in range(2):
        ctx.round(1, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    nv = 8
    for _ in range(nv):
        ctx.round(1, 0)
    torch.cuda.synchronize()
    vanilla_tps = nv / (time.perf_counter() - t0)
    # ---- the draft layer pass on its own: a round with E = L and gamma = 0 is L one-row layer passes in its
    #      draft segment (no head there) and nothing in its verify segment
    ctx.prefill(prompt)
    run(W)
    lp = []
    for _ in range(8):
        T = ctx.state()[0]
        ctx.round(cfg.n_layers, 0)
        lp.append((T, ctx.timings()[0]))
    # ---- static (E, gamma) schedules around DEL's choice (the LayerSkip baseline of Section 5.1)
    meanE = sum(r[0] for r in timed) / len(timed)
    statics = []
    for Es in sorted({max(1, int(round(meanE)) + dE) for dE in (-4, -2, 0, 2)}):
        for gs in sorted({min(cfg.d_max, g) for g in (2, 3, 4, 6)}):
            if Es >= cfg.n_layers:
                continue
            ctx.prefill(prompt)
            for _ in range(2):
                ctx.round(Es, gs)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            nt = sum(len(ctx.round(Es, gs)) for _ in range(12))
            torch.cuda.synchronize()
            statics.append((nt / (time.perf_counter() - t0), Es, gs))
    best_static = max(statics) if statics else None
    # ---- the same K rounds with dynamic draft-exiting (Section 4.4): E and tau_E from the statistics
    ctx.prefill(prompt)

    def run_dynamic(n_rounds):
        tokens, drafted = 0, 0
        st = ctx.stats()
        for _ in range(n_rounds):
            E = st["next_E"]
            out, g, _ = ctx.round_dynamic(E, st["tau"][E], cfg.d_max)
            tokens += len(out); drafted += g
            st = ctx.stats()
        return tokens, drafted
    run_dynamic(W)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    dyn_tokens, dyn_drafted = run_dynamic(K)
    torch.cuda.synchronize()
    dyn_tps = dyn_tokens / (time.perf_counter() - t0)
    # ---- the same K rounds with speculative sampling (Section 2; temperature 0.6, top_p 0.95 as in the
    #      paper's sampling runs), DEL-selected (E, gamma); and its auto-regressive counterpart (gamma = 0)
    from synthdata import gen_uniforms
    ctx.prefill(prompt)
    ctx.sample_first(0.6, 0.95, 0.5)

    def run_sampled(n_rounds, stream0, fixed=None):
        tokens = 0
        st = ctx.stats()
        for k in range(n_rounds):
            E, g = fixed if fixed else (st["next_E"], st["next_gamma"])
            tokens += len(ctx.round_sample(E, g, 0.6, 0.95, gen_uniforms(cfg, stream0 + k, 2 * g + 1).tolist()))
            st = ctx.stats()
        return tokens
    run_sampled(W, 10000)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    smp_tokens = run_sampled(K, 20000)
    torch.cuda.synchronize()
    smp_tps = smp_tokens / (time.perf_counter() - t0)
    ctx.prefill(prompt)
    ctx.sample_first(0.6, 0.95, 0.5)
    run_sampled(2, 30000, fixed=(1, 0))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_sampled(8, 40000, fixed=(1, 0))
    torch.cuda.synchronize()
    smp_vanilla_tps = 8 / (time.perf_counter() - t0)
    # ---- the prefill on its own (not part of the metric): steady-state time, and the wide GEMMs'
    #      matrix-core rate from their own start/stop timestamps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.prefill(prompt)
    torch.cuda.synchronize()
    prefill_steady_s = time.perf_counter() - t0
    ctx.profile_enable(True)
    ctx.prefill(prompt)
    pprof = [e for e in ctx.profile_read() if e["kernel"].startswith("gemm_wide_k")]
    ctx.profile_enable(False)
    prefill_info = {"tokens": len(prompt), "ms": round(1e3 * prefill_steady_s, 2),
                    "tokens_per_s": round(len(prompt) / prefill_steady_s, 1)}
    if pprof:
        # multiply-adds of a launch = weight elements x token rows; the activations enter as a bf16
        # high and low part, so the matrix cores execute twice that
        pw = max(pprof, key=lambda e: e["total_ms"])     # one class per (epilogue, matrix size)
        macs = sum(e["weight_bytes"] / 2 * e["rows"] * e["launches"] for e in pprof)
        ms = sum(e["total_ms"] for e in pprof)
        pw_tf = 2 * 2 * (pw["weight_bytes"] / 2) * pw["rows"] * pw["launches"] / (pw["total_ms"] * 1e-3) / 1e12
        prefill_info["mfma"] = {"bound": "mfma", "kernel": pw["kernel"], "rows": pw["rows"],
                                "achieved": round(pw_tf, 1), "peak": 2500.0, "unit": "TFLOP/s",
                                "frac": round(pw_tf / 2500.0, 4),
                                "model_TFLOPs": round(pw_tf / 2, 1), "frac_model_flops": round(pw_tf / 2 / 2500.0, 4),
                                "all_wide_gemms_TFLOPs": round(4 * macs / (ms * 1e-3) / 1e12, 1),
                                "all_wide_gemms_ms": round(ms, 2),
                                "note": "bf16 matrix instructions executed (activations as high + low part: "
                                        "twice the model's multiply-adds)"}
    stream_gbs = ctx.stream_read_gbps(min(4 << 30, cfg.layer_weight_bytes() * cfg.n_layers), 10)
    copy_gbs = ctx.stream_copy_gbps(1 << 30, 5)     # also the known-size kernel for counter calibration

    # one-row layer pass: time and algorithmic bytes (a layer's weights + its KV rows read and one row written)
    es = 2 if cfg.weight_dtype == "bf16" else 4
    kv_row = 2 * cfg.n_kv_heads * cfg.head_dim * es
    lp_us = 1e3 * sum(t for _, t in lp) / len(lp) / cfg.n_layers
    lp_T = int(sum(T for T, _ in lp) / len(lp))
    lp_bytes = cfg.layer_weight_bytes() + (lp_T + 2) * kv_row
    # the shadow-head GEMM (Section 4.2): rows, HBM and matrix-core fractions; model flops = 2 * rows * d * V, the
    # matrix cores execute twice that (activations enter as a bf16 high and low part)
    shadow_info = None
    hk = [e for e in prof if e["kernel"] in ("head_gemm_k", "head_gemm4_k")]
    if hk:
        h_ms = sum(e["total_ms"] for e in hk)
        h_n = sum(e["launches"] for e in hk)
        h_rows = sum(e["rows"] * e["launches"] for e in hk) / h_n
        h_bytes = sum(e["weight_bytes"] * e["launches"] for e in hk)
        h_flops = sum(2.0 * e["rows"] * cfg.d_model * cfg.vocab * e["launches"] for e in hk)
        blocked = hk[0]["kernel"] == "head_gemm4_k"
        shadow_info = {"kernel": hk[0]["kernel"], "launches": h_n, "mean_rows": round(h_rows, 1),
                       "avg_us": round(1e3 * h_ms / h_n, 2),
                       "hbm_frac": round(h_bytes / (h_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "mfma_frac_model_flops": round(h_flops / (h_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                       "mfma_frac_executed": round(2 * h_flops / (h_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                       "hi_lo_factor": 2,
                       "note": f"weights streamed once per {8 if blocked else 16} blocks of 16 token rows (hbm_frac counts every "
                               "pass); executed = model flops x 2"}

    result = {
        "metric": "accepted tokens/sec at batch 1 (Llama-2-7B shape)",
        "value": round(value, 2),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(1e3 * dt / K, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.weight_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: L={cfg.n_layers} d={cfg.d_model} ffn={cfg.d_ffn} "
                               f"vocab={cfg.vocab}, batch 1, {cfg.prompt_len}-token prompt, DEL-selected "
                               f"(E, gamma<={cfg.d_max}), greedy",
                   "tokens_in_timed_region": tokens, "prefill_s": round(prefill_s, 3)},
        "roofline": {
            "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(cfg.name, dom_name),
            "kernel": dom_name, "bytes_per_launch": int(dom_bytes), "avg_launch_us": round(dom_us, 2),
            "launches": dom["launches"],
        },
        "round": {
            "draft_ms": round(seg[0], 4), "verify_ms": round(seg[1], 4), "shadow_ms": round(seg[2], 4),
            "algorithmic_GB_per_round": round(alg_bytes / len(recs) / 1e9, 3),
            "hbm_frac_whole_round": round(alg_bytes / (round_ms_prof * 1e-3 * len(recs)) / 1e9 / HBM_PEAK_GBS, 4),
            "eTPL": round(etpl, 5), "tokens_per_round": round(sum(r[3] for r in recs) / len(recs), 3),
            "mean_E": round(sum(r[0] for r in recs) / len(recs), 2),
            "mean_gamma": round(sum(r[1] for r in recs) / len(recs), 2),
            "vanilla_tokens_per_s": round(vanilla_tps, 2),
            "speedup_over_vanilla": round(value / vanilla_tps, 3),
            "with_draft_exiting_tokens_per_s": round(dyn_tps, 2),
            "with_draft_exiting_mean_gamma": round(dyn_drafted / K, 2),
            "sampling_tokens_per_s": round(smp_tps, 2),
            "sampling_tokens_per_round": round(smp_tokens / K, 3),
            "sampling_autoregressive_tokens_per_s": round(smp_vanilla_tps, 2),
            "stream_read_GBs": round(stream_gbs, 1), "stream_copy_GBs": round(copy_gbs, 1),
            "paper_speedup_over_autoregressive": "2.16-2.62x on A100-40G / 2xH100-PCIe (context only)",
        },
        "segments": {
            "note": "from the timed run's own per-round event times; algorithmic bytes / time / 8 TB/s "
                    "(and / the measured stream-read ceiling); draft_segment includes the gamma draft heads",
            "draft_segment_hbm_frac": round(draft_seg_bytes / draft_s / 1e9 / HBM_PEAK_GBS, 4),
            "verify_layers_hbm_frac": round(verify_seg_bytes / verify_s / 1e9 / HBM_PEAK_GBS, 4) if verify_s > 0 else None,
            "verify_layer_pass_us": round(1e6 * verify_s / max(1, verify_layer_passes), 2),
            "shadow_segment_hbm_frac": round(shadow_seg_bytes / shadow_s / 1e9 / HBM_PEAK_GBS, 4),
            "draft_layer_pass_us": round(lp_us, 2), "draft_layer_pass_T": lp_T,
            "draft_layers_hbm_frac": round(lp_bytes / (lp_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
            "draft_layers_frac_of_stream_ceiling": round(lp_bytes / (lp_us * 1e-6) / 1e9 / stream_gbs, 4),
            "verify_layers_frac_of_stream_ceiling": round(verify_seg_bytes / verify_s / 1e9 / stream_gbs, 4) if verify_s > 0 else None,
            "draft_layer_pass_source": "8 rounds with E = L, gamma = 0: their draft segment is L one-row layer passes, no head",
        },
        "shadow_head": shadow_info,
        "best_static_schedule": ({"E": best_static[1], "gamma": best_static[2], "tokens_per_s": round(best_static[0], 2),
                                  "del_tokens_per_s": round(value, 2), "tried": len(statics),
                                  "note": "static (E, gamma) around DEL's mean exit layer, 12 rounds each; the paper's cost "
                                          "model (Section 4.1) ignores the LM head, 0.65 of a layer per draft step here"}
                                 if best_static else None),
        "prefill": prefill_info,
        "kernels": {n: {"launches": k["launches"], "avg_us": round(1e3 * k["total_ms"] / k["launches"], 2),
                        "GBs": round(k["bytes"] / (k["total_ms"] * 1e-3) / 1e9, 1)}
                    for n, k in sorted(by_kernel.items())},
    }
    ctx.close()
    torch.cuda.empty_cache()

    if want_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, host, prompt)
    print(json.dumps(result), flush=True)


def micro(cfg, DelContext):
    """Where a one-row GEMV launch spends its time beyond the weight stream: the library's GEMV with parts
    switched off (del_bench_gemv_parts), at this config's matrix shapes and launch geometry, back-to-back
    launches over different parts of the (zero-filled) weight arena.  Prints a table, not the bench line."""
    ctx = DelContext(cfg)
    d, f, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    qkv_rows = (cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim
    up16 = lambda n: (n + 15) // 16
    up8 = lambda n: (n + 7) // 8
    shapes = [("QKV", up16(qkv_rows), d // 32), ("O", up16(d), cfg.n_q_heads * cfg.head_dim // 32),
              ("gate/up", up8(f), d // 32), ("down", up16(d), (f + 31) // 32), ("head", up16(V), d // 32)]
    cols = [("tile loads only", 0), ("+ decode/FMA (constant row)", 2), ("+ row staged via LDS", 3),
            ("loads + FMA + reduce/store", 6), ("whole kernel", 7)]
    ceiling = ctx.stream_read_gbps(min(4 << 30, cfg.layer_weight_bytes() * cfg.n_layers), 10)
    print(f"# del_bench_gemv_parts, {cfg.name}: microseconds per launch (200 back-to-back launches, rotating matrices)")
    print(f"# streaming read of the arena: {ceiling:.0f} GB/s; ideal = tile bytes / that rate")
    print(f"{'matrix':8s} {'blocks':>6s} {'ktiles':>6s} {'waves':>5s} {'MB':>7s} {'ideal':>7s} " + " ".join(f"{c[0]:>28s}" for c in cols))
    for name, nb, kt in shapes:
        if kt > 480:
            print(f"{name:8s} k tiles {kt} beyond the measurement kernel's limit")
            continue
        waves = 8 if nb * 8 >= 2 * 3072 else 16   # the library's own choice of waves per row block
        mb = nb * kt * 1024
        row = [ctx.gemv_parts_us(nb, kt, waves, parts) for _, parts in cols]
        print(f"{name:8s} {nb:6d} {kt:6d} {waves:5d} {mb / 1e6:7.1f} {mb / ceiling / 1e3:7.2f} " + " ".join(f"{v:28.2f}" for v in row))
    # issue rate of the two bf16 matrix instructions (del_bench_mfma_rate): one wave per SIMD, independent accumulators,
    # no memory traffic; TFLOP/s = 1024 SIMDs x flops per instruction / time per instruction
    print("# del_bench_mfma_rate: ns per instruction and SIMD, TFLOP/s over 256 CUs x 4 SIMDs (dense bf16 peak 2500)")
    for shape, label, flops, accs in ((0, "v_mfma_f32_16x16x32_bf16", 16384, (2, 4, 8, 16)), (1, "v_mfma_f32_32x32x16_bf16", 32768, (1, 2, 4))):
        for n_acc in accs:
            ns = min(ctx.mfma_rate_ns(shape, n_acc) for _ in range(3))
            print(f"{label:26s} {n_acc:2d} accumulators {ns:7.2f} ns {1024 * flops / ns / 1e3:8.1f} TFLOP/s")
    ctx.close()


def cpu_baseline(cfg, host, prompt):
    """The oracle as it stands, timed on a bounded sample: prefill on the first 64 prompt tokens
    (untimed), then DEL-driven rounds until ~20 s of CPU time have passed (at least 2 rounds)."""
    import torch
    from oracle.del_oracle import Oracle
    n_prompt = min(64, len(prompt))
    oracle = Oracle(cfg, host, dtype=torch.float32, max_context=n_prompt + 40 * (cfg.d_max + 1))
    t0 = time.time()
    pre = oracle.prefill(prompt[:n_prompt])
    log(f"[bench] oracle prefill({n_prompt}) {time.time() - t0:.1f}s")
    E, g = pre.next_E, pre.next_gamma
    tokens, rounds = 0, 0
    t0 = time.perf_counter()
    while rounds < 2 or (time.perf_counter() - t0 < 20.0 and rounds < 30):
        r = oracle.round(E, g)
        tokens += len(r.out_tokens)
        rounds += 1
        E, g = r.next_E, r.next_gamma
    dt = time.perf_counter() - t0
    return {"value": round(tokens / dt, 3), "unit": "tokens/s", "cores": torch.get_num_threads(),
            "kind": "oracle",
            "sample": f"same weights; prefill on the first {n_prompt} prompt tokens (untimed), then "
                      f"{rounds} DEL-driven rounds ({tokens} tokens) in {dt:.1f}s, fp32"}


if __name__ == "__main__":
    main()
