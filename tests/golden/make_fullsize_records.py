"""Writes tests/golden/fullsize_<config>.npz: the CPU oracle's per-round records of a DEL-driven
greedy self-speculative generation (Algorithm 1 without the confidence break) at a full-size shape.

Imports only oracle/ and synthdata/ and runs on the CPU; nothing here comes from the HIP path.
The GPU tests replay these records in lock-step (tests/test_gpu_fullsize_records.py).

    python tests/golden/make_fullsize_records.py --config llama7b            # whole generation
    python tests/golden/make_fullsize_records.py --config llama70b --max-rounds 8

Weights are regenerated tensor by tensor with the shared seeded generator (its C fast path) and held
as exactly widened fp32 (or as bf16, widened at each use) for as many of the lowest layers as fit
`--resident-gb`; the other layers are regenerated whenever they are used, so the 70B shape fits a
64 GB host.  The oracle itself runs unchanged, in fp32 (the full-size precision the parity tests use).

Record layout (one npz per config), R rounds, L layers, D = d_max, w = prefill window:
  meta (json), prompt [P]
  pre_first_token, pre_first_gap, pre_window, pre_shadow [L+1, w], pre_gaps, pre_conf, pre_c [L+1],
  pre_alpha, pre_tau, pre_tcs, pre_fcs [L+1], pre_next_E, pre_next_gamma, pre_hidden [3, d] (last prompt position)
  E, gamma, T_before, u, n, next_E, next_gamma [R]; draft_ids [R, D], target_ids [R, D+1] (-1 padded)
  shadow, gaps, conf [R, L+1, D+1]; c, alpha, S_c, S_tcs, S_fcs, tau [R, L+1]; S_n [R]
  hidden_layers [3], hidden_rounds [H], hidden [H, 3, D+1, d]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle.del_oracle import Oracle                     # noqa: E402
from synthdata import gen_prompt, get_config             # noqa: E402
from synthdata import fastgen                            # noqa: E402
from synthdata.generator import LAYER_KINDS, tensor_shape  # noqa: E402


class LazyWeights:
    """(layer, kind) -> tensor.  Global tensors and the lowest layers that fit the budget stay in
    memory (fp32: widened once; or bf16: widened by the oracle at each use); the rest is regenerated
    at every access.  Values are the generator's, unchanged."""

    def __init__(self, cfg, resident_bytes: float, store_fp32: bool):
        self.cfg = cfg
        self.store_fp32 = store_fp32
        per_elem = 4 if store_fp32 else 2
        layer_elems = sum(tensor_shape(cfg, k)[0] * tensor_shape(cfg, k)[1] for k in LAYER_KINDS)
        self.n_resident = int(min(cfg.n_layers, resident_bytes // (layer_elems * per_elem)))
        self.store = {}
        self.regenerated = 0

    def _make(self, key):
        t = fastgen.gen_tensor_fast(self.cfg, key[0], key[1])
        return t

    def __getitem__(self, key):
        layer, kind = key
        if key in self.store:
            return self.store[key]
        t = self._make(key)
        if layer < 0 or layer < self.n_resident:
            if layer < 0 or self.store_fp32:
                t = t.to(torch.float32)
            self.store[key] = t
        else:
            self.regenerated += 1
        return t


def pad(rows, width, fill=-1, dtype=np.int32):
    out = np.full((len(rows), width), fill, dtype=dtype)
    for i, r in enumerate(rows):
        out[i, :len(r)] = r
    return out


def pad3(mats, width, dtype):
    """list of [L+1][<=width] -> [R, L+1, width], zero padded."""
    R, Lp1 = len(mats), len(mats[0])
    out = np.zeros((R, Lp1, width), dtype=dtype)
    for r, m in enumerate(mats):
        for l, row in enumerate(m):
            out[r, l, :len(row)] = row
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", required=True)
    ap.add_argument("--tokens", type=int, default=None, help="tokens to generate (default: the config's)")
    ap.add_argument("--max-rounds", type=int, default=None)
    ap.add_argument("--resident-gb", type=float, default=40.0)
    ap.add_argument("--store", choices=["fp32", "bf16"], default="fp32")
    ap.add_argument("--hidden-at", default="0,7,31",
                    help="round indices whose hidden rows are stored (the last round is always added)")
    ap.add_argument("--out", default=None)
    args = ap.parse_args()

    cfg = get_config(args.config)
    n_tokens = args.tokens or cfg.gen_len
    out_path = args.out or os.path.join(HERE, f"fullsize_{cfg.name}.npz")
    if not os.path.exists(os.path.join(ROOT, "synthdata", "libfastgen.so")):
        fastgen.build()
    L, D, d = cfg.n_layers, cfg.d_max, cfg.d_model
    hid_layers = [1, L // 2 + 1, L]
    t0 = time.time()

    def log(*a):
        print(f"[{cfg.name} {time.time() - t0:7.0f}s]", *a, flush=True)

    weights = LazyWeights(cfg, args.resident_gb * 1e9, args.store == "fp32")
    log(f"resident layers: {weights.n_resident}/{L} as {args.store}")
    oracle = Oracle(cfg, weights, dtype=torch.float32, cache_widened=False)
    prompt = gen_prompt(cfg).tolist()
    pre = oracle.prefill(prompt, keep_hidden=True)
    log(f"prefill done: first token {pre.first_token} gap {pre.first_gap:.3g} next (E, gamma) = "
        f"({pre.next_E}, {pre.next_gamma})")

    recs = []
    kept_hidden = {}
    toks = [pre.first_token]
    E, gamma = pre.next_E, pre.next_gamma

    def save(final: bool):
        R = len(recs)
        have = sorted(kept_hidden)
        hidden = np.zeros((len(have), 3, D + 1, d), dtype=np.float32)
        for k, r in enumerate(have):
            h = kept_hidden[r]
            hidden[k, :, :h.shape[1]] = h
        meta = dict(config=cfg.as_dict(), n_tokens=n_tokens, tokens_emitted=len(toks), rounds=R, complete=bool(final and len(toks) >= n_tokens),
                    oracle_dtype="float32", prompt_len=len(prompt),
                    schedule="DEL-selected (E, gamma), gamma clamped to remaining - 1",
                    writer="tests/golden/make_fullsize_records.py (oracle/ + synthdata/ only)")
        np.savez_compressed(
            out_path, meta=np.array(json.dumps(meta)), prompt=np.array(prompt, dtype=np.int32),
            tokens=np.array(toks, dtype=np.int32),
            pre_first_token=np.int32(pre.first_token), pre_first_gap=np.float32(pre.first_gap),
            pre_window=np.int32(pre.window), pre_shadow=np.array(pre.shadow, dtype=np.int32),
            pre_gaps=np.array(pre.gaps, dtype=np.float32), pre_conf=np.array(pre.conf, dtype=np.float64),
            pre_c=np.array(pre.c, dtype=np.int32), pre_alpha=np.array(pre.alpha, dtype=np.float64),
            pre_tau=np.array(pre.tau, dtype=np.float64), pre_next_E=np.int32(pre.next_E),
            pre_next_gamma=np.int32(pre.next_gamma),
            pre_tcs=np.array(oracle.stats.tcs_hist[0], dtype=np.float64),
            pre_fcs=np.array(oracle.stats.fcs_hist[0], dtype=np.float64),
            pre_hidden=np.stack([pre.hidden[l, -1].float().numpy() for l in hid_layers]),
            E=np.array([r.E for r in recs], dtype=np.int32), gamma=np.array([r.gamma for r in recs], dtype=np.int32),
            T_before=np.array([r.T_before for r in recs], dtype=np.int32),
            u=np.array([r.u for r in recs], dtype=np.int32), n=np.array([r.n for r in recs], dtype=np.int32),
            next_E=np.array([r.next_E for r in recs], dtype=np.int32),
            next_gamma=np.array([r.next_gamma for r in recs], dtype=np.int32),
            draft_ids=pad([r.draft_ids for r in recs], D), target_ids=pad([r.target_ids for r in recs], D + 1),
            shadow=pad3([r.shadow for r in recs], D + 1, np.int32) if R else np.zeros((0, L + 1, D + 1), np.int32),
            gaps=pad3([r.gaps for r in recs], D + 1, np.float32) if R else np.zeros((0, L + 1, D + 1), np.float32),
            conf=pad3([r.conf for r in recs], D + 1, np.float64) if R else np.zeros((0, L + 1, D + 1), np.float64),
            c=np.array([r.c for r in recs], dtype=np.int32).reshape(R, L + 1),
            alpha=np.array([r.alpha for r in recs], dtype=np.float64).reshape(R, L + 1),
            S_c=np.array([r.S_c for r in recs], dtype=np.float64).reshape(R, L + 1),
            S_tcs=np.array([r.S_tcs for r in recs], dtype=np.float64).reshape(R, L + 1),
            S_fcs=np.array([r.S_fcs for r in recs], dtype=np.float64).reshape(R, L + 1),
            tau=np.array([r.tau for r in recs], dtype=np.float64).reshape(R, L + 1),
            S_n=np.array([r.S_n for r in recs], dtype=np.float64),
            hidden_layers=np.array(hid_layers, dtype=np.int32), hidden_rounds=np.array(have, dtype=np.int32),
            hidden=hidden)

    hidden_at = set(int(x) for x in args.hidden_at.split(",") if x != "")
    while len(toks) < n_tokens and (args.max_rounds is None or len(recs) < args.max_rounds):
        g = min(gamma, n_tokens - len(toks) - 1)
        r = oracle.round(E, g, keep_hidden=True)
        idx = len(recs)
        # stored: the rounds asked for and, always, the latest one
        for k in list(kept_hidden):
            if k not in hidden_at:
                del kept_hidden[k]
        kept_hidden[idx] = np.stack([r.hidden[l].float().numpy() for l in hid_layers])
        r.hidden = None
        recs.append(r)
        toks.extend(r.out_tokens)
        near = sum(1 for l in range(1, L + 1) for x in r.gaps[l] if x < 1e-2)
        log(f"round {len(recs)} E={r.E} gamma={r.gamma} u={r.u} tokens={len(toks)} near-ties={near} "
            f"next=({r.next_E}, {r.next_gamma}) regenerated={weights.regenerated}")
        E, gamma = r.next_E, r.next_gamma
        if len(recs) % 8 == 0:
            save(False)
    save(True)
    log(f"wrote {out_path}: {len(recs)} rounds, {len(toks)} tokens, hidden rows of rounds {sorted(kept_hidden)}")


if __name__ == "__main__":
    main()
