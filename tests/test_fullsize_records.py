"""The stored full-size oracle records (tests/golden/fullsize_*.npz) and the generator's C fast path.

The records are written by tests/golden/make_fullsize_records.py from the oracle alone.  Here they are
held, on the CPU, to what Sections 2, 4.2 and 4.3 fix about any such run, recomputed from the stored
ids with the oracle's policy functions: u_r is the first draft that differs from the target's token,
c_r^l recounts from the shadow ids, the decayed sums follow S <- omega * S + a, alpha_l = S(c^l) / S(n),
the next (E, gamma) is the TPL arg-max, every round emits u_r + 1 tokens in [1, gamma + 1], the KV length
advances by that many, and each round runs with the previous round's selection.
"""
import glob
import json
import os

import numpy as np
import pytest
import torch

from oracle.del_oracle import first_mismatch, matched_counts, select_exit_and_length
from synthdata import fastgen, gen_prompt, gen_tensor, get_config

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FILES = sorted(glob.glob(os.path.join(GOLDEN, "fullsize_*.npz")))


def test_all_four_full_size_records_are_present():
    names = {os.path.basename(f)[len("fullsize_"):-4] for f in FILES}
    assert {"llama1b", "llama7b", "llama13b", "llama70b"} <= names


@pytest.mark.parametrize("path", FILES, ids=[os.path.basename(f) for f in FILES])
def test_records_are_self_consistent(path):
    check_record_file(path)


def test_the_record_writer_runs_end_to_end_on_the_tiny_shape(tmp_path):
    """tests/golden/make_fullsize_records.py itself (lazy weights, bf16 store, a budget that keeps only some
    layers resident), on the tiny shape: its output passes the same checks, and the oracle fed with the
    ordinary eager weights emits the same tokens."""
    import subprocess
    import sys
    from oracle.del_oracle import Oracle
    from synthdata import iter_tensor_specs
    out = tmp_path / "fullsize_tiny.npz"
    root = os.path.dirname(GOLDEN.rstrip(os.sep).rsplit(os.sep, 1)[0])
    script = os.path.join(GOLDEN, "make_fullsize_records.py")
    res = subprocess.run([sys.executable, script, "--config", "tiny", "--out", str(out), "--max-rounds", "5",
                          "--store", "bf16", "--resident-gb", "0.0001", "--hidden-at", "0,2"],
                         cwd=root, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:]
    check_record_file(str(out), min_rounds=3)
    z = np.load(str(out))
    cfg = get_config("tiny")
    host = {(layer, kind): gen_tensor(cfg, layer, kind) for layer, kind in iter_tensor_specs(cfg)}
    oracle = Oracle(cfg, host, dtype=torch.float32)
    pre = oracle.prefill(gen_prompt(cfg).tolist())
    toks = [pre.first_token]
    E, g = pre.next_E, pre.next_gamma
    for r in range(len(z["E"])):
        rec = oracle.round(E, min(g, cfg.gen_len - len(toks) - 1))
        toks.extend(rec.out_tokens)
        E, g = rec.next_E, rec.next_gamma
    assert toks == z["tokens"].tolist()


def check_record_file(path, min_rounds=3):
    z = np.load(path)
    meta = json.loads(str(z["meta"]))
    cfg = get_config(meta["config"]["name"])
    assert cfg.as_dict() == meta["config"]
    assert z["prompt"].tolist() == gen_prompt(cfg).tolist()
    L, D, om = cfg.n_layers, cfg.d_max, cfg.omega
    R = len(z["E"])
    assert R == meta["rounds"] and R >= min_rounds
    # prefill pseudo-round over the window
    w = int(z["pre_window"])
    pre_sh = z["pre_shadow"]
    assert int(z["pre_first_token"]) == int(pre_sh[L, w - 1])
    c0 = matched_counts(pre_sh.tolist(), pre_sh[L].tolist(), w - 1)
    assert c0 == z["pre_c"].tolist()
    Sc = np.array(c0, dtype=np.float64)
    Sn = float(w)
    assert np.allclose(z["pre_alpha"][1:], Sc[1:] / Sn, rtol=0, atol=1e-12)
    E, g = select_exit_and_length((Sc / Sn).tolist(), L, D)
    assert (E, g) == (int(z["pre_next_E"]), int(z["pre_next_gamma"]))
    tokens = [int(z["pre_first_token"])]
    T = len(z["prompt"])
    n_tokens = meta["n_tokens"]
    for r in range(R):
        gr = min(g, n_tokens - len(tokens) - 1)
        assert (int(z["E"][r]), int(z["gamma"][r])) == (E, gr), (r, E, gr)
        assert int(z["T_before"][r]) == T
        drafts = z["draft_ids"][r, :gr].tolist()
        target = z["target_ids"][r, :gr + 1].tolist()
        shadow = z["shadow"][r, :, :gr + 1]
        assert shadow[L].tolist() == target
        # the drafted tokens are layer E's greedy tokens at the drafted positions (same hidden states)
        assert shadow[E, :gr].tolist() == drafts
        u = first_mismatch(drafts, target, gr)
        assert u == int(z["u"][r]) and int(z["n"][r]) == u + 1 and 1 <= u + 1 <= gr + 1
        c = matched_counts(shadow.tolist(), target, u)
        assert c == z["c"][r].tolist() and c[L] == u + 1
        Sc = om * Sc + np.array(c, dtype=np.float64)
        Sn = om * Sn + (u + 1)
        assert np.allclose(z["S_c"][r, 1:], Sc[1:], rtol=1e-12) and abs(z["S_n"][r] - Sn) <= 1e-12 * Sn
        assert np.allclose(z["alpha"][r, 1:], Sc[1:] / Sn, rtol=0, atol=1e-12)
        # selection from the stored alpha (the very numbers the oracle selected from)
        E, g = select_exit_and_length(z["alpha"][r].tolist(), L, D)
        assert (E, g) == (int(z["next_E"][r]), int(z["next_gamma"][r]))
        tokens.extend(target[:u + 1])
        T += u + 1
        assert np.all(z["gaps"][r, 1:, :gr + 1] >= 0)
        assert np.all((z["conf"][r, 1:, :gr + 1] > 0) & (z["conf"][r, 1:, :gr + 1] <= 1.0 + 1e-12))
    assert tokens == z["tokens"].tolist()
    if meta["tokens_emitted"] >= n_tokens:    # a record cut short by --max-rounds holds fewer
        assert len(tokens) == n_tokens
    assert z["hidden"].shape[0] == len(z["hidden_rounds"]) >= 1
    assert np.isfinite(z["hidden"]).all() and np.abs(z["hidden"][0, :, 0]).max() > 0


def test_c_fast_path_of_the_generator_is_bit_identical():
    if not os.path.exists(os.path.join(os.path.dirname(fastgen.__file__), "libfastgen.so")):
        fastgen.build()
    for name in ("tiny", "mini_gqa", "mini_fp32", "mini_mha"):
        cfg = get_config(name)
        for layer, kind in [(-1, "embed"), (-1, "lm_head"), (-1, "final_norm"), (0, "wq"), (1, "wd"),
                            (2, "attn_norm"), (2, "wo"), (1, "wg")]:
            a, b = gen_tensor(cfg, layer, kind), fastgen.gen_tensor_fast(cfg, layer, kind)
            assert a.dtype == b.dtype and a.shape == b.shape
            bits = torch.int16 if a.dtype == torch.bfloat16 else torch.int32
            assert torch.equal(a.view(bits), b.view(bits)), (name, layer, kind)
    # a slice of a full-size tensor (the C path is what regenerates those)
    cfg = get_config("llama7b")
    a, b = gen_tensor(cfg, 5, "wk"), fastgen.gen_tensor_fast(cfg, 5, "wk")
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
