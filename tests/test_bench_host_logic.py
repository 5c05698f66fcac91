"""Host-side pieces of bench.py that need no GPU: the one-GPU contract, the algorithmic byte counts behind the
roofline figures (Section 4.1: a round loads gamma * E + L layers), and the lookup of the stored HBM-traffic figure."""
import os
import subprocess
import sys

import bench
from synthdata import get_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode != 0
    assert "one GPU" in res.stdout


def test_round_bytes_follow_the_loaded_layer_count():
    cfg = get_config("llama7b")
    L, b_layer, b_head = cfg.n_layers, cfg.layer_weight_bytes(), cfg.head_weight_bytes()
    # weights alone: (gamma * E + L) layers and gamma + 1 heads; the rest (cache rows, hidden rows) is small beside them
    for E, gamma, T in ((12, 3, 1050), (1, 0, 64), (L, 8, 1279)):
        total = bench.round_bytes(cfg, E, gamma, T)
        weights = (gamma * E + L) * b_layer + (gamma + 1) * b_head
        assert weights < total < 1.12 * weights, (E, gamma, T)
        # the four segments account for the same bytes (they count the hidden rows of the shadow pass only)
        parts = sum(bench.segment_bytes(cfg, E, gamma, T))
        assert abs(parts - total) < 0.01 * total, (E, gamma, T, parts, total)
    # one more cached position costs every layer pass one more K and V row
    kv_row = 2 * cfg.n_kv_heads * cfg.head_dim * 2
    d = bench.round_bytes(cfg, 12, 3, 1051) - bench.round_bytes(cfg, 12, 3, 1050)
    assert d == (4 * 12 + (L - 12)) * kv_row


def test_stored_traffic_is_reported_only_for_the_sources_it_was_measured_on():
    assert bench.measured_traffic("no_such_config", "gemv_rows_k<2,3,4>") is None
    assert bench.measured_traffic("llama7b", "no_such_kernel") is None
    v = bench.measured_traffic("llama7b", "gemv_rows_k<2,3,4>")
    # None when the kernel sources have changed since the profile was taken; otherwise the gate/up matrix's bytes
    # plus a little (input row, output, counters' granularity)
    assert v is None or 1.0 <= v / 180355072 < 1.05
    h = bench.library_source_hash()
    assert len(h) == 16 and int(h, 16) >= 0 and h == bench.library_source_hash()
