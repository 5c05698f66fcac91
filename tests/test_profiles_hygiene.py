"""The committed profiler summaries: short text files that state the command that produced them."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def test_summaries_are_short_text_with_their_command():
    names = sorted(os.listdir(PROFILES))
    assert names, "no profiler summaries"
    for name in names:
        path = os.path.join(PROFILES, name)
        assert name.endswith((".txt", ".md")), name
        assert os.path.getsize(path) < 64 * 1024, name
        text = open(path, encoding="utf-8").read()
        assert re.search(r"(?im)^#.*command", text), f"{name}: no command line"
        assert "bench.py" in text or "paper_2504_05598_amd" in text, f"{name}: the command runs no committed file"


def test_the_traffic_summary_names_the_sources_it_was_measured_on():
    text = open(os.path.join(PROFILES, "bench_llama7b_hbm_traffic.txt"), encoding="utf-8").read()
    assert re.search(r"(?m)^library_source_hash [0-9a-f]{16}$", text)
    assert re.search(r"(?m)^traffic_bytes_per_launch \S+ \d+$", text)
    assert "stream_copy_k" in text      # the known-size kernel the counters are scaled by
