"""The C-ABI library loads and exports every symbol include/del.h declares (no GPU needed)."""
import ctypes
import os
import re

from conftest import ROOT


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "del.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(del_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_named_entry_points():
    names = _declared_symbols()
    for need in ("del_load_weights", "del_prefill", "del_round", "del_layer_stats",
                 "del_create", "del_destroy"):
        assert need in names


def test_library_exports_every_declared_symbol():
    from paper_2504_05598_amd import lib_path, EXPORTS
    path = lib_path()
    assert os.path.exists(path), "build first: python -m paper_2504_05598_amd.build"
    lib = ctypes.CDLL(path)
    names = _declared_symbols()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(EXPORTS) == names          # the binding covers the whole header


def test_error_strings_without_a_context():
    from paper_2504_05598_amd import load_library
    lib = load_library()
    assert lib.del_strerror(0) == b"ok"
    assert b"order" in lib.del_strerror(2)
    assert lib.del_create(None, None, None) == 1       # DEL_E_ARG, no device touched


def test_binding_rejects_misshapen_logits_before_any_device_call():
    import numpy as np
    import pytest
    from paper_2504_05598_amd import binding
    good = np.zeros((2, 10), dtype=np.float32)
    for bad in (np.zeros((2, 10), dtype=np.float64), np.zeros((2, 9), dtype=np.float32),
                np.zeros((10, 2), dtype=np.float32).T, np.zeros((1, 10), dtype=np.float32)):
        with pytest.raises(ValueError):
            binding.del_debug_spec_sample(None, good[:1].copy(), bad, 1, 1.0, 0.9, [0.1, 0.1, 0.1], 10)
    with pytest.raises(ValueError):
        binding.del_debug_spec_sample(None, good[:1].copy(), good, 1, 1.0, 0.9, [0.1], 10)
