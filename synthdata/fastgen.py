"""Host fast path of gen_tensor: the same values, bit for bit, from a small C routine.

The torch integer code in generator.py is the definition (it runs unchanged on the GPU); this
module only makes regenerating a full-size model on the CPU affordable.  `build()` compiles
fastgen.c with gcc; `gen_tensor_fast` raises if the library has not been built.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import torch

from .configs import ModelConfig
from .generator import _std_for, _tensor_key, tensor_shape

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastgen.c")
_LIB = os.path.join(_HERE, "libfastgen.so")
_lib = None


def build() -> str:
    cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", _SRC, "-o", _LIB]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RuntimeError("synthdata/libfastgen.so is not built: call synthdata.fastgen.build()")
        _lib = ctypes.CDLL(_LIB)
        _lib.synth_fill.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _lib.synth_fill.restype = None
    return _lib


def gen_tensor_fast(cfg: ModelConfig, layer: int, kind: str) -> torch.Tensor:
    """Same tensor as generator.gen_tensor(cfg, layer, kind, device="cpu")."""
    lib = _load()
    if kind == "lm_head" and cfg.tied_embeddings:
        kind = "embed"
    rows, cols = tensor_shape(cfg, kind)
    n = rows * cols
    is_gain = kind.endswith("norm")
    out_dtype = torch.float32 if (is_gain or cfg.weight_dtype == "fp32") else torch.bfloat16
    out = torch.empty(n, dtype=out_dtype)
    if is_gain and cfg.norm_gain_std == 0.0:
        out.fill_(1.0)
        return out.view(rows, cols)
    std = torch.tensor(cfg.norm_gain_std if is_gain else _std_for(cfg, layer, kind), dtype=torch.float32).item()
    key = _tensor_key(cfg.weight_seed, layer, kind) & ((1 << 64) - 1)
    lib.synth_fill(key, 0, n, std, 1 if is_gain else 0, 1 if out_dtype == torch.bfloat16 else 0,
                   ctypes.c_void_p(out.data_ptr()))
    return out.view(rows, cols)
