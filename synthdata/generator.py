"""Counter-based, integer-only generator for synthetic weights and prompts.

Every element of every tensor is a pure function of (seed, tensor id, element
index), built from 64-bit integer operations and one fp32 multiply, so the CPU
and the GPU produce identical bits and any element can be addressed on its own.

Recipe per element e of tensor t:
  key   = mix(seed XOR mix(t))                      (mix = splitmix64 finaliser)
  z_j   = mix(key + (3e + j + 1) * GOLDEN), j=0,1,2  (three 64-bit draws)
  s     = sum of the twelve 16-bit fields of z_0, z_1, z_2
  n     = (s - 393210) / 65536      Irwin-Hall(12), mean 0, variance ~1, exact in fp32
  value = fp32(n) * fp32(std)       then round-to-nearest-even to bf16 if requested
The distribution is a slightly platykurtic stand-in for N(0, 1).

Norm gains are 1, or 1 + norm_gain_std * n for the test shapes that set it.
Prompt ids are (z_0 >> 33) mod vocab.

All code here is torch integer arithmetic that runs unchanged on "cpu" or "cuda".
"""
from __future__ import annotations

from typing import Iterator, Tuple

import torch

from .configs import ModelConfig

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int -> two's complement signed 64-bit value."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)

GLOBAL_KINDS = ("embed", "lm_head", "final_norm")
LAYER_KINDS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "wg", "wu", "wd")
KINDS = GLOBAL_KINDS + LAYER_KINDS
_KIND_ID = {k: i for i, k in enumerate(KINDS)}


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _tensor_key(seed: int, layer: int, kind: str) -> int:
    tid = (layer + 1) * 16 + _KIND_ID[kind]
    return _s64(_mix_int(seed ^ _mix_int(tid)))


_F16 = 0x0000FFFF0000FFFF


def _field_sum(z: torch.Tensor) -> torch.Tensor:
    """Sum of the four 16-bit fields of each int64."""
    s = (z & _F16) + (_lsr(z, 16) & _F16)
    return (s & 0xFFFFFFFF) + _lsr(s, 32)


def _normal_chunk(key: int, start: int, count: int, device) -> torch.Tensor:
    e = torch.arange(start, start + count, dtype=torch.int64, device=device)
    base = e * 3
    acc = torch.zeros(count, dtype=torch.int64, device=device)
    for j in range(3):
        z = _mix((base + (j + 1)) * _GOLDEN + key)
        acc += _field_sum(z)
    return (acc - 393210).to(torch.float32) * (1.0 / 65536.0)


def tensor_shape(cfg: ModelConfig, kind: str) -> Tuple[int, int]:
    d, f, v = cfg.d_model, cfg.d_ffn, cfg.vocab
    q = cfg.n_q_heads * cfg.head_dim
    kv = cfg.n_kv_heads * cfg.head_dim
    return {
        "embed": (v, d), "lm_head": (v, d), "final_norm": (1, d),
        "attn_norm": (1, d), "ffn_norm": (1, d),
        "wq": (q, d), "wk": (kv, d), "wv": (kv, d), "wo": (d, q),
        "wg": (f, d), "wu": (f, d), "wd": (d, f),
    }[kind]


def _std_for(cfg: ModelConfig, layer: int, kind: str) -> float:
    std = cfg.init_std
    if kind in ("wo", "wd"):
        std = std * (cfg.branch_decay ** layer)
    return std


def gen_tensor(cfg: ModelConfig, layer: int, kind: str, device="cpu",
               chunk: int | None = None) -> torch.Tensor:
    """Tensor `kind` of `layer` (-1 for the global tensors) as [rows, cols].

    Weight matrices are row-major [out_features, in_features].  dtype is
    cfg.weight_dtype for matrices and fp32 for norm gains.  A tied lm_head is
    the embedding tensor (same key).
    """
    if kind == "lm_head" and cfg.tied_embeddings:
        kind = "embed"
    if chunk is None:  # cache-sized pieces on the CPU, large ones on the GPU
        chunk = (1 << 18) if torch.device(device).type == "cpu" else (1 << 24)
    rows, cols = tensor_shape(cfg, kind)
    n = rows * cols
    key = _tensor_key(cfg.weight_seed, layer, kind)
    is_gain = kind.endswith("norm")
    out_dtype = torch.float32 if (is_gain or cfg.weight_dtype == "fp32") else torch.bfloat16
    out = torch.empty(n, dtype=out_dtype, device=device)
    if is_gain and cfg.norm_gain_std == 0.0:
        out.fill_(1.0)
        return out.view(rows, cols)
    std = torch.tensor(cfg.norm_gain_std if is_gain else _std_for(cfg, layer, kind),
                       dtype=torch.float32).item()
    for start in range(0, n, chunk):
        cnt = min(chunk, n - start)
        x = _normal_chunk(key, start, cnt, device) * std
        if is_gain:
            x = x + 1.0
        out[start:start + cnt] = x.to(out_dtype)
    return out.view(rows, cols)


def gen_prompt(cfg: ModelConfig, device="cpu", length: int | None = None) -> torch.Tensor:
    """Prompt of `length` (default cfg.prompt_len) token ids, int32, uniform in [0, vocab)."""
    n = cfg.prompt_len if length is None else length
    key = _s64(_mix_int(cfg.prompt_seed ^ _mix_int(0x70726F6D)))
    e = torch.arange(1, n + 1, dtype=torch.int64, device=device)
    z = _mix(e * _GOLDEN + key)
    return (_lsr(z, 33) % cfg.vocab).to(torch.int32)


def gen_uniforms(cfg: ModelConfig, stream: int, count: int) -> torch.Tensor:
    """`count` numbers k / 2^24, k uniform in [0, 2^24), as float32 (exact): the random numbers a
    sampling run consumes.  `stream` separates draws (e.g. the round number)."""
    key = _s64(_mix_int(cfg.prompt_seed ^ _mix_int(0x756E6966 + 0x10001 * int(stream))))
    e = torch.arange(1, count + 1, dtype=torch.int64)
    z = _mix(e * _GOLDEN + key)
    return (_lsr(z, 40).to(torch.float64) / float(1 << 24)).to(torch.float32)


def iter_tensor_specs(cfg: ModelConfig) -> Iterator[Tuple[int, str]]:
    """(layer, kind) of every tensor a model needs, global tensors first."""
    yield (-1, "embed")
    if not cfg.tied_embeddings:
        yield (-1, "lm_head")
    yield (-1, "final_norm")
    for l in range(cfg.n_layers):
        for k in LAYER_KINDS:
            yield (l, k)
