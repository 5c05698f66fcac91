"""ctypes binding of include/del.h: argument marshalling only.

The module-level functions carry the C names (del_create, del_load_weights,
del_prefill, del_round, del_layer_stats, ...); DelContext is a small
convenience wrapper around them.  There is no CPU fallback: if the HIP library
is missing, load_library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))

EXPORTS = ["del_create", "del_destroy", "del_load_weights", "del_prefill", "del_round", "del_round_dynamic",
           "del_layer_stats", "del_set_layer_stats", "del_last_timings", "del_debug_hidden",
           "del_debug_logits", "del_debug_state", "del_debug_set_pending", "del_debug_last_rows", "del_profile_enable", "del_profile_read", "del_policy_step", "del_sample_first", "del_round_sample", "del_round_sample_dynamic", "del_debug_spec_sample", "del_spec_sample_static", "del_bench_stream_read", "del_bench_stream_copy", "del_bench_gemv_parts", "del_bench_mfma_rate", "del_strerror",
           "del_last_error_text"]

DEL_DTYPE_FP32, DEL_DTYPE_BF16 = 0, 1
DEL_MEM_HOST, DEL_MEM_DEVICE = 0, 1
KIND_IDS = {"embed": 0, "lm_head": 1, "final_norm": 2, "attn_norm": 3, "wq": 4, "wk": 5, "wv": 6,
            "wo": 7, "ffn_norm": 8, "wg": 9, "wu": 10, "wd": 11}


class DelError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"del status {status}: {text}")
        self.status = status


class del_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("tied_embeddings", C.c_int32), ("weight_dtype", C.c_int32),
                ("max_context", C.c_int32), ("d_max", C.c_int32), ("prefill_window", C.c_int32),
                ("omega", C.c_double), ("use_mfma", C.c_int32)]


class del_tensor(C.Structure):
    _fields_ = [("layer", C.c_int32), ("kind", C.c_int32), ("location", C.c_int32),
                ("reserved", C.c_int32), ("data", C.c_void_p), ("rows", C.c_int64),
                ("cols", C.c_int64)]


class del_prof_entry(C.Structure):
    _fields_ = [("flavour", C.c_int32), ("epilogue", C.c_int32), ("rows", C.c_int32),
                ("launches", C.c_int32), ("total_ms", C.c_double), ("weight_bytes", C.c_int64)]


class del_stats(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("rounds", C.c_int32), ("next_E", C.c_int32),
                ("next_gamma", C.c_int32), ("last_E", C.c_int32), ("last_gamma", C.c_int32),
                ("last_u", C.c_int32), ("last_n", C.c_int32), ("S_n", C.c_double),
                ("S_c", C.POINTER(C.c_double)), ("alpha", C.POINTER(C.c_double)),
                ("last_c", C.POINTER(C.c_int32)), ("last_shadow", C.POINTER(C.c_int32)),
                ("last_draft", C.POINTER(C.c_int32)),
                ("S_tcs", C.POINTER(C.c_double)), ("S_fcs", C.POINTER(C.c_double)),
                ("tau", C.POINTER(C.c_double)), ("last_conf", C.POINTER(C.c_float)),
                ("last_draft_conf", C.POINTER(C.c_float)), ("last_stopped", C.c_int32)]


_lib = None


def lib_path() -> str:
    return os.path.join(_HERE, "libdel_hip.so")


def load_library():
    """dlopen the HIP library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2504_05598_amd.build` "
                                "(or __graft_entry__.build()) first")
    lib = C.CDLL(path)
    P = C.POINTER
    lib.del_create.argtypes = [P(del_config), C.c_void_p, P(C.c_void_p)]
    lib.del_destroy.argtypes = [C.c_void_p]
    lib.del_destroy.restype = None
    lib.del_load_weights.argtypes = [C.c_void_p, P(del_tensor), C.c_int32]
    lib.del_prefill.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32, P(C.c_int32), P(C.c_int32),
                                P(C.c_int32)]
    lib.del_round.argtypes = [C.c_void_p, C.c_int32, C.c_int32, P(C.c_int32), P(C.c_int32)]
    lib.del_round_dynamic.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_int32, P(C.c_int32), P(C.c_int32),
                                      P(C.c_int32), P(C.c_int32)]
    lib.del_layer_stats.argtypes = [C.c_void_p, P(del_stats)]
    lib.del_set_layer_stats.argtypes = [C.c_void_p, P(del_stats)]
    lib.del_last_timings.argtypes = [C.c_void_p, P(C.c_float), P(C.c_float), P(C.c_float)]
    lib.del_debug_hidden.argtypes = [C.c_void_p, C.c_int32, C.c_int32, P(C.c_float)]
    lib.del_debug_logits.argtypes = [C.c_void_p, C.c_int32, C.c_int32, P(C.c_float)]
    lib.del_debug_state.argtypes = [C.c_void_p, P(C.c_int32), P(C.c_int32)]
    lib.del_debug_set_pending.argtypes = [C.c_void_p, C.c_int32]
    lib.del_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    lib.del_profile_read.argtypes = [C.c_void_p, P(del_prof_entry), C.c_int32, P(C.c_int32)]
    lib.del_bench_stream_read.argtypes = [C.c_void_p, C.c_int64, C.c_int32, P(C.c_float)]
    lib.del_bench_gemv_parts.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, P(C.c_float)]
    lib.del_bench_mfma_rate.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, P(C.c_float)]
    lib.del_bench_stream_copy.argtypes = [C.c_void_p, C.c_int64, C.c_int32, P(C.c_float)]
    lib.del_policy_step.argtypes = [C.c_int32, C.c_int32, C.c_double, P(C.c_int32), C.c_int32, P(C.c_double),
                                    P(C.c_double), P(C.c_double), P(C.c_double), P(C.c_double), P(C.c_double),
                                    P(C.c_double), P(C.c_double), P(C.c_int32), P(C.c_int32)]
    lib.del_debug_last_rows.argtypes = [C.c_void_p, P(C.c_int32)]
    lib.del_sample_first.argtypes = [C.c_void_p, C.c_double, C.c_double, C.c_float, P(C.c_int32)]
    lib.del_round_sample.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_double, P(C.c_float),
                                     P(C.c_int32), P(C.c_int32)]
    lib.del_round_sample_dynamic.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_int32, C.c_double, C.c_double,
                                             P(C.c_float), P(C.c_int32), P(C.c_int32), P(C.c_int32), P(C.c_int32)]
    lib.del_debug_spec_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_double,
                                          P(C.c_float), P(C.c_int32), P(C.c_int32), P(C.c_int32)]
    lib.del_spec_sample_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_double,
                                           C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.del_strerror.argtypes = [C.c_int]
    lib.del_strerror.restype = C.c_char_p
    lib.del_last_error_text.argtypes = [C.c_void_p]
    lib.del_last_error_text.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("del_destroy", "del_strerror", "del_last_error_text"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(status: int, ctx=None) -> None:
    if status != 0:
        lib = load_library()
        text = lib.del_strerror(status).decode()
        if ctx:
            extra = lib.del_last_error_text(ctx).decode()
            if extra:
                text += " (" + extra + ")"
        raise DelError(status, text)


# ---- functions with the C names -------------------------------------------------------
def del_create(cfg: del_config, stream: int = 0) -> C.c_void_p:
    ctx = C.c_void_p()
    _check(load_library().del_create(C.byref(cfg), C.c_void_p(stream), C.byref(ctx)))
    return ctx


def del_destroy(ctx) -> None:
    load_library().del_destroy(ctx)


def del_load_weights(ctx, tensors: Sequence[Tuple[int, str, int, int, int, int]]) -> None:
    """tensors: (layer, kind name, data pointer, location, rows, cols)."""
    arr = (del_tensor * len(tensors))()
    for i, (layer, kind, ptr, loc, rows, cols) in enumerate(tensors):
        arr[i] = del_tensor(layer, KIND_IDS[kind], loc, 0, ptr, rows, cols)
    _check(load_library().del_load_weights(ctx, arr, len(tensors)), ctx)


def del_prefill(ctx, prompt: Sequence[int]) -> Tuple[int, int, int]:
    n = len(prompt)
    buf = (C.c_int32 * n)(*prompt)
    first, E, g = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load_library().del_prefill(ctx, buf, n, C.byref(first), C.byref(E), C.byref(g)), ctx)
    return first.value, E.value, g.value


def del_round(ctx, E: int, gamma: int) -> List[int]:
    out = (C.c_int32 * (gamma + 1))()
    n = C.c_int32()
    _check(load_library().del_round(ctx, E, gamma, out, C.byref(n)), ctx)
    return list(out[:n.value])


def del_round_dynamic(ctx, E: int, tau: float, d_cap: int) -> Tuple[List[int], int, bool]:
    """Returns (accepted tokens, tokens drafted, stopped early)."""
    out = (C.c_int32 * (d_cap + 1))()
    n, g, stop = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load_library().del_round_dynamic(ctx, E, tau, d_cap, out, C.byref(n), C.byref(g), C.byref(stop)), ctx)
    return list(out[:n.value]), g.value, bool(stop.value)


def del_sample_first(ctx, temperature: float, top_p: float, r: float) -> int:
    tok = C.c_int32()
    _check(load_library().del_sample_first(ctx, temperature, top_p, r, C.byref(tok)), ctx)
    return tok.value


def del_round_sample(ctx, E: int, gamma: int, temperature: float, top_p: float,
                     uniforms: Sequence[float]) -> List[int]:
    """uniforms: 2 * gamma + 1 numbers in [0, 1): drafts, acceptances, last token."""
    if len(uniforms) < 2 * gamma + 1:
        raise ValueError("need 2 * gamma + 1 uniform numbers")
    un = (C.c_float * (2 * gamma + 1))(*[float(x) for x in uniforms[:2 * gamma + 1]])
    out = (C.c_int32 * (gamma + 1))()
    n = C.c_int32()
    _check(load_library().del_round_sample(ctx, E, gamma, temperature, top_p, un, out, C.byref(n)), ctx)
    return list(out[:n.value])


def del_round_sample_dynamic(ctx, E: int, tau: float, d_cap: int, temperature: float, top_p: float,
                             uniforms: Sequence[float]) -> Tuple[List[int], int, bool]:
    """uniforms: 2 * d_cap + 1 numbers.  Returns (tokens, tokens drafted, stopped early)."""
    if len(uniforms) < 2 * d_cap + 1:
        raise ValueError("need 2 * d_cap + 1 uniform numbers")
    un = (C.c_float * (2 * d_cap + 1))(*[float(x) for x in uniforms[:2 * d_cap + 1]])
    out = (C.c_int32 * (d_cap + 1))()
    n, g, stop = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load_library().del_round_sample_dynamic(ctx, E, tau, d_cap, temperature, top_p, un, out, C.byref(n),
                                                   C.byref(g), C.byref(stop)), ctx)
    return list(out[:n.value]), g.value, bool(stop.value)


def del_debug_spec_sample(ctx, q_logits, p_logits, gamma: int, temperature: float, top_p: float,
                          uniforms: Sequence[float], vocab: int) -> Tuple[List[int], int, int]:
    """q_logits [gamma, vocab] and p_logits [gamma + 1, vocab]: contiguous float32 numpy arrays (host).
    Returns (drafts, u, last token)."""
    if len(uniforms) < 2 * gamma + 1:
        raise ValueError("need 2 * gamma + 1 uniform numbers")
    for name, arr, rows in (("q_logits", q_logits, gamma), ("p_logits", p_logits, gamma + 1)):
        if rows == 0:
            continue
        if (str(arr.dtype) != "float32" or not arr.flags["C_CONTIGUOUS"] or arr.ndim != 2 or arr.shape[0] < rows
                or arr.shape[1] != vocab):
            raise ValueError(f"{name}: need a C-contiguous float32 array of shape [>= {rows}, {vocab}]")
    un = (C.c_float * (2 * gamma + 1))(*[float(x) for x in uniforms[:2 * gamma + 1]])
    drafts = (C.c_int32 * max(1, gamma))()
    u, last = C.c_int32(), C.c_int32()
    qp = q_logits.ctypes.data if gamma > 0 else None
    _check(load_library().del_debug_spec_sample(ctx, qp, p_logits.ctypes.data, gamma, temperature, top_p, un,
                                                drafts, C.byref(u), C.byref(last)), ctx)
    return list(drafts[:gamma]), u.value, last.value


def del_spec_sample_static(q_logits_ptr: int, p_logits_ptr: int, ld_logits: int, vocab: int, gamma: int,
                           temperature: float, top_p: float, uniforms_ptr: int, out_ptr: int, stream: int = 0) -> None:
    """Every pointer is a DEVICE address (an int); out receives 3 + gamma ints once the stream has passed
    the call: u, u + 1, the last token, the drafts.  Allocates nothing and does not wait."""
    _check(load_library().del_spec_sample_static(C.c_void_p(q_logits_ptr), C.c_void_p(p_logits_ptr), ld_logits, vocab,
                                                 gamma, temperature, top_p, C.c_void_p(uniforms_ptr),
                                                 C.c_void_p(out_ptr), C.c_void_p(stream)))


def del_layer_stats(ctx, n_layers: int, d_max: int) -> dict:
    L = n_layers
    S_c = (C.c_double * (L + 1))()
    alpha = (C.c_double * (L + 1))()
    last_c = (C.c_int32 * (L + 1))()
    shadow = (C.c_int32 * ((L + 1) * (d_max + 1)))()
    draft = (C.c_int32 * max(1, d_max))()
    S_tcs = (C.c_double * (L + 1))()
    S_fcs = (C.c_double * (L + 1))()
    tau = (C.c_double * (L + 1))()
    conf = (C.c_float * ((L + 1) * (d_max + 1)))()
    dconf = (C.c_float * (d_max + 1))()
    st = del_stats()
    st.S_tcs = C.cast(S_tcs, C.POINTER(C.c_double))
    st.S_fcs = C.cast(S_fcs, C.POINTER(C.c_double))
    st.tau = C.cast(tau, C.POINTER(C.c_double))
    st.last_conf = C.cast(conf, C.POINTER(C.c_float))
    st.last_draft_conf = C.cast(dconf, C.POINTER(C.c_float))
    st.S_c = C.cast(S_c, C.POINTER(C.c_double))
    st.alpha = C.cast(alpha, C.POINTER(C.c_double))
    st.last_c = C.cast(last_c, C.POINTER(C.c_int32))
    st.last_shadow = C.cast(shadow, C.POINTER(C.c_int32))
    st.last_draft = C.cast(draft, C.POINTER(C.c_int32))
    _check(load_library().del_layer_stats(ctx, C.byref(st)), ctx)
    g = st.last_gamma
    return {
        "rounds": st.rounds, "next_E": st.next_E, "next_gamma": st.next_gamma,
        "last_E": st.last_E, "last_gamma": g, "last_u": st.last_u, "last_n": st.last_n,
        "S_n": st.S_n, "S_c": list(S_c), "alpha": list(alpha), "last_c": list(last_c),
        "last_shadow": [list(shadow[l * (d_max + 1): l * (d_max + 1) + g + 1]) for l in range(L + 1)],
        "last_draft": list(draft[:g]),
        "S_tcs": list(S_tcs), "S_fcs": list(S_fcs), "tau": list(tau),
        "last_conf": [list(conf[l * (d_max + 1): l * (d_max + 1) + g + 1]) for l in range(L + 1)],
        "last_draft_conf": list(dconf[:g + (1 if st.last_stopped else 0)]),
        "last_stopped": bool(st.last_stopped),
    }


def del_set_layer_stats(ctx, S_c: Sequence[float], S_n: float,
                        S_tcs: Optional[Sequence[float]] = None, S_fcs: Optional[Sequence[float]] = None) -> None:
    arr = (C.c_double * len(S_c))(*S_c)
    st = del_stats()
    st.S_c = C.cast(arr, C.POINTER(C.c_double))
    st.S_n = S_n
    if S_tcs is not None and S_fcs is not None:
        a = (C.c_double * len(S_tcs))(*S_tcs)
        b = (C.c_double * len(S_fcs))(*S_fcs)
        st.S_tcs = C.cast(a, C.POINTER(C.c_double))
        st.S_fcs = C.cast(b, C.POINTER(C.c_double))
    _check(load_library().del_set_layer_stats(ctx, C.byref(st)), ctx)


def del_last_timings(ctx) -> Tuple[float, float, float]:
    a, b, c = C.c_float(), C.c_float(), C.c_float()
    _check(load_library().del_last_timings(ctx, C.byref(a), C.byref(b), C.byref(c)), ctx)
    return a.value, b.value, c.value


def del_policy_step(n_layers: int, d_max: int, omega: float, c: Sequence[int], n: int,
                    tcs: Sequence[float], fcs: Sequence[float], state: dict) -> dict:
    """One host-only policy update.  state: {"S_c", "S_n", "S_tcs", "S_fcs"} (lists indexed by layer
    number); returns the new state plus alpha, tau, next_E, next_gamma."""
    L = n_layers
    D = C.c_double * (L + 1)
    S_c, S_t, S_f = D(*state["S_c"]), D(*state["S_tcs"]), D(*state["S_fcs"])
    S_n = C.c_double(state["S_n"])
    alpha, tau = D(), D()
    E, g = C.c_int32(), C.c_int32()
    _check(load_library().del_policy_step(L, d_max, omega, (C.c_int32 * (L + 1))(*c), n, D(*tcs), D(*fcs),
                                          S_c, C.byref(S_n), S_t, S_f, alpha, tau, C.byref(E), C.byref(g)))
    return {"S_c": list(S_c), "S_n": S_n.value, "S_tcs": list(S_t), "S_fcs": list(S_f), "alpha": list(alpha),
            "tau": list(tau), "next_E": E.value, "next_gamma": g.value}


# ---- convenience wrapper ----------------------------------------------------------------
def make_config(cfg, use_mfma: bool = True, max_context: Optional[int] = None) -> del_config:
    """del_config from a synthdata.ModelConfig-like object."""
    return del_config(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                      cfg.d_ffn, cfg.vocab, cfg.rope_theta, cfg.rms_eps,
                      int(cfg.tied_embeddings),
                      DEL_DTYPE_BF16 if cfg.weight_dtype == "bf16" else DEL_DTYPE_FP32,
                      max_context or cfg.max_context, cfg.d_max, cfg.prefill_window, cfg.omega,
                      int(use_mfma))


class DelContext:
    """RAII wrapper: create / load / prefill / round / stats through the C ABI."""

    def __init__(self, cfg, use_mfma: bool = True, max_context: Optional[int] = None, stream: int = 0):
        self.cfg = cfg
        self.ccfg = make_config(cfg, use_mfma, max_context)
        self.ctx = del_create(self.ccfg, stream)

    def close(self) -> None:
        if self.ctx:
            del_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def load_tensor(self, layer: int, kind: str, tensor) -> None:
        """tensor: a contiguous torch tensor on the CPU or on the GPU (pointer + shape only)."""
        t = tensor.contiguous()
        loc = DEL_MEM_DEVICE if t.is_cuda else DEL_MEM_HOST
        rows, cols = (1, t.numel()) if kind.endswith("norm") else (t.shape[0], t.shape[1])
        del_load_weights(self.ctx, [(layer, kind, t.data_ptr(), loc, rows, cols)])

    def prefill(self, prompt: Sequence[int]) -> Tuple[int, int, int]:
        return del_prefill(self.ctx, prompt)

    def round(self, E: int, gamma: int) -> List[int]:
        return del_round(self.ctx, E, gamma)

    def round_dynamic(self, E: int, tau: float, d_cap: Optional[int] = None) -> Tuple[List[int], int, bool]:
        return del_round_dynamic(self.ctx, E, tau, self.cfg.d_max if d_cap is None else d_cap)

    def sample_first(self, temperature: float, top_p: float, r: float) -> int:
        return del_sample_first(self.ctx, temperature, top_p, r)

    def round_sample(self, E: int, gamma: int, temperature: float, top_p: float, uniforms) -> List[int]:
        return del_round_sample(self.ctx, E, gamma, temperature, top_p, uniforms)

    def round_sample_dynamic(self, E: int, tau: float, d_cap: int, temperature: float, top_p: float, uniforms):
        return del_round_sample_dynamic(self.ctx, E, tau, d_cap, temperature, top_p, uniforms)

    def spec_sample(self, q_logits, p_logits, gamma: int, temperature: float, top_p: float, uniforms):
        return del_debug_spec_sample(self.ctx, q_logits, p_logits, gamma, temperature, top_p, uniforms,
                                     self.cfg.vocab)

    def last_rows(self) -> int:
        """Rows the last pass filled; after a prefill the last prompt position is row last_rows() - 1."""
        n = C.c_int32()
        _check(load_library().del_debug_last_rows(self.ctx, C.byref(n)), self.ctx)
        return n.value

    def stats(self) -> dict:
        return del_layer_stats(self.ctx, self.cfg.n_layers, self.cfg.d_max)

    def set_stats(self, S_c: Sequence[float], S_n: float, S_tcs=None, S_fcs=None) -> None:
        del_set_layer_stats(self.ctx, S_c, S_n, S_tcs, S_fcs)

    def timings(self) -> Tuple[float, float, float]:
        return del_last_timings(self.ctx)

    def hidden(self, layer: int, row: int):
        import numpy as np
        buf = np.empty(self.cfg.d_model, dtype=np.float32)
        _check(load_library().del_debug_hidden(self.ctx, layer, row,
                                               buf.ctypes.data_as(C.POINTER(C.c_float))), self.ctx)
        return buf

    def logits(self, layer: int, row: int):
        import numpy as np
        buf = np.empty(self.cfg.vocab, dtype=np.float32)
        _check(load_library().del_debug_logits(self.ctx, layer, row,
                                               buf.ctypes.data_as(C.POINTER(C.c_float))), self.ctx)
        return buf

    def state(self) -> Tuple[int, int]:
        a, b = C.c_int32(), C.c_int32()
        _check(load_library().del_debug_state(self.ctx, C.byref(a), C.byref(b)), self.ctx)
        return a.value, b.value

    def set_pending(self, token: int) -> None:
        _check(load_library().del_debug_set_pending(self.ctx, token), self.ctx)

    def profile_enable(self, on: bool) -> None:
        _check(load_library().del_profile_enable(self.ctx, int(on)), self.ctx)

    def _rows_name(self, e):
        ng = self._rows_ng(e)   # template arguments as the profiler prints them: groups, epilogue, tiles per group
        return f"gemv_rows_k<2,{e.epilogue},5>" if ng == "2,5" else f"gemv_rows_k<{ng},{e.epilogue},4>"

    def _rows_ng(self, e):
        """Template argument NG of gemv_rows_k (k tiles = 64 * NG): the input width is the model width,
        except with the residual epilogue (1), where it follows from the bytes of the [d_model, K] matrix."""
        k = e.weight_bytes // (2 * self.cfg.d_model) if e.epilogue == 1 else self.cfg.d_model
        return "2,5" if k == 5120 else str(k // 2048)      # 160 k tiles: two groups of 5 tiles per wave

    def profile_read(self) -> List[dict]:
        cap = 256
        arr = (del_prof_entry * cap)()
        n = C.c_int32()
        _check(load_library().del_profile_read(self.ctx, arr, cap, C.byref(n)), self.ctx)
        names = {0: "store", 1: "resid", 2: "qkv_rope", 3: "swiglu", 4: "argmax"}
        out = []
        for e in arr[:min(n.value, cap)]:
            if e.launches:
                kernel = (f"gemm_valu_k<8,{e.rows},{e.epilogue}>" if e.flavour == 0
                          else f"gemm_mfma_k<{e.epilogue}>" if e.flavour == 1
                          else f"gemm_wide_k<{e.epilogue}>" if e.flavour == 3
                          else self._rows_name(e) if e.flavour == 4
                          else f"gemm_mfma_rows_k<{e.epilogue}>" if e.flavour == 5
                          else "head_gemm4_k" if e.flavour == 6 else "head_gemm_k")
                out.append({"kernel": kernel, "flavour": ("valu", "mfma", "mfma", "mfma", "valu", "mfma", "mfma")[e.flavour],
                            "epilogue": names[e.epilogue], "rows": e.rows, "launches": e.launches,
                            "total_ms": e.total_ms, "avg_us": 1e3 * e.total_ms / e.launches,
                            "weight_bytes": e.weight_bytes})
        return out

    def stream_copy_gbps(self, nbytes: int, iters: int = 10) -> float:
        """GB/s of a plain copy kernel counting bytes read plus bytes written."""
        ms = C.c_float()
        _check(load_library().del_bench_stream_copy(self.ctx, nbytes, iters, C.byref(ms)), self.ctx)
        return 2 * nbytes / (ms.value * 1e-3) / 1e9

    def gemv_parts_us(self, n_blocks: int, k_tiles: int, waves: int, parts: int, iters: int = 200) -> float:
        """del_bench_gemv_parts: microseconds per launch of the one-row GEMV with only `parts` switched on."""
        us = C.c_float(0.0)
        _check(load_library().del_bench_gemv_parts(self.ctx, n_blocks, k_tiles, waves, parts, iters, C.byref(us)), self.ctx)
        return float(us.value)

    def mfma_rate_ns(self, shape: int, n_acc: int, iters: int = 20000) -> float:
        """del_bench_mfma_rate: nanoseconds per matrix instruction and SIMD (shape 0: 16x16x32 bf16, 1: 32x32x16 bf16)."""
        ns = C.c_float(0.0)
        _check(load_library().del_bench_mfma_rate(self.ctx, shape, n_acc, iters, C.byref(ns)), self.ctx)
        return float(ns.value)

    def stream_read_gbps(self, nbytes: int, iters: int = 20) -> float:
        ms = C.c_float()
        _check(load_library().del_bench_stream_read(self.ctx, nbytes, iters, C.byref(ms)), self.ctx)
        return nbytes / (ms.value * 1e-3) / 1e9
