"""Measurement entry points of the C ABI on the GPU: they run, return plausible figures and reject
arguments out of range (nothing here checks the method's arithmetic)."""
import ctypes as C

import pytest

pytestmark = pytest.mark.gpu


def test_gemv_parts_and_stream_hooks_run_and_validate():
    from paper_2504_05598_amd.binding import DelContext, load_library
    from synthdata import get_config
    cfg = get_config("mini_gqa")
    ctx = DelContext(cfg)   # weights not loaded: the arena is zero-filled, which a timing hook does not mind
    try:
        kt = cfg.d_model // 32
        nb = cfg.d_model // 16
        loads = ctx.gemv_parts_us(nb, kt, 8, 0, iters=20)
        whole = ctx.gemv_parts_us(nb, kt, 8, 7, iters=20)
        assert 0.0 < loads < 1e4 and 0.0 < whole < 1e4
        assert ctx.stream_read_gbps(1 << 20, 5) > 0.0
        lib = load_library()
        us = C.c_float(0.0)
        for bad in ((0, kt, 8, 0), (nb, 0, 8, 0), (nb, 481, 8, 0), (nb, kt, 5, 0), (nb, kt, 8, 8), (nb, kt, 8, -1)):
            assert lib.del_bench_gemv_parts(ctx.ctx, *bad, 5, C.byref(us)) == 1, bad          # DEL_E_ARG
        assert lib.del_bench_gemv_parts(ctx.ctx, nb, kt, 8, 0, 0, C.byref(us)) == 1
        assert lib.del_bench_gemv_parts(ctx.ctx, 1 << 24, 480, 8, 0, 5, C.byref(us)) == 3     # DEL_E_CAPACITY
    finally:
        ctx.close()


def test_matrix_instruction_rate_hook_runs_and_validates():
    from paper_2504_05598_amd.binding import DelContext, load_library
    from synthdata import get_config
    ctx = DelContext(get_config("mini_gqa"))
    try:
        for shape, n_acc in ((0, 2), (0, 4), (0, 8), (0, 16), (1, 1), (1, 2), (1, 4)):
            ns = ctx.mfma_rate_ns(shape, n_acc, iters=2000)
            # a 16x16x32 instruction cannot take less than 16 clocks, a 32x32x16 one less than 32; the clock is below 3 GHz
            assert (5.0 if shape == 0 else 10.0) < ns < 1e3, (shape, n_acc, ns)
        lib = load_library()
        out = C.c_float(0.0)
        for bad in ((2, 2), (-1, 2), (0, 3), (0, 1), (1, 8), (1, 0)):
            assert lib.del_bench_mfma_rate(ctx.ctx, bad[0], bad[1], 100, C.byref(out)) == 1, bad   # DEL_E_ARG
        assert lib.del_bench_mfma_rate(ctx.ctx, 0, 2, 0, C.byref(out)) == 1
    finally:
        ctx.close()
