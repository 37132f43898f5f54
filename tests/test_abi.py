"""The C-ABI library loads, exports every function include/grass.h declares, and rejects
bad arguments on the host before anything is launched (CPU only: no call here reaches a
kernel launch)."""
import ctypes as C
import os
import re

import pytest

from paper_2406_17660_amd import grass

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = C.c_void_p(0x1000)  # never dereferenced: validation fails first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "grass.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(grass_[a-z_]+)\s*\(", text)))


def test_header_and_library_agree():
    names = declared_functions()
    assert len(names) >= 12
    assert sorted(grass.EXPORTS) == names
    L = grass.lib()
    for name in names:
        assert hasattr(L, name), name


def test_header_is_plain_c_and_cxx(tmp_path):
    """include/grass.h stands on its own as C99 and as C++11 (no torch or HIP types in it)."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for compiler, std, ext in (("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "cpp")):
        if shutil.which(compiler) is None:
            pytest.skip(f"{compiler} not installed")
        src = tmp_path / f"use_header.{ext}"
        src.write_text('#include "include/grass.h"\nint main(void) { return (int)GRASS_OK; }\n')
        r = subprocess.run([compiler, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                            "-I", root, str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_status_strings():
    seen = {grass.status_string(c) for c in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert grass.status_string(99) == "unknown status"


def test_workspace_queries_are_pure_host_functions():
    assert grass.select_workspace(4096, 1024, grass.SEL_TOPR, False) >= 4
    a = grass.select_workspace(4096, 1024, grass.SEL_MULTI_NORM, True)
    b = grass.select_workspace(8192, 1024, grass.SEL_MULTI_NORM, True)
    assert b > a >= 4096 * 12
    assert grass.select_workspace(13824, 1024, grass.SEL_MULTI_NORM, False) >= 13824 * 8
    assert grass.cgrad_workspace(131072, 4096, 4096, 1024, grass.BF16) >= 131072 * 1024 * 2
    assert grass.cgrad_workspace(512, 256, 256, 16, grass.F32) == 0
    assert grass.dense_workspace(1024, 512, 512, grass.BF16) >= 512 * 512 * 4


def test_row_stats_validation():
    L = grass.lib()
    assert L.grass_row_stats(None, grass.F32, 4, 4, 4, FAKE, None) == grass.ERR_NULL
    assert L.grass_row_stats(FAKE, grass.F32, 4, 4, 4, None, None) == grass.ERR_NULL
    assert L.grass_row_stats(FAKE, 7, 4, 4, 4, FAKE, None) == grass.ERR_DTYPE
    assert L.grass_row_stats(FAKE, grass.F32, -1, 4, 4, FAKE, None) == grass.ERR_SHAPE
    assert L.grass_row_stats(FAKE, grass.F32, 4, 4, 3, FAKE, None) == grass.ERR_SHAPE


def test_select_validation():
    L = grass.lib()
    f = L.grass_select_rows
    ok_ws = 1 << 20
    assert f(None, 8, 2, 0, 0, 0, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_NULL
    assert f(FAKE, 8, 2, 9, 0, 0, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_DTYPE
    assert f(FAKE, 8, 2, 0, 0, 5, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_DTYPE
    # forced 1/sqrt(r q) makes no sense for Top-r
    assert f(FAKE, 8, 2, grass.SEL_TOPR, 0, grass.SCALE_INV_SQRT_RQ, 0, 0, FAKE, FAKE, FAKE, ok_ws,
             None) == grass.ERR_DTYPE
    assert f(FAKE, 8, 9, grass.SEL_TOPR, 0, 0, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_SHAPE
    assert f(FAKE, 8, 9, grass.SEL_UNIFORM, 0, 0, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_SHAPE
    assert f(FAKE, 0, 1, grass.SEL_UNIFORM, 1, 0, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_SHAPE
    assert f(FAKE, 8, -1, 0, 0, 0, 0, 0, FAKE, FAKE, FAKE, ok_ws, None) == grass.ERR_SHAPE
    assert f(FAKE, 8, 2, grass.SEL_MULTI_NORM, 1, 0, 0, 0, FAKE, FAKE, None, ok_ws, None) == grass.ERR_WORKSPACE
    assert f(FAKE, 8, 2, grass.SEL_MULTI_NORM, 1, 0, 0, 0, FAKE, FAKE, FAKE, 8, None) == grass.ERR_WORKSPACE


def test_select_static_validation():
    """The no-allocation form validates like grass_select_rows and refuses, on the host and
    before any HIP call, what its built-in scratch cannot hold."""
    f = grass.lib().grass_select_rows_static
    cap = grass.select_static_capacity()
    assert cap == 1 << 20
    ok = (FAKE, 4096, 1024, grass.SEL_MULTI_NORM, 1, grass.SCALE_PAPER, 1, 0, FAKE, FAKE, None, None)

    def call(**kw):
        names = ("sumsq", "m", "r", "method", "replacement", "scale", "seed", "refresh_id", "idx",
                 "rho", "status", "stream")
        return f(*[kw.get(n, v) for n, v in zip(names, ok)])
    assert call(sumsq=None) == grass.ERR_NULL
    assert call(idx=None) == grass.ERR_NULL
    assert call(m=-1) == grass.ERR_SHAPE
    assert call(replacement=0, r=5000) == grass.ERR_SHAPE
    assert call(method=9) == grass.ERR_DTYPE
    assert call(method=grass.SEL_TOPR, scale=grass.SCALE_INV_SQRT_RQ) == grass.ERR_DTYPE
    for m, repl in ((100000, 1), (200000, 0)):
        assert grass.select_workspace(m, 10, grass.SEL_MULTI_NORM, repl) > cap
        assert call(m=m, r=10, replacement=repl) == grass.ERR_WORKSPACE
    for repl in (0, 1):  # 65536 rows fit for every rule
        assert grass.select_workspace(65536, 1024, grass.SEL_MULTI_NORM2, repl) <= cap


def test_compressed_grad_validation():
    L = grass.lib()
    f = L.grass_compressed_grad
    big = 1 << 40
    args = dict(dY=FAKE, layout=0, ldy=64, X=FAKE, ldx=32, dt=grass.BF16, T=128, m=64, n=32, r=8,
                idx=FAKE, rho=FAKE, GC=FAKE, ldgc=32, ws=FAKE, wsb=big, stream=None)

    def call(**kw):
        a = dict(args, **kw)
        return f(a["dY"], a["layout"], a["ldy"], a["X"], a["ldx"], a["dt"], a["T"], a["m"], a["n"],
                 a["r"], a["idx"], a["rho"], a["GC"], a["ldgc"], a["ws"], a["wsb"], a["stream"])

    assert call(dY=None) == grass.ERR_NULL
    assert call(idx=None) == grass.ERR_NULL
    assert call(GC=None) == grass.ERR_NULL
    assert call(dt=5) == grass.ERR_DTYPE
    assert call(layout=3) == grass.ERR_DTYPE
    assert call(ldx=31) == grass.ERR_SHAPE
    assert call(ldy=63) == grass.ERR_SHAPE
    assert call(layout=1, ldy=127) == grass.ERR_SHAPE  # m x T storage needs ldy >= T
    assert call(ldgc=31) == grass.ERR_SHAPE
    assert call(T=-1) == grass.ERR_SHAPE
    assert call(ws=None) == grass.ERR_WORKSPACE
    assert call(wsb=1024) == grass.ERR_WORKSPACE


def test_compressed_grad_group_validation():
    import ctypes as C
    L = grass.lib()
    f = L.grass_compressed_grad_group
    big = 1 << 40

    def i64(*v):
        return (C.c_int64 * len(v))(*v)

    def ptrs(*v):
        return (C.c_void_p * len(v))(*v)

    def call(count=2, dY=(FAKE, FAKE), ldy=(64, 48), ldx=32, dt=grass.BF16, T=128, m=(64, 48), n=32,
             r=(8, 5), idx=(FAKE, FAKE), rho=(FAKE, FAKE), GC=(FAKE, FAKE), ldgc=(32, 40), ws=FAKE,
             wsb=big):
        return f(count, ptrs(*dY), 0, i64(*ldy), FAKE, ldx, dt, T, i64(*m), n, i64(*r), ptrs(*idx),
                 ptrs(*rho), ptrs(*GC), i64(*ldgc), ws, wsb, None)

    assert call(count=0) == grass.ERR_SHAPE
    assert call(count=9) == grass.ERR_SHAPE
    assert call(dY=(FAKE, None)) == grass.ERR_NULL
    assert call(idx=(None, FAKE)) == grass.ERR_NULL
    assert call(GC=(FAKE, None)) == grass.ERR_NULL
    assert call(ldy=(64, 47)) == grass.ERR_SHAPE
    assert call(ldgc=(32, 31)) == grass.ERR_SHAPE
    assert call(r=(8, -1)) == grass.ERR_SHAPE
    assert call(dt=7) == grass.ERR_DTYPE
    assert call(ws=None) == grass.ERR_WORKSPACE
    assert call(wsb=512) == grass.ERR_WORKSPACE
    # the group's workspace covers the packed panel of all sets and is a pure host query
    one = L.grass_cgrad_workspace(4096, 64, 512, 256, grass.BF16, 0)
    two = L.grass_cgrad_group_workspace(4096, 512, 2, i64(256, 256), grass.BF16, 0)
    assert two > one > 0
    assert L.grass_cgrad_group_workspace(4096, 512, 0, i64(), grass.BF16, 0) == 0


def test_sizes_of_2_to_the_31_and_more_are_refused_everywhere():
    """Every size is below 2^31, so that no product of two of them can leave 64 bits."""
    L = grass.lib()
    big = 1 << 31
    assert L.grass_row_stats(FAKE, grass.F32, 4, big, big, FAKE, None) == grass.ERR_SHAPE
    assert L.grass_row_stats(FAKE, grass.F32, big, 4, 4, FAKE, None) == grass.ERR_SHAPE
    assert L.grass_adam_rows(FAKE, big, FAKE, FAKE, 2, big, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE,
                             None) == grass.ERR_SHAPE
    assert L.grass_adam_rows(FAKE, 8, FAKE, FAKE, big, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE,
                             None) == grass.ERR_SHAPE
    assert L.grass_scatter_update(FAKE, 0, big, 8, 8, FAKE, FAKE, 1.0, FAKE, 2,
                                  None) == grass.ERR_SHAPE
    assert L.grass_scatter_update_cols(FAKE, 0, big, 8, 8, FAKE, FAKE, 1.0, FAKE, 2,
                                       None) == grass.ERR_SHAPE
    assert L.grass_gather_rows(FAKE, 0, 4, big, big, FAKE, FAKE, 2, FAKE, big,
                               None) == grass.ERR_SHAPE
    assert grass.cgrad_workspace(big, 256, 256, 16, grass.BF16) == 0
    assert grass.dense_workspace(1024, big, 512, grass.BF16) == 0


def test_adam_and_scatter_validation():
    L = grass.lib()
    a = L.grass_adam_rows
    assert a(None, 8, FAKE, FAKE, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE, None) == grass.ERR_NULL
    assert a(FAKE, 8, FAKE, FAKE, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, None, None) == grass.ERR_NULL
    assert a(FAKE, 7, FAKE, FAKE, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE, None) == grass.ERR_SHAPE
    assert a(FAKE, 8, FAKE, FAKE, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 0, FAKE, None) == grass.ERR_SHAPE
    assert a(FAKE, 8, FAKE, FAKE, 2, 8, 1e-3, 1.0, 0.999, 1e-8, 1, FAKE, None) == grass.ERR_SHAPE
    assert a(FAKE, 8, FAKE, FAKE, 2, 8, 1e-3, 0.9, -0.1, 1e-8, 1, FAKE, None) == grass.ERR_SHAPE
    s = L.grass_scatter_update
    assert s(None, 0, 4, 8, 8, FAKE, FAKE, 1.0, FAKE, 2, None) == grass.ERR_NULL
    assert s(FAKE, 3, 4, 8, 8, FAKE, FAKE, 1.0, FAKE, 2, None) == grass.ERR_DTYPE
    assert s(FAKE, 0, 4, 8, 7, FAKE, FAKE, 1.0, FAKE, 2, None) == grass.ERR_SHAPE
    assert s(FAKE, 0, 4, 8, 8, FAKE, FAKE, 1.0, FAKE, 70000, None) == grass.ERR_SHAPE
    sc = L.grass_scatter_update_cols
    assert sc(None, 0, 4, 8, 8, FAKE, FAKE, 1.0, FAKE, 2, None) == grass.ERR_NULL
    assert sc(FAKE, 0, 4, 8, 8, FAKE, FAKE, 1.0, None, 2, None) == grass.ERR_NULL
    assert sc(FAKE, 5, 4, 8, 8, FAKE, FAKE, 1.0, FAKE, 2, None) == grass.ERR_DTYPE
    assert sc(FAKE, 0, 4, 8, 7, FAKE, FAKE, 1.0, FAKE, 2, None) == grass.ERR_SHAPE
    f = L.grass_adam_scatter
    assert f(FAKE, 8, FAKE, FAKE, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, None, 0, 4, 8, FAKE, FAKE, 1.0,
             None) == grass.ERR_NULL
    assert f(FAKE, 8, FAKE, FAKE, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 0, FAKE, 0, 4, 8, FAKE, FAKE, 1.0,
             None) == grass.ERR_SHAPE
    # the state-dtype forms: same checks plus the dtype of the moments
    a2 = L.grass_adam_rows_state
    assert a2(FAKE, 8, FAKE, FAKE, grass.BF16, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, None, None) == grass.ERR_NULL
    assert a2(FAKE, 8, None, FAKE, grass.BF16, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE, None) == grass.ERR_NULL
    assert a2(FAKE, 8, FAKE, FAKE, 2, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE, None) == grass.ERR_DTYPE
    assert a2(FAKE, 8, FAKE, FAKE, grass.BF16, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 0, FAKE, None) == grass.ERR_SHAPE
    f2 = L.grass_adam_scatter_state
    assert f2(FAKE, 8, FAKE, FAKE, 9, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE, 0, 4, 8, FAKE, FAKE, 1.0,
              None) == grass.ERR_DTYPE
    assert f2(FAKE, 8, FAKE, FAKE, grass.BF16, 2, 8, 1e-3, 0.9, 0.999, 1e-8, 1, FAKE, 0, 4, 7, FAKE,
              FAKE, 1.0, None) == grass.ERR_SHAPE
    d = L.grass_dense_grad
    assert d(FAKE, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, None, 0, 32, FAKE, 1 << 40, None) == grass.ERR_NULL
    assert d(FAKE, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, FAKE, 4, 32, FAKE, 1 << 40, None) == grass.ERR_DTYPE
    assert d(FAKE, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, FAKE, 0, 32, FAKE, 16, None) == grass.ERR_WORKSPACE
    g = L.grass_gather_rows
    assert g(FAKE, 0, 4, 8, 8, None, FAKE, 2, FAKE, 8, None) == grass.ERR_NULL
    assert g(FAKE, 0, 4, 8, 8, FAKE, FAKE, 2, FAKE, 7, None) == grass.ERR_SHAPE


def test_replayable_adam_validation_and_step_scalars():
    import ctypes as C
    L = grass.lib()
    out = (C.c_float * 3)()
    assert L.grass_adam_step_scalars(1e-3, 0.9, 0.999, 1, out) == grass.OK
    # t = 1: the corrections are 1 / (1 - beta); float32 of the double-precision value
    import numpy as np
    assert out[0] == np.float32(1e-3)
    assert out[1] == np.float32(1.0 / (1.0 - float(np.float32(0.9))))
    assert out[2] == np.float32(1.0 / (1.0 - float(np.float32(0.999))))
    assert L.grass_adam_step_scalars(1e-3, 0.9, 0.999, 0, out) == grass.ERR_SHAPE
    assert L.grass_adam_step_scalars(1e-3, 1.0, 0.999, 1, out) == grass.ERR_SHAPE
    assert L.grass_adam_step_scalars(1e-3, 0.9, 0.999, 1, None) == grass.ERR_NULL
    f = L.grass_adam_scatter_replayable
    args = [FAKE, 8, FAKE, FAKE, grass.F32, 2, 8, 0.9, 0.999, 1e-8, FAKE, FAKE, 0, 4, 8, FAKE, FAKE,
            1.0, None]
    bad = list(args); bad[10] = None
    assert f(*bad) == grass.ERR_NULL
    bad = list(args); bad[4] = 7
    assert f(*bad) == grass.ERR_DTYPE
    bad = list(args); bad[14] = 7
    assert f(*bad) == grass.ERR_SHAPE


def test_step_group_validation():
    import ctypes as C
    L = grass.lib()
    f = L.grass_step_group
    big = 1 << 40

    def layer(**kw):
        d = dict(dY=FAKE, ldy=64, m=64, r=8, idx=FAKE, rho=FAKE, GC=None, ldgc=0, M=FAKE, V=FAKE,
                 W=FAKE, ldw=32)
        d.update(kw)
        return grass.StepLayer(d["dY"], d["ldy"], d["m"], d["r"], d["idx"], d["rho"], d["GC"],
                               d["ldgc"], d["M"], d["V"], d["W"], d["ldw"])

    def call(layers, count=None, ldx=32, dt=grass.BF16, T=128, n=32, sdt=grass.F32, wdt=grass.BF16,
             t=1, scal=None, ws=FAKE, wsb=big):
        arr = (grass.StepLayer * len(layers))(*layers)
        return f(len(layers) if count is None else count, arr, 0, FAKE, ldx, dt, T, n, sdt, wdt, 1e-3,
                 0.9, 0.999, 1e-8, t, scal, 0.25, ws, wsb, None, None, None)

    assert call([layer()], count=0) == grass.ERR_SHAPE
    assert call([layer()], count=9) == grass.ERR_SHAPE
    assert call([layer(dY=None)]) == grass.ERR_NULL
    assert call([layer(M=None)]) == grass.ERR_NULL
    assert call([layer(W=None)]) == grass.ERR_NULL
    assert call([layer(idx=None)]) == grass.ERR_NULL
    assert call([layer(ldy=63)]) == grass.ERR_SHAPE
    assert call([layer(ldw=31)]) == grass.ERR_SHAPE
    assert call([layer(GC=FAKE, ldgc=31)]) == grass.ERR_SHAPE
    assert call([layer()], t=0) == grass.ERR_SHAPE
    assert call([layer()], sdt=5) == grass.ERR_DTYPE
    assert call([layer()], wdt=5) == grass.ERR_DTYPE
    assert call([layer()], ws=None) == grass.ERR_WORKSPACE
    assert call([layer()], wsb=1024) == grass.ERR_WORKSPACE
    i64 = (C.c_int64 * 2)(256, 256)
    a = L.grass_step_group_workspace(4096, 512, 2, i64, grass.BF16, 0)
    b = L.grass_cgrad_group_workspace(4096, 512, 2, i64, grass.BF16, 0)
    assert a >= b + 2 * 256 * 512 * 4  # room for a G_C per layer that does not name one


def test_step_cols_validation():
    L = grass.lib()
    f = L.grass_step_cols
    T, m, n, r = 128, 64, 32, 8
    big_ws = 1 << 30
    ok = dict(dY=FAKE, ldy=m, X=FAKE, ldx=n, dt=grass.BF16, T=T, m=m, n=n, r=r, idx=FAKE, rho=FAKE,
              GC=None, ldgc=0, M=FAKE, V=FAKE, sdt=grass.F32, U=FAKE, W=FAKE, wdt=grass.BF16, ldw=n,
              lr=1e-3, b1=0.9, b2=0.999, eps=1e-8, t=1, alpha=0.25, ws=FAKE, ws_bytes=big_ws,
              stream=None, e0=None, e1=None)

    def call(**kw):
        a = dict(ok, **kw)
        return f(*a.values())
    assert grass.step_cols_workspace(T, m, n, r, grass.BF16) >= r * m * 4
    assert grass.step_cols_workspace(T, m, n, 70000, grass.BF16) == 0
    assert call(dY=None) == grass.ERR_NULL
    assert call(U=None) == grass.ERR_NULL
    assert call(W=None) == grass.ERR_NULL
    assert call(ldw=n - 1) == grass.ERR_SHAPE
    assert call(ldy=m - 1) == grass.ERR_SHAPE
    assert call(GC=FAKE, ldgc=m - 1) == grass.ERR_SHAPE
    assert call(r=70000) == grass.ERR_SHAPE
    assert call(t=0) == grass.ERR_SHAPE
    assert call(U=C.c_void_p(FAKE.value + 4)) == grass.ERR_SHAPE  # 16-byte aligned scratch
    assert call(wdt=5) == grass.ERR_DTYPE
    assert call(sdt=5) == grass.ERR_DTYPE
    assert call(ws=None) == grass.ERR_WORKSPACE
    assert call(ws_bytes=16) == grass.ERR_WORKSPACE


def test_probe_library_validation():
    """The benchmark's measurement aid lives in a library and header of its own."""
    from paper_2406_17660_amd import probe
    f = probe.lib().mfma_rate_probe
    flops = C.c_double(0.0)
    ok = (0, None, 0, FAKE, 1 << 16, 10, C.byref(flops), None)

    def call(**kw):
        names = ("source", "operands", "operand_bytes", "out", "out_floats", "iters", "flops", "stream")
        return f(*[kw.get(n, v) for n, v in zip(names, ok)])
    assert call(out=None) == probe.ERR_NULL
    assert call(flops=None) == probe.ERR_NULL
    assert call(iters=0) == probe.ERR_SIZE
    assert call(out_floats=1000) == probe.ERR_SIZE
    assert call(source=3) == probe.ERR_SOURCE
    for source in (probe.REGISTERS, probe.LDS):  # these read the caller's values
        assert call(source=source) == probe.ERR_NULL
        assert call(source=source, operands=FAKE, operand_bytes=65535) == probe.ERR_SIZE
        assert call(source=source, operands=C.c_void_p(FAKE.value + 2), operand_bytes=65536) == probe.ERR_SIZE
    assert not hasattr(grass.lib(), "grass_probe_mfma_rate") and not hasattr(grass.lib(), "mfma_rate_probe")


def test_plan_query_and_test_options():
    """grass_cgrad_plan is a pure host function; the test hooks change what it reports."""
    assert grass.cgrad_plan(131072, 4096, 1024, grass.BF16) == (256, 4)
    tile, slices = grass.cgrad_plan(65536, 512, 128, grass.BF16)
    assert tile == 128 and slices > 8  # the short, wide problems of the small models
    assert grass.cgrad_plan(512, 256, 16, grass.F32) == (64, 1)
    assert grass.cgrad_plan(1056, 264, 260, grass.BF16)[0] == 128
    grass.set_test_option(grass.TEST_GEMM_TILE, 256)
    try:
        assert grass.cgrad_plan(1056, 264, 260, grass.BF16)[0] == 256
    finally:
        grass.set_test_option(grass.TEST_GEMM_TILE, 0)
    assert grass.cgrad_plan(1056, 264, 260, grass.BF16)[0] == 128
    grass.set_test_option(grass.TEST_MAX_K_SLICES, 6)
    try:
        assert grass.cgrad_plan(65536, 512, 128, grass.BF16) == (128, 6)
    finally:
        grass.set_test_option(grass.TEST_MAX_K_SLICES, 0)
    assert grass.cgrad_plan(65536, 512, 128, grass.BF16)[1] > 8
    # narrow layers (row length of dY given): the gather runs inside the GEMM, tile code 0
    assert grass.cgrad_plan(65536, 512, 128, grass.BF16, m=512) == (0, 128)
    assert grass.cgrad_plan(65536, 512, 384, grass.BF16, m=512, count=3) == (0, 84)
    assert grass.cgrad_plan(65536, 512, 256, grass.BF16, m=1376, count=2)[0] == 256  # rows of dY too long
    assert grass.cgrad_plan(65536, 1376, 128, grass.BF16, m=512)[0] == 128          # too many column tiles
    assert grass.cgrad_plan(65536, 512, 264, grass.BF16, m=512)[0] != 0             # more than one row tile
    assert grass.cgrad_plan(65528, 512, 128, grass.BF16, m=512)[0] != 0             # ragged K
    assert grass.cgrad_plan(65536, 512, 128, grass.BF16, grass.DY_MxT, m=512)[0] != 0
    for option, value in ((grass.TEST_NO_NARROW_GATHER, 1), (grass.TEST_GEMM_TILE, 128)):
        grass.set_test_option(option, value)
        try:
            assert grass.cgrad_plan(65536, 512, 128, grass.BF16, m=512) == (128, 94)
        finally:
            grass.set_test_option(option, 0)
    grass.set_test_option(grass.TEST_MAX_K_SLICES, 9)
    try:
        assert grass.cgrad_plan(65536, 512, 128, grass.BF16, m=512) == (0, 9)
    finally:
        grass.set_test_option(grass.TEST_MAX_K_SLICES, 0)
    L = grass.lib()
    assert L.grass_set_test_option(17, 1) == grass.ERR_DTYPE
    t, k = C.c_int(0), C.c_int(0)
    assert L.grass_cgrad_plan(64, 0, 64, 8, 1, grass.BF16, 0, None, C.byref(k)) == grass.ERR_NULL
    assert L.grass_cgrad_plan(-1, 0, 64, 8, 1, grass.BF16, 0, C.byref(t), C.byref(k)) == grass.ERR_SHAPE
    assert L.grass_cgrad_plan(64, 0, 64, 8, 0, grass.BF16, 0, C.byref(t), C.byref(k)) == grass.ERR_SHAPE
    assert L.grass_cgrad_plan(64, 0, 64, 8, 1, 7, 0, C.byref(t), C.byref(k)) == grass.ERR_DTYPE


def test_grad_row_stats_validation():
    L = grass.lib()
    f = L.grass_grad_row_stats
    assert f(None, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, FAKE, FAKE, 1 << 30, None) == grass.ERR_NULL
    assert f(FAKE, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, None, FAKE, 1 << 30, None) == grass.ERR_NULL
    assert f(FAKE, 0, 63, FAKE, 32, grass.BF16, 128, 64, 32, FAKE, FAKE, 1 << 30, None) == grass.ERR_SHAPE
    assert f(FAKE, 0, 64, FAKE, 32, 9, 128, 64, 32, FAKE, FAKE, 1 << 30, None) == grass.ERR_DTYPE
    assert f(FAKE, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, FAKE, None, 1 << 30, None) == grass.ERR_WORKSPACE
    assert f(FAKE, 0, 64, FAKE, 32, grass.BF16, 128, 64, 32, FAKE, FAKE, 64, None) == grass.ERR_WORKSPACE


def test_missing_library_is_an_error(monkeypatch):
    monkeypatch.setattr(grass, "_lib", None)
    monkeypatch.setattr(grass, "LIB_PATH", "/nonexistent/libgrass.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        grass.lib()
