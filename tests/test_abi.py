"""CPU-only checks of the C ABI: the library loads, exports every function include/dbp.h declares,
and rejects bad arguments before touching the GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

import paper_2004_04729_amd as dbp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, STEP, DTYPE, WORKSPACE, UNSUPPORTED, OVERFLOW, DEVICE = range(9)
FAKE = 0x10000       # a non-NULL, 256-aligned address that is never dereferenced by the checks under test


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dbp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith(("dbp_", "nsd_", "dithered_", "dense_"))})


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"nsd_quantize", "dithered_linear_backward", "dithered_conv2d_backward", "dense_linear_backward",
            "dense_conv2d_backward", "dbp_linear_products", "dbp_conv2d_products", "dbp_format_layout_of",
            "dbp_linear_workspace_bytes", "dbp_conv2d_workspace_bytes", "dbp_status_string",
            "dbp_abi_version"} <= set(names)
    raw = C.CDLL(dbp.lib_path())
    for n in names:
        assert hasattr(raw, n), n


def test_version_and_status_strings():
    assert dbp.abi_version() == 1
    seen = {dbp.status_string(c) for c in range(9)}
    assert len(seen) == 9 and dbp.status_string(99) == "unknown status"


def test_format_layout():
    L = dbp.format_layout(64, 300)
    assert L["tiles_per_row"] == 2 and L["n_tiles"] == 128
    assert L["bitmap_offset"] == 0 and L["tile_nnz_offset"] >= 128 * 32
    assert L["entries_offset"] >= L["tile_nnz_offset"] + 128 * 2
    assert L["total_bytes"] >= L["entries_offset"] + 128 * 512
    assert all(L[k] % 256 == 0 for k in ("tile_nnz_offset", "entries_offset", "total_bytes"))
    with pytest.raises(dbp.DbpError) as e:
        dbp.format_layout(0, 5)
    assert e.value.code == SHAPE


def test_workspace_sizes():
    assert dbp.linear_workspace_bytes(64, 784, 300) > 64 * 300
    assert dbp.linear_workspace_bytes(0, 784, 300) == 0 and dbp.linear_workspace_bytes(64, 784, 300, 7) == 0
    assert dbp.conv2d_workspace_bytes(128, 64, 32, 32, 64, 3, 3, 1, 1) > 128 * 64 * 32 * 32
    assert dbp.conv2d_workspace_bytes(128, 64, 32, 32, 64, 3, 3, 2, 1) > 128 * 64 * 16 * 16      # stride 2: P = Q = 16
    assert dbp.conv2d_workspace_bytes(1, 1, 2, 2, 1, 5, 5, 1, 0) == 0             # kernel larger than input


def _code(fn, *a, **k):
    with pytest.raises(dbp.DbpError) as e:
        fn(*a, **k)
    return e.value.code


def test_nsd_argument_errors():
    q = dbp.nsd_quantize
    assert _code(q, None, 4, 4, 1.0, 1, 0, FAKE) == NULL
    assert _code(q, FAKE, 4, 4, 1.0, 1, 0, None) == NULL
    assert _code(q, FAKE, 0, 4, 1.0, 1, 0, FAKE) == SHAPE
    assert _code(q, FAKE, 4, -1, 1.0, 1, 0, FAKE) == SHAPE
    assert _code(q, FAKE, 1 << 30, 1 << 30, 1.0, 1, 0, FAKE) == SHAPE
    for bad in (0.0, -1.0, float("nan"), float("inf"), 1e-45, 3.4e38):
        assert _code(q, FAKE, 4, 4, bad, 1, 0, FAKE) == STEP
    raw = dbp.lib()
    assert raw.nsd_quantize(FAKE, 4, 4, 1.0, 1, 0, FAKE, FAKE, 16, None, None) == WORKSPACE     # too small
    assert raw.nsd_quantize(FAKE, 4, 4, 1.0, 1, 0, FAKE, FAKE + 8, 1 << 20, None, None) == WORKSPACE  # misaligned


def test_linear_argument_errors():
    f = dbp.lib().dithered_linear_backward
    big = 1 << 30

    def call(delta=FAKE, W=FAKE, X=FAKE, xd=0, B=8, i=8, o=8, step=1.0, dX=FAKE, dW=FAKE, ws=FAKE, wsb=big, path=0):
        return f(delta, W, X, xd, B, i, o, step, 1, 0, None, dX, dW, ws, wsb, None, path, None)

    assert call(delta=None) == NULL and call(W=None) == NULL and call(X=None) == NULL
    assert call(dX=None, dW=None) == NULL
    assert call(B=0) == SHAPE and call(i=-3) == SHAPE and call(o=1 << 31) == SHAPE
    assert call(step=0.0) == STEP
    assert call(xd=5) == DTYPE
    assert call(path=9) == UNSUPPORTED
    assert call(ws=None) == WORKSPACE and call(wsb=100) == WORKSPACE and call(ws=FAKE + 4) == WORKSPACE
    assert call(xd=1, B=140000) == OVERFLOW
    # the gather kernels that serve odd shapes number their workgroups by row: rejected on the host, not at the launch
    assert call(path=2, B=70000) == UNSUPPORTED and call(path=2, o=70000) == UNSUPPORTED
    g = dbp.lib().dense_linear_backward
    assert g(None, FAKE, FAKE, 0, 8, 8, 8, FAKE, FAKE, FAKE, big, None) == NULL
    assert g(FAKE, FAKE, FAKE, 1, 8, 8, 8, FAKE, FAKE, FAKE, big, None) == UNSUPPORTED
    assert g(FAKE, FAKE, FAKE, 0, 8, 8, 8, FAKE, FAKE, FAKE, 10, None) == WORKSPACE
    h = dbp.lib().dbp_linear_products
    assert h(FAKE, None, 1.0, FAKE, FAKE, 0, 8, 8, 8, FAKE, FAKE, FAKE, big, 2, None) == NULL    # gather needs the format
    assert h(None, None, 1.0, FAKE, FAKE, 0, 8, 8, 8, FAKE, FAKE, FAKE, big, 1, None) == NULL


def test_conv_argument_errors():
    f = dbp.lib().dithered_conv2d_backward
    big = 1 << 34

    def call(delta=FAKE, W=FAKE, X=FAKE, xd=0, N=2, Cc=3, H=8, Wd=8, K=4, R=3, S=3, stride=1, pad=1, step=1.0,
             dX=FAKE, dW=FAKE, ws=FAKE, wsb=big, path=0):
        return f(delta, W, X, xd, N, Cc, H, Wd, K, R, S, stride, pad, step, 1, 0, None, dX, dW, ws, wsb, None, path, None)

    assert call(delta=None) == NULL and call(dX=None, dW=None) == NULL
    assert call(N=0) == SHAPE and call(R=9, pad=0, H=4) == SHAPE and call(pad=-1) == SHAPE
    assert call(step=float("nan")) == STEP and call(xd=3) == DTYPE
    assert call(stride=0) == SHAPE and call(path=3) == UNSUPPORTED
    # the gather kernels keep four input planes in LDS and give every tap a lane
    assert call(path=2, H=200, Wd=200) == UNSUPPORTED and call(path=2, R=9, S=9, pad=4, H=16, Wd=16) == UNSUPPORTED
    assert call(wsb=1000) == WORKSPACE
    assert call(xd=1, N=64, H=64, Wd=64) == OVERFLOW
    g = dbp.lib().dense_conv2d_backward
    assert g(FAKE, FAKE, FAKE, 0, 2, 3, 8, 8, 4, 3, 3, 0, 1, FAKE, FAKE, FAKE, big, None) == SHAPE          # stride 0
    assert g(FAKE, FAKE, FAKE, 0, 2, 3, 8, 8, 4, 3, 3, 2, 1, FAKE, FAKE, FAKE, 64, None) == WORKSPACE      # stride 2 is served
    assert g(FAKE, FAKE, None, 0, 2, 3, 8, 8, 4, 3, 3, 1, 1, FAKE, FAKE, FAKE, big, None) == NULL


def test_algorithm1_entry_points_reject_bad_arguments():
    assert dbp.step_size_workspace_bytes(0) == 0 and dbp.step_size_workspace_bytes(1 << 20) >= 2 * 256 * 8
    ws = dbp.step_size_workspace_bytes(4096)
    raw = dbp.lib()
    assert raw.dbp_step_size(None, None, 16, 4.0, FAKE, FAKE, ws, None) == NULL
    assert raw.dbp_step_size(FAKE, None, 16, 4.0, None, FAKE, ws, None) == NULL
    assert raw.dbp_step_size(FAKE, None, 0, 4.0, FAKE, FAKE, ws, None) == SHAPE
    for bad in (0.0, -2.0, float("nan"), float("inf")):
        assert raw.dbp_step_size(FAKE, None, 16, bad, FAKE, FAKE, ws, None) == STEP
    assert raw.dbp_step_size(FAKE, None, 16, 4.0, FAKE, None, ws, None) == WORKSPACE
    assert raw.dbp_step_size(FAKE, None, 16, 4.0, FAKE, FAKE, 8, None) == WORKSPACE
    # extras of the quantiser
    q = dbp.nsd_quantize_ex
    assert _code(q, FAKE, 4, 8, 1.0, 1, 0, FAKE, bias_grad=FAKE) == NULL                          # gradient without sums
    assert _code(q, FAKE, 4, 8, 1.0, 1, 0, FAKE, bias_sums=FAKE, bias_len=7) == SHAPE             # per column: len == cols
    assert _code(q, FAKE, 4, 8, 1.0, 1, 0, FAKE, bias_sums=FAKE, bias_mode=dbp.BIAS_PER_ROW_GROUP, bias_len=3) == SHAPE
    assert _code(q, FAKE, 4, 8, 1.0, 1, 0, FAKE, bias_sums=FAKE, bias_mode=5, bias_len=8) == UNSUPPORTED
    assert _code(q, FAKE, 4, 8, 0.0, 1, 0, FAKE) == STEP                                          # host step still checked ...
    assert _code(q, FAKE, 0, 8, 0.0, 1, 0, FAKE, step_dev=FAKE) == SHAPE                          # ... unless a device step is given
    # whole-layer calls
    wl = dbp.linear_layer_workspace_bytes(8, 16, 12)
    assert wl > dbp.linear_workspace_bytes(8, 16, 12)
    f = dbp.dithered_linear_layer_backward
    assert _code(f, None, None, FAKE, FAKE, dbp.F32, 8, 16, 12, 4.0, 1, 0, None, FAKE, FAKE, None, None, None) == NULL
    assert _code(f, FAKE, None, FAKE, FAKE, dbp.F32, 8, 16, 12, 4.0, 1, 0, None, None, None, None, None, None) == NULL
    assert _code(f, FAKE, None, FAKE, FAKE, dbp.F32, 8, 0, 12, 4.0, 1, 0, None, FAKE, FAKE, None, None, None) == SHAPE
    assert _code(f, FAKE, None, FAKE, FAKE, dbp.F32, 8, 16, 12, 0.0, 1, 0, None, FAKE, FAKE, None, None, None) == STEP
    assert _code(f, FAKE, None, FAKE, FAKE, dbp.F32, 8, 16, 12, 4.0, 1, 0, None, FAKE, FAKE, None, None, None) == WORKSPACE
    wc = dbp.conv2d_layer_workspace_bytes(2, 3, 8, 8, 4, 3, 3, 1, 1)
    assert wc > dbp.conv2d_workspace_bytes(2, 3, 8, 8, 4, 3, 3, 1, 1)
    g = dbp.dithered_conv2d_layer_backward
    assert _code(g, FAKE, None, FAKE, FAKE, dbp.F32, 2, 3, 8, 8, 4, 3, 3, 0, 1, 4.0, 1, 0, None, FAKE, FAKE, None, None, None) == SHAPE
    assert _code(g, FAKE, None, FAKE, FAKE, dbp.F32, 2, 3, 8, 8, 4, 3, 3, 1, 1, -1.0, 1, 0, None, FAKE, FAKE, None, None, None) == STEP
    assert _code(g, FAKE, None, FAKE, FAKE, dbp.F32, 2, 3, 8, 8, 4, 3, 3, 1, 1, 4.0, 1, 0, None, FAKE, FAKE, None, None, None) == WORKSPACE


def test_full_8bit_entry_points_reject_bad_arguments():
    raw = dbp.lib()
    wq = dbp.quantize_int8_workspace_bytes(1000)
    assert wq >= 256 and dbp.quantize_int8_workspace_bytes(0) == 0
    assert raw.dbp_quantize_int8(None, 16, FAKE, FAKE, FAKE, wq, None) == NULL
    assert raw.dbp_quantize_int8(FAKE, 16, None, FAKE, FAKE, wq, None) == NULL
    assert raw.dbp_quantize_int8(FAKE, 16, FAKE, None, FAKE, wq, None) == NULL
    assert raw.dbp_quantize_int8(FAKE, 0, FAKE, FAKE, FAKE, wq, None) == SHAPE
    assert raw.dbp_quantize_int8(FAKE, 16, FAKE, FAKE, None, wq, None) == WORKSPACE
    assert raw.dbp_quantize_int8(FAKE, 16, FAKE, FAKE, FAKE, 8, None) == WORKSPACE
    f = dbp.dithered_linear_backward_q8
    assert _code(f, None, FAKE, FAKE, 8, 16, 12, 1.0, 1, 0, None, FAKE, FAKE, None) == NULL
    assert _code(f, FAKE, None, FAKE, 8, 16, 12, 1.0, 1, 0, None, FAKE, None, None) == NULL           # dX32 needs W8
    assert _code(f, FAKE, FAKE, None, 8, 16, 12, 1.0, 1, 0, None, None, FAKE, None) == NULL           # dW32 needs X8
    assert _code(f, FAKE, FAKE, FAKE, 8, 16, 12, 1.0, 1, 0, None, None, None, None) == NULL
    assert _code(f, FAKE, FAKE, FAKE, 8, 0, 12, 1.0, 1, 0, None, FAKE, FAKE, None) == SHAPE
    assert _code(f, FAKE, FAKE, FAKE, 8, 16, 12, 0.0, 1, 0, None, FAKE, FAKE, None) == STEP
    assert _code(f, FAKE, FAKE, FAKE, 8, 16, 140000, 1.0, 1, 0, None, FAKE, None, None) == OVERFLOW  # 140000*127*127 >= 2^31
    assert _code(f, FAKE, FAKE, FAKE, 140000, 16, 12, 1.0, 1, 0, None, None, FAKE, None) == OVERFLOW
    assert _code(f, FAKE, FAKE, FAKE, 8, 16, 12, 1.0, 1, 0, None, FAKE, FAKE, None) == WORKSPACE
    g = dbp.dithered_conv2d_backward_q8
    assert _code(g, FAKE, FAKE, FAKE, 2, 3, 8, 8, 4, 3, 3, 0, 1, 1.0, 1, 0, None, FAKE, FAKE, None) == SHAPE
    assert _code(g, FAKE, FAKE, FAKE, 2, 3, 8, 8, 4, 3, 3, 1, 1, -1.0, 1, 0, None, FAKE, FAKE, None) == STEP
    assert _code(g, FAKE, FAKE, FAKE, 2, 3, 8, 8, 20000, 3, 3, 1, 1, 1.0, 1, 0, None, FAKE, None, None) == OVERFLOW
    assert _code(g, FAKE, FAKE, FAKE, 2, 3, 8, 8, 4, 3, 3, 1, 1, 1.0, 1, 0, None, FAKE, FAKE, None) == WORKSPACE


def test_bench_refuses_more_than_one_gpu():
    # the hot path has no collectives: the bench says so instead of pretending to scale
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
