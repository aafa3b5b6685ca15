"""GPU parity of the fully connected backward products (Eqs. (qda),(qdw)) against the CPU oracle."""
import numpy as np
import pytest

import workloads
from workloads import LinearProblem

pytestmark = pytest.mark.gpu


def _problem(B, in_, out, c=4.0, seed=0, x_zero_frac=0.5):
    rng = np.random.default_rng(seed + B * 31 + in_ * 7 + out)
    X = np.maximum(rng.standard_normal((B, in_)), 0).astype(np.float32) if x_zero_frac else \
        rng.standard_normal((B, in_)).astype(np.float32)
    W = (rng.standard_normal((out, in_)) / np.sqrt(in_)).astype(np.float32)
    d = rng.laplace(0, 1e-3, size=(B, out)).astype(np.float32)
    return LinearProblem("t_%dx%dx%d" % (B, in_, out), d, W, X, float(np.float32(c * 1.4142e-3)))


def _check_fp32(p, res):
    from gpu_util import check_products
    from oracle import oracle as O
    k_ref, st = O.nsd(p.delta, p.step, p.seed)
    assert np.array_equal(res["codes"], k_ref)
    if res.get("stats") is not None:          # the fused entry point sums the statistics in the products' launch
        got = res["stats"]
        assert (got.nnz, got.n_saturated, got.n_nonfinite, got.max_abs_code) == \
               (st.nnz, st.n_saturated, st.n_nonfinite, st.max_abs_code)
    rX, rW, _ = O.linear_backward(p.W, p.X, codes=k_ref, step=p.step)
    aX, aW, _ = O.linear_backward(np.abs(p.W), np.abs(p.X), codes=np.abs(k_ref), step=p.step)
    e1 = check_products(res["dX"], rX, aX, p.name + " dX") if res["dX"] is not None else 0
    e2 = check_products(res["dW"], rW, aW, p.name + " dW") if res["dW"] is not None else 0
    return max(e1, e2)


SHAPES = [(1, 1, 1), (5, 3, 2), (37, 301, 129), (64, 784, 300), (300, 520, 1030), (256, 1024, 1000), (257, 130, 33),
          (8, 2000, 515)]


@pytest.mark.parametrize("B,in_,out", SHAPES)
@pytest.mark.parametrize("path", ["mfma", "gather"])
def test_fc_products_match_oracle(B, in_, out, path):
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    p = _problem(B, in_, out)
    res = run_linear(p, path=dbp.PATH_MFMA if path == "mfma" else dbp.PATH_GATHER)
    worst = _check_fp32(p, res)
    assert worst < 1e-4


@pytest.mark.parametrize("path", ["mfma", "gather"])
def test_fc_dense_codes_and_extreme_values(path):
    # small step: dense codes up to +-127, so every bf16 plane and every code magnitude is exercised
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    p = _problem(96, 200, 260, c=0.02, x_zero_frac=0)
    p.W[::3] *= 1e4
    p.W[1::3] *= 1e-6
    res = run_linear(p, path=dbp.PATH_MFMA if path == "mfma" else dbp.PATH_GATHER)
    assert np.abs(res["codes"]).max() == 127
    _check_fp32(p, res)


@pytest.mark.parametrize("path", ["mfma", "gather"])
def test_fc_all_zero_codes_and_single_products(path):
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    pp = dbp.PATH_MFMA if path == "mfma" else dbp.PATH_GATHER
    p = _problem(40, 96, 300)
    p.delta[:] = 0
    res = run_linear(p, path=pp)
    assert not res["codes"].any() and not res["dX"].any() and not res["dW"].any()
    p = _problem(70, 260, 300, c=8.0)
    p.delta[10:50] = 0                       # structured: whole rows of zeros
    p.delta[:, 100:228] = 0                  # and whole column blocks
    _check_fp32(p, run_linear(p, path=pp, want_dw=False))
    _check_fp32(p, run_linear(p, path=pp, want_dx=False))


@pytest.mark.parametrize("B,in_,out", [(5, 3, 2), (37, 301, 129), (256, 520, 300), (1000, 64, 70)])
@pytest.mark.parametrize("path", ["mfma", "gather"])
def test_fc_int8_mode_is_bit_exact(B, in_, out, path):
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    from oracle import oracle as O
    p = _problem(B, in_, out, c=1.0)
    X8 = workloads.int8_relu_uniform(np.random.default_rng(B), (B, in_))
    res = run_linear(p, path=dbp.PATH_MFMA if path == "mfma" else dbp.PATH_GATHER, x_i8=X8)
    k_ref, _ = O.nsd(p.delta, p.step, p.seed)
    assert np.array_equal(res["codes"], k_ref)
    assert np.array_equal(res["dW"], O.linear_dw_i8(k_ref, X8))
    # dX stays fp32 (weights are fp32)
    from gpu_util import check_products
    rX, _, _ = O.linear_backward(p.W, p.X, codes=k_ref, step=p.step, want_dw=False)
    aX, _, _ = O.linear_backward(np.abs(p.W), p.X, codes=np.abs(k_ref), step=p.step, want_dw=False)
    check_products(res["dX"], rX, aX, "int8-mode dX")


def test_fc_results_are_deterministic_and_paths_agree_on_codes():
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    p = _problem(256, 1024, 1000, c=8.0)
    a = run_linear(p, path=dbp.PATH_MFMA)
    b = run_linear(p, path=dbp.PATH_MFMA)
    assert a["dX"].tobytes() == b["dX"].tobytes() and a["dW"].tobytes() == b["dW"].tobytes()
    g = run_linear(p, path=dbp.PATH_GATHER, fused=False)
    assert np.array_equal(g["codes"], a["codes"])


@pytest.mark.parametrize("B,in_,out", [(5, 3, 2), (37, 301, 129), (256, 520, 300)])
def test_dense_baseline_matches_oracle(B, in_, out):
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream, check_products
    from oracle import oracle as O
    p = _problem(B, in_, out)
    dX = torch.empty((B, in_), dtype=torch.float32, device="cuda:0")
    dW = torch.empty((out, in_), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device="cuda:0")
    dbp.dense_linear_backward(dev(p.delta), dev(p.W), dev(p.X), dbp.F32, B, in_, out, dX, dW, ws, stream())
    torch.cuda.synchronize()
    rX, rW, _ = O.linear_backward(p.W, p.X, dense=p.delta)
    aX, aW, _ = O.linear_backward(np.abs(p.W), np.abs(p.X), dense=np.abs(p.delta))
    check_products(dX.cpu().numpy(), rX, aX, "dense dX")
    check_products(dW.cpu().numpy(), rW, aW, "dense dW")


# Shapes that drive the role-specialised kernel (batch and out above 128) through its edges: a batch that is not a
# multiple of 4 (the dW reduction ends inside a window of 32 and inside a dword), ragged row and column tiles, a
# reduction shorter than two windows, many column tiles, out just above the kernel's lower limit.
@pytest.mark.parametrize("B,in_,out", [(258, 260, 200), (1000, 136, 260), (130, 4100, 140), (133, 128, 129), (513, 516, 388)])
def test_fc_large_layer_kernel_edges(B, in_, out):
    from gpu_util import run_linear
    p = _problem(B, in_, out, seed=B + in_)
    _check_fp32(p, run_linear(p))
    _check_fp32(p, run_linear(p, want_dw=False))
    _check_fp32(p, run_linear(p, want_dx=False))


def test_fc_many_items_per_workgroup():
    # 256 x 8192 x 8192: 2048 dW tiles and 64 split dX tiles, about ten work items per workgroup; every element
    from gpu_util import run_linear
    p = _problem(256, 8192, 8192, seed=99, c=8.0)
    _check_fp32(p, run_linear(p))


def test_fc_two_groups_of_unequal_size():
    # 300 x 4096 x 4000: the products run on two groups of workgroups (160 for dX, two splits per tile; 96 for dW), with
    # ragged row tiles, a ragged last K step on both sides and idle workgroups in the first group
    from gpu_util import run_linear
    p = _problem(300, 4096, 4000, seed=41, c=8.0)
    _check_fp32(p, run_linear(p))


def test_config1_and_config2_full_size():
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    for p in [workloads.config1()] + workloads.config2(8.0):
        _check_fp32(p, run_linear(p, path=dbp.PATH_AUTO))


@pytest.mark.parametrize("B,in_,out", [(64, 512, 384), (300, 520, 1030), (33, 70, 129)])
def test_fc_fused_call_reports_statistics(B, in_, out):
    # saturating and non-finite gradients, through the single-call entry point (its statistics are summed
    # inside the products' launch on the fast path, by a launch of their own otherwise)
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    from oracle import oracle as O
    p = _problem(B, in_, out, c=2.0)
    flat = p.delta.reshape(-1)
    flat[::97] = 10.0
    flat[5::211] = -10.0
    flat[7::1013] = np.nan
    flat[11::1999] = np.inf
    res = run_linear(p, path=dbp.PATH_MFMA)
    _, st = O.nsd(p.delta, p.step, p.seed)
    assert st.n_saturated > 0 and st.n_nonfinite > 0 and st.max_abs_code == 127
    _check_fp32(p, res)


def _auto_flag(ws, rows, cols):
    """The density gate's flag of a dithered_* call with DBP_PATH_AUTO (1: the gather kernels ran), read back from the workspace."""
    import paper_2004_04729_amd as dbp
    off = dbp.format_layout(rows, cols)["scratch_offset"] + 16384 * 16
    return int(ws[off:off + 4].cpu().numpy().view(np.int32)[0])


@pytest.mark.parametrize("c,expect", [(8.0, 0), (128.0, 1)])
def test_fc_auto_dispatches_by_density_on_the_device(c, expect):
    # 256 x 4096 x 16384: a layer wide enough that the gather kernels' fixed cost (streaming W, writing dW) is below the
    # matrix-core time, so both kernel families are launched behind the density gate; at 91 % zeros the matrix-core
    # kernels run, at 99.4 % the gather kernels -- decided on the device from the quantiser's nonzero count
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream
    B, in_, out = 256, 4096, 16384
    p = _problem(B, in_, out, seed=5, c=c)
    codes = torch.empty((B, out), dtype=torch.int8, device="cuda:0")
    dX = torch.full((B, in_), float("nan"), dtype=torch.float32, device="cuda:0")
    dW = torch.full((out, in_), float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.zeros(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device="cuda:0")
    ws[dbp.format_layout(B, out)["scratch_offset"] + 16384 * 16] = 77          # stale flag: the call must overwrite it
    d, W, X = dev(p.delta), dev(p.W), dev(p.X)
    for stats in (torch.zeros(32, dtype=torch.uint8, device="cuda:0"), None):
        dbp.dithered_linear_backward(d, W, X, dbp.F32, B, in_, out, p.step, p.seed, 0, codes, dX, dW, ws, stats, dbp.PATH_AUTO, stream())
        torch.cuda.synchronize()
        assert _auto_flag(ws, B, out) == expect
        res = {"codes": codes.cpu().numpy(), "dX": dX.cpu().numpy(), "dW": dW.cpu().numpy(),
               "stats": None if stats is None else dbp.Stats.from_tensor(stats)}
        _check_fp32(p, res)
        dX.fill_(float("nan")); dW.fill_(float("nan"))


def test_fc_auto_leaves_the_gate_out_where_gather_cannot_win():
    # 2048^3: the gather kernels' fixed cost alone exceeds the matrix-core time (measured: 0.13 ms at 99.5 % zeros against
    # 0.093 ms), so AUTO launches the matrix-core family only and the flag word is not written
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream
    B = in_ = out = 2048
    p = _problem(B, in_, out, seed=5, c=128.0)
    codes = torch.empty((B, out), dtype=torch.int8, device="cuda:0")
    dX = torch.empty((B, in_), dtype=torch.float32, device="cuda:0")
    dW = torch.empty((out, in_), dtype=torch.float32, device="cuda:0")
    ws = torch.zeros(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device="cuda:0")
    ws[dbp.format_layout(B, out)["scratch_offset"] + 16384 * 16] = 77
    dbp.dithered_linear_backward(dev(p.delta), dev(p.W), dev(p.X), dbp.F32, B, in_, out, p.step, p.seed, 0, codes, dX, dW, ws, None,
                                 dbp.PATH_AUTO, stream())
    torch.cuda.synchronize()
    assert _auto_flag(ws, B, out) == 77
    _check_fp32(p, {"codes": codes.cpu().numpy(), "dX": dX.cpu().numpy(), "dW": dW.cpu().numpy()})


@pytest.mark.parametrize("B,in_,out", [(256, 516, 260), (300, 1028, 1000), (128, 256, 4100), (520, 260, 64), (1030, 132, 520)])
def test_fc_gather_row_list_kernel_edges(B, in_, out):
    # the LDS-staged gather kernels at their edges: column slabs and row blocks that end inside a tile, reductions that
    # end inside a chunk of 64, code rows that are only 4-byte aligned, several row blocks with a split reduction
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    p = _problem(B, in_, out, seed=B + out, c=6.0)
    _check_fp32(p, run_linear(p, path=dbp.PATH_GATHER))
    _check_fp32(p, run_linear(p, path=dbp.PATH_GATHER, want_dw=False))
    _check_fp32(p, run_linear(p, path=dbp.PATH_GATHER, want_dx=False))
