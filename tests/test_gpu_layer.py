"""GPU parity of Algorithm 1 on the device (sigma = std(delta_z), Delta = s*sigma), of the rectifier's derivative
applied on load (delta_z = delta_a (.) f'(z)) and of the bias gradient, against the CPU oracle."""
import numpy as np
import pytest

import workloads
from workloads import LinearProblem, ConvProblem

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _gpu_step(delta, act, s):
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import stream
    n = delta.size
    out = torch.full((2,), float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(dbp.step_size_workspace_bytes(n), dtype=torch.uint8, device="cuda:0")
    dbp.step_size(_dev(delta), None if act is None else _dev(act), n, s, out, ws, stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("size", [1, 15, 16, 17, 255, 256, 4095, 4096, 4097, 65536 + 3, 70001, (1 << 20) + 77])
def test_step_size_matches_oracle_bit_for_bit(size):
    from oracle import oracle as O
    rng = np.random.default_rng(size)
    d = rng.laplace(0, 1e-3, size=size).astype(np.float32)
    got = _gpu_step(d, None, 8.0)
    step, _ = O.step_size(d, 8.0)
    assert got[0] == np.float32(step)
    if step > 0:
        assert got[1] == np.float32(1.0) / np.float32(step)
    else:
        assert got[1] == 0.0
    # unaligned start (the tensor is a slice): same definition, same bits
    if size > 3:
        import torch
        import paper_2004_04729_amd as dbp
        from gpu_util import stream
        buf = _dev(np.concatenate([np.zeros(3, np.float32), d]))
        out = torch.zeros(2, dtype=torch.float32, device="cuda:0")
        ws = torch.empty(dbp.step_size_workspace_bytes(size), dtype=torch.uint8, device="cuda:0")
        dbp.step_size(buf[3:], None, size, 8.0, out, ws, stream())
        torch.cuda.synchronize()
        assert out.cpu().numpy()[0] == np.float32(step)


def test_step_size_laws_mask_and_degenerate_layers():
    from oracle import oracle as O
    rng = np.random.default_rng(11)
    # heavy-tailed mixture, non-zero mean, rectifier mask
    d = (workloads.laplace_mixture(rng, (300, 777)) + 3e-4).astype(np.float32)
    z = rng.standard_normal(d.shape).astype(np.float32)
    got = _gpu_step(d, z, 4.0)
    assert got[0] == np.float32(O.step_size(O.relu_backward(d, z), 4.0)[0])
    # order sensitivity: the values of the oracle's tree pin (sum of squares 2^54 + 16 in tree order)
    x = np.array([2.0 ** 27] + [1.0] * 31, dtype=np.float32)
    assert _gpu_step(x, None, 1.0)[0] == np.float32(O.step_size(x, 1.0)[0])
    y = np.array([2.0 ** 27] + [1.0] * (15 + 16 * 16), dtype=np.float32)
    assert _gpu_step(y, None, 1.0)[0] == np.float32(O.step_size(y, 1.0)[0])
    # degenerate layers: constant gradient (sigma = 0), everything masked, non-finite gradient -> {0, 0}
    assert _gpu_step(np.full(5000, 0.25, np.float32), None, 4.0).tolist() == [0.0, 0.0]
    assert _gpu_step(d, -np.abs(z), 4.0).tolist() == [0.0, 0.0]
    bad = d.copy()
    bad[7, 7] = np.inf
    assert _gpu_step(bad, None, 4.0).tolist() == [0.0, 0.0]


def _run_nsd_ex(delta, act, rows, cols, step, seed, mode, blen, step_dev=None, with_format=True):
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import stream
    codes = torch.full((rows, cols), 99, dtype=torch.int8, device="cuda:0")
    L = dbp.format_layout(rows, cols)
    fmt = torch.empty(L["total_bytes"], dtype=torch.uint8, device="cuda:0") if with_format else None
    st = torch.full((32,), 0xEE, dtype=torch.uint8, device="cuda:0")
    sums = torch.full((blen,), -12345, dtype=torch.int64, device="cuda:0")
    grad = torch.full((blen,), float("nan"), dtype=torch.float32, device="cuda:0")
    dbp.nsd_quantize_ex(_dev(delta), rows, cols, step, seed, 0, codes, fmt, st, act=None if act is None else _dev(act),
                        step_dev=step_dev, bias_sums=sums, bias_grad=grad, bias_mode=mode, bias_len=blen, stream=stream())
    torch.cuda.synchronize()
    return codes.cpu().numpy(), sums.cpu().numpy(), grad.cpu().numpy(), dbp.Stats.from_tensor(st)


@pytest.mark.parametrize("rows,cols", [(1, 1), (7, 5), (64, 300), (33, 257), (256, 1000), (5, 4099)])
@pytest.mark.parametrize("with_format", [True, False])
def test_fused_mask_and_bias_per_column(rows, cols, with_format):
    import paper_2004_04729_amd as dbp
    from oracle import oracle as O
    rng = np.random.default_rng(rows * 131 + cols)
    d = rng.laplace(0, 1e-3, size=(rows, cols)).astype(np.float32)
    z = rng.standard_normal((rows, cols)).astype(np.float32)
    z.reshape(-1)[::17] = -0.0
    z.reshape(-1)[3::29] = np.nan
    step = float(np.float32(4e-3))
    codes, sums, grad, st = _run_nsd_ex(d, z, rows, cols, step, 5, dbp.BIAS_PER_COLUMN, cols, with_format=with_format)
    k_ref, st_ref = O.nsd(O.relu_backward(d, z), step, 5)
    assert np.array_equal(codes, k_ref)
    assert (st.nnz, st.n_saturated, st.n_nonfinite, st.max_abs_code) == (st_ref.nnz, st_ref.n_saturated, st_ref.n_nonfinite, st_ref.max_abs_code)
    s_ref, g_ref = O.bias_grad(k_ref, rows, cols, True, cols, step)
    assert np.array_equal(sums, s_ref)
    assert np.array_equal(grad, g_ref)


@pytest.mark.parametrize("rows,cols", [(5000, 1700), (33001, 520), (66000, 1030), (530003, 257)])
def test_bias_per_column_on_tall_matrices_walks_the_columns(rows, cols):
    # from 32768 tiles on, a pass without the format keeps the column sums in registers over runs of 2 .. 64 rows of one
    # 256-column segment (here 2, 6, 20 and 64 rows; the last three with rows past the tensor in the last run)
    import paper_2004_04729_amd as dbp
    from oracle import oracle as O
    rng = np.random.default_rng(rows + cols)
    d = rng.laplace(0, 1e-3, size=(rows, cols)).astype(np.float32)
    z = rng.standard_normal((rows, cols)).astype(np.float32)
    step = float(np.float32(6e-3))
    codes, sums, grad, st = _run_nsd_ex(d, z, rows, cols, step, 9, dbp.BIAS_PER_COLUMN, cols, with_format=False)
    k_ref, st_ref = O.nsd(O.relu_backward(d, z), step, 9)
    assert np.array_equal(codes, k_ref)
    assert (st.nnz, st.n_saturated, st.n_nonfinite, st.max_abs_code) == (st_ref.nnz, st_ref.n_saturated, st_ref.n_nonfinite, st_ref.max_abs_code)
    s_ref, g_ref = O.bias_grad(k_ref, rows, cols, True, cols, step)
    assert np.array_equal(sums, s_ref)
    assert np.array_equal(grad, g_ref)


@pytest.mark.parametrize("N,K,PQ", [(1, 1, 1), (3, 5, 49), (4, 24, 196), (2, 7, 1024), (6, 3, 300)])
def test_fused_mask_and_bias_per_channel(N, K, PQ):
    import paper_2004_04729_amd as dbp
    from oracle import oracle as O
    rng = np.random.default_rng(N * 1000 + K * 10 + PQ)
    d = rng.laplace(0, 5e-4, size=(N * K, PQ)).astype(np.float32)
    d[::3] *= 200.0                                               # saturating rows: large channel sums
    a = np.maximum(rng.standard_normal(d.shape), 0).astype(np.float32)      # a = f(z) carries the mask
    step = float(np.float32(2e-3))
    codes, sums, grad, st = _run_nsd_ex(d, a, N * K, PQ, step, 9, dbp.BIAS_PER_ROW_GROUP, K)
    k_ref, st_ref = O.nsd(O.relu_backward(d, a), step, 9)
    assert np.array_equal(codes, k_ref)
    assert st.n_saturated == st_ref.n_saturated and st.nnz == st_ref.nnz
    s_ref, g_ref = O.bias_grad(k_ref, N * K, PQ, False, K, step)
    assert np.array_equal(sums, s_ref)
    assert np.array_equal(grad, g_ref)


def test_quantiser_takes_the_step_from_device_memory():
    import torch
    import paper_2004_04729_amd as dbp
    from oracle import oracle as O
    rng = np.random.default_rng(21)
    d = rng.laplace(0, 1e-3, size=(128, 520)).astype(np.float32)
    step, _ = O.step_size(d, 8.0)
    pair = torch.tensor([step, np.float32(1.0) / np.float32(step)], dtype=torch.float32, device="cuda:0")   # oracle's Delta
    codes, sums, grad, _ = _run_nsd_ex(d, None, 128, 520, 123.0, 3, dbp.BIAS_PER_COLUMN, 520, step_dev=pair)
    k_ref, _ = O.nsd(d, step, 3)
    assert np.array_equal(codes, k_ref)
    assert np.array_equal(grad, O.bias_grad(k_ref, 128, 520, True, 520, step)[1])


def _linear_layer(p, s, act, want_db=True, path=None, x_i8=None):
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import stream
    B, in_, out = p.dims
    i8 = x_i8 is not None
    xd = dbp.I8 if i8 else dbp.F32
    codes = torch.empty((B, out), dtype=torch.int8, device="cuda:0")
    dX = torch.full((B, in_), float("nan"), dtype=torch.float32, device="cuda:0")
    dW = torch.full((out, in_), -77, dtype=torch.int32, device="cuda:0") if i8 else \
        torch.full((out, in_), float("nan"), dtype=torch.float32, device="cuda:0")
    db = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda:0") if want_db else None
    pair = torch.full((2,), float("nan"), dtype=torch.float32, device="cuda:0")
    st = torch.full((32,), 0xEE, dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(dbp.linear_layer_workspace_bytes(B, in_, out, xd), dtype=torch.uint8, device="cuda:0")
    dbp.dithered_linear_layer_backward(_dev(p.delta), None if act is None else _dev(act), _dev(p.W),
                                       _dev(x_i8 if i8 else p.X), xd, B, in_, out, s, p.seed, 0, codes, dX, dW, db, pair, ws, st,
                                       dbp.PATH_AUTO if path is None else path, stream())
    torch.cuda.synchronize()
    return dict(codes=codes.cpu().numpy(), dX=dX.cpu().numpy(), dW=dW.cpu().numpy(), db=None if db is None else db.cpu().numpy(),
                pair=pair.cpu().numpy(), stats=dbp.Stats.from_tensor(st))


# the step size's sum tree: 1, 5, 76, 63 partial sums; 17 (a second level of two groups), 256 (the most the quantiser
# finishes itself) and 269 (finished by the kernel of its own)
@pytest.mark.parametrize("B,in_,out", [(5, 3, 2), (64, 784, 300), (300, 520, 1030), (256, 1024, 1000),
                                       (65, 8, 1024), (1024, 16, 1024), (1100, 64, 1000)])
@pytest.mark.parametrize("path", ["mfma", "gather"])
def test_linear_layer_backward_is_algorithm_1(B, in_, out, path):
    import paper_2004_04729_amd as dbp
    from gpu_util import check_products
    from oracle import oracle as O
    rng = np.random.default_rng(B + in_ + out)
    X = np.maximum(rng.standard_normal((B, in_)), 0).astype(np.float32)
    W = (rng.standard_normal((out, in_)) / np.sqrt(in_)).astype(np.float32)
    da = rng.laplace(0, 1e-3, size=(B, out)).astype(np.float32)
    z = rng.standard_normal((B, out)).astype(np.float32)
    p = LinearProblem("layer_%dx%dx%d" % (B, in_, out), da, W, X, 1.0)
    res = _linear_layer(p, 4.0, z, path=dbp.PATH_MFMA if path == "mfma" else dbp.PATH_GATHER)
    dz = O.relu_backward(da, z)
    step, _ = O.step_size(dz, 4.0)
    assert res["pair"][0] == np.float32(step)
    k_ref, st = O.nsd(dz, step, p.seed)
    assert np.array_equal(res["codes"], k_ref)
    assert (res["stats"].nnz, res["stats"].max_abs_code) == (st.nnz, st.max_abs_code)
    assert np.array_equal(res["db"], O.bias_grad(k_ref, B, out, True, out, step)[1])
    rX, rW, _ = O.linear_backward(W, X, codes=k_ref, step=step)
    aX, aW, _ = O.linear_backward(np.abs(W), np.abs(X), codes=np.abs(k_ref), step=step)
    check_products(res["dX"], rX, aX, p.name + " dX")
    check_products(res["dW"], rW, aW, p.name + " dW")


def test_linear_layer_backward_8bit_and_degenerate():
    from gpu_util import check_products
    from oracle import oracle as O
    rng = np.random.default_rng(2)
    B, in_, out = 96, 200, 260
    W = (rng.standard_normal((out, in_)) / np.sqrt(in_)).astype(np.float32)
    X8 = workloads.int8_relu_uniform(rng, (B, in_))
    da = rng.laplace(0, 1e-3, size=(B, out)).astype(np.float32)
    p = LinearProblem("layer_i8", da, W, X8.astype(np.float32), 1.0)
    res = _linear_layer(p, 2.0, None, x_i8=X8)
    step, _ = O.step_size(da, 2.0)
    k_ref, _ = O.nsd(da, step, p.seed)
    assert np.array_equal(res["codes"], k_ref)
    assert np.array_equal(res["dW"], O.linear_dw_i8(k_ref, X8))           # raw integer sums: no Delta
    rX, _, _ = O.linear_backward(W, p.X, codes=k_ref, step=step, want_dw=False)
    aX, _, _ = O.linear_backward(np.abs(W), p.X, codes=np.abs(k_ref), step=step, want_dw=False)
    check_products(res["dX"], rX, aX, "layer_i8 dX")
    # a layer whose gradient is constant has sigma = 0: zero codes, zero products, zero bias gradient
    p0 = LinearProblem("layer_const", np.full((B, out), 1e-3, np.float32), W, np.abs(p.X), 1.0)
    res = _linear_layer(p0, 4.0, None)
    assert res["pair"].tolist() == [0.0, 0.0]
    assert not res["codes"].any() and not res["dX"].any() and not res["dW"].any() and not res["db"].any()
    assert res["stats"].nnz == 0
    # a gradient with +-Inf or NaN in it has no finite deviation: the same degenerate layer, every code 0 (t = Inf * 0 + u
    # is NaN, and a NaN t quantises to 0 as in the oracle's quantiser), the non-finite inputs counted
    bad = da.copy()
    bad[3, 7], bad[50, 100], bad[95, 259] = np.inf, -np.inf, np.nan
    res = _linear_layer(LinearProblem("layer_inf", bad, W, np.abs(p.X), 1.0), 4.0, None)
    assert res["pair"].tolist() == [0.0, 0.0]
    assert not res["codes"].any() and not res["dX"].any() and not res["dW"].any() and not res["db"].any()
    assert (res["stats"].nnz, res["stats"].n_saturated, res["stats"].n_nonfinite, res["stats"].max_abs_code) == (0, 0, 3, 0)


@pytest.mark.parametrize("case", [(2, 5, 9, 7, 6, 3, 3, 1), (3, 16, 14, 14, 24, 3, 3, 1), (2, 33, 14, 14, 20, 1, 1, 0),
                                  (2, 64, 30, 30, 40, 3, 3, 1), (2, 8, 15, 14, 12, 3, 3, 1, 2), (2, 6, 23, 20, 8, 7, 7, 3, 2)])
@pytest.mark.parametrize("i8", [False, True])
@pytest.mark.parametrize("path", ["auto", "gather"])
def test_conv_layer_backward_is_algorithm_1(case, i8, path):
    _conv_layer_case(case, i8, path, 4.0)


@pytest.mark.parametrize("s,flags", [(4.0, [0, 0, 1]), (60.0, [0, 1, 0])])
def test_conv_layer_backward_through_the_dw_gate(s, flags):
    # a layer large enough to arm the density gate's dW state: the statistics sum that writes the flags also carries the bias
    # gradient, and rides in the dX kernel's weight preparation; at s = 60 (> 98 % zeros) dW comes from the gather kernel
    got = _conv_layer_case((16, 128, 56, 56, 128, 3, 3, 1), False, "auto", s, want_flags=True)
    assert got == flags


def _conv_layer_case(case, i8, path, s_mult, want_flags=False):
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import check_products, stream
    from oracle import oracle as O
    N, C, H, Wd, K, R, S, pad = case[:8]
    stride = case[8] if len(case) > 8 else 1
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    rng = np.random.default_rng(sum(case))
    X = workloads.int8_relu_uniform(rng, (N, C, H, Wd)) if i8 else np.maximum(rng.standard_normal((N, C, H, Wd)), 0).astype(np.float32)
    W = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
    da = rng.laplace(0, 5e-4, size=(N, K, P, Q)).astype(np.float32)
    a = np.maximum(rng.standard_normal((N, K, P, Q)), 0).astype(np.float32)
    xd = dbp.I8 if i8 else dbp.F32
    codes = torch.empty((N, K, P, Q), dtype=torch.int8, device="cuda:0")
    dX = torch.full((N, C, H, Wd), float("nan"), dtype=torch.float32, device="cuda:0")
    dW = torch.full((K, C, R, S), -77, dtype=torch.int32, device="cuda:0") if i8 else \
        torch.full((K, C, R, S), float("nan"), dtype=torch.float32, device="cuda:0")
    db = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda:0")
    pair = torch.zeros(2, dtype=torch.float32, device="cuda:0")
    st = torch.zeros(32, dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(dbp.conv2d_layer_workspace_bytes(N, C, H, Wd, K, R, S, stride, pad, xd), dtype=torch.uint8, device="cuda:0")
    off = dbp.format_layout(N * K, P * Q)["scratch_offset"] + 16384 * 16
    ws[off:off + 12] = 255                                     # the density flags read back as -1 unless a gated call writes them
    dbp.dithered_conv2d_layer_backward(_dev(da), _dev(a), _dev(W), _dev(X), xd, N, C, H, Wd, K, R, S, stride, pad, s_mult, 1, 0,
                                       codes, dX, dW, db, pair, ws, st, dbp.PATH_AUTO if path == "auto" else dbp.PATH_GATHER, stream())
    torch.cuda.synchronize()
    flags = [int(v) for v in ws[off:off + 12].cpu().numpy().view(np.int32)]
    dz = O.relu_backward(da, a)
    step, _ = O.step_size(dz, s_mult)
    assert pair.cpu().numpy()[0] == np.float32(step)
    k_ref, sref = O.nsd(dz, step, 1)
    assert np.array_equal(codes.cpu().numpy(), k_ref)
    assert dbp.Stats.from_tensor(st).nnz == sref.nnz
    assert np.array_equal(db.cpu().numpy(), O.bias_grad(k_ref, N * K, P * Q, False, K, step)[1])
    Xf = X.astype(np.float32)
    rX, rW, _ = O.conv2d_backward(W, Xf, codes=k_ref, step=step, stride=stride, pad=pad)
    aX, aW, _ = O.conv2d_backward(np.abs(W), np.abs(Xf), codes=np.abs(k_ref), step=step, stride=stride, pad=pad)
    check_products(dX.cpu().numpy(), rX, aX, "conv layer dX")
    if i8:
        assert np.array_equal(dW.cpu().numpy(), O.conv2d_dw_i8(k_ref, X, R, S, stride=stride, pad=pad))
    else:
        check_products(dW.cpu().numpy(), rW, aW, "conv layer dW")
    return flags if want_flags else None
