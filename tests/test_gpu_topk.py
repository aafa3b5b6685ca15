"""GPU parity of the top-k sparsifier (Sec. "Comparison to meProp") against the CPU oracle: codes, statistics and the
tile-sparse format, bit-exact, on every kernel variant of the selection (one wavefront per vector with 4/16/64 keys per
lane, sixteen wavefronts with 16/64 keys per lane, vectors too long for registers), with ties, special values and the
degenerate k; then the products on its output against the oracle's products on the oracle's codes."""
import numpy as np
import pytest
import torch

import paper_2004_04729_amd as dbp
from oracle import oracle as O
from gpu_util import check_products

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_topk(delta, rows, cols, vec_rows, k, step, with_format=True):
    d = torch.from_numpy(np.ascontiguousarray(delta, dtype=np.float32).reshape(-1)).to(DEV)
    codes = torch.full((rows * cols,), 99, dtype=torch.int8, device=DEV)
    L = dbp.format_layout(rows, cols)
    fmt = torch.full((L["total_bytes"],), 0xFF, dtype=torch.uint8, device=DEV) if with_format else None
    st = torch.full((32,), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.full((dbp.topk_workspace_bytes(rows, vec_rows),), 0xAB, dtype=torch.uint8, device=DEV)
    dbp.topk_quantize(d, rows, cols, vec_rows, k, step, codes, ws, fmt, st, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    out = {"codes": codes.cpu().numpy().reshape(rows, cols), "stats": dbp.Stats.from_tensor(st), "codes_dev": codes, "fmt_dev": fmt}
    if with_format:
        raw = fmt.cpu().numpy()
        nt = L["n_tiles"]
        out["bitmap"] = raw[L["bitmap_offset"]:L["bitmap_offset"] + nt * 32].view(np.uint64).reshape(nt, 4)
        out["tile_nnz"] = raw[L["tile_nnz_offset"]:L["tile_nnz_offset"] + nt * 2].view(np.uint16)
        out["entries"] = raw[L["entries_offset"]:L["entries_offset"] + nt * 512].view(np.uint16).reshape(nt, 256)
    return out


def check(delta, rows, cols, vec_rows, k, step, with_format=True):
    got = run_topk(delta, rows, cols, vec_rows, k, step, with_format)
    ref, st = O.topk_quantize(np.asarray(delta, dtype=np.float32).reshape(rows // vec_rows, vec_rows * cols), k, step)
    ref = ref.reshape(rows, cols)
    bad = int((got["codes"] != ref).sum())
    assert bad == 0, "codes differ at %d of %d elements" % (bad, ref.size)
    s = got["stats"]
    assert (s.nnz, s.n_saturated, s.n_nonfinite, s.max_abs_code) == (st.nnz, st.n_saturated, st.n_nonfinite, st.max_abs_code)
    if with_format:
        bm, tn, en = O.tile_format(ref, rows, cols)
        assert np.array_equal(got["bitmap"], bm) and np.array_equal(got["tile_nnz"], tn)
        used = np.arange(256)[None, :] < tn[:, None].astype(np.int64)
        assert np.array_equal(got["entries"][used], en[used])
    return got, ref


# (rows, cols, vec_rows, k): vector lengths on both sides of every variant's limit (256, 1024, 4096, 16384, 65536)
CASES = [(1, 1, 1, 1), (5, 3, 1, 2), (9, 256, 1, 10), (7, 257, 1, 25), (300, 500, 1, 30), (13, 1024, 1, 100), (6, 1025, 1, 1),
         (5, 4096, 1, 400), (3, 4097, 1, 37), (16, 16384, 1, 1000), (2, 16385, 1, 500), (3, 65536, 1, 2000), (2, 70001, 1, 3000),
         (12, 196, 4, 50), (64, 49, 16, 7), (6, 3136, 3, 900), (8, 12544, 8, 5000),
         (2100, 300, 1, 20), (2048, 1025, 1, 40), (2052, 2049, 1, 300)]        # many vectors: one wavefront each (16 / 64 keys per lane)


@pytest.mark.parametrize("rows,cols,vec_rows,k", CASES)
def test_codes_stats_and_format_match_oracle(rows, cols, vec_rows, k):
    rng = np.random.default_rng(rows * 131 + cols)
    d = (rng.laplace(0, 1e-3, size=(rows, cols)) * rng.uniform(0.1, 10.0, size=(rows, 1))).astype(np.float32)
    step = float(np.float32(np.abs(d).max() / 127))
    check(d, rows, cols, vec_rows, k, step)
    check(d, rows, cols, vec_rows, k, step * 8, with_format=False)


def test_ties_zeros_and_special_values():
    rng = np.random.default_rng(3)
    d = (rng.integers(-6, 7, size=(40, 700)) * 0.125).astype(np.float32)          # 13 distinct magnitudes: ties everywhere
    d[:, ::3] = 0.0
    d[0, :6] = [np.inf, -np.inf, np.nan, -0.0, 1e-42, 3e38]
    d[1, :] = 0.0                                                                  # an all-zero vector
    d[2, :] = np.nan
    d[3, :5] = [1e-45, -1e-45, 2e-45, 1e-38, -1e-38]                               # subnormal magnitudes order like the others
    for k in (1, 2, 50, 233, 234, 699, 700):
        check(d, 40, 700, 1, k, 0.125)
    check(d, 40, 700, 1, 5, 1e-3)                                                   # saturating survivors
    check(d, 40, 700, 40, 1000, 0.125)                                              # one long vector (28000 elements)


@pytest.mark.parametrize("k", [0, -3, 500, 501, 10 ** 12])
def test_degenerate_k(k):
    rng = np.random.default_rng(4)
    d = rng.standard_normal((33, 500)).astype(np.float32)
    got, ref = check(d, 33, 500, 1, k, 0.05)
    if k <= 0:
        assert not got["codes"].any()


def test_vec_rows_and_shape_errors():
    d = torch.zeros(12 * 100, device=DEV)
    codes = torch.zeros(12 * 100, dtype=torch.int8, device=DEV)
    ws = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    for vec_rows in (0, -1, 5, 24):
        with pytest.raises(dbp.DbpError):
            dbp.topk_quantize(d, 12, 100, vec_rows, 3, 0.1, codes, ws)
    with pytest.raises(dbp.DbpError):
        dbp.topk_quantize(d, 12, 100, 1, 3, 0.0, codes, ws)
    with pytest.raises(dbp.DbpError):
        dbp.topk_quantize(d, 12, 100, 1, 3, 0.1, codes, None)
    assert dbp.topk_workspace_bytes(12, 5) == 0 and dbp.topk_workspace_bytes(12, 4) == 256


def test_products_on_top_k_codes_fc_layer():
    # the sparsifier feeds the same product kernels: 5 % of each example's gradient survives, 256 x 1024 x 2048 layer
    rng = np.random.default_rng(12)
    B, n_in, n_out, k = 256, 1024, 2048, 102
    d = rng.laplace(0, 1e-3, size=(B, n_out)).astype(np.float32)
    W = (rng.standard_normal((n_out, n_in)) * 0.03).astype(np.float32)
    X = np.maximum(rng.standard_normal((B, n_in)), 0).astype(np.float32)
    step = float(np.float32(np.abs(d).max() / 127))
    got, ref = check(d, B, n_out, 1, k, step)
    assert 0 < got["stats"].nnz <= B * k
    dX_ref, dW_ref, _ = O.linear_backward(W, X, codes=ref, step=step)
    Wd, Xd = torch.from_numpy(W).to(DEV), torch.from_numpy(X).to(DEV)
    for path in (dbp.PATH_MFMA, dbp.PATH_GATHER):
        dX = torch.empty((B, n_in), device=DEV)
        dW = torch.empty((n_out, n_in), device=DEV)
        ws = torch.empty(dbp.linear_workspace_bytes(B, n_in, n_out), dtype=torch.uint8, device=DEV)
        dbp.linear_products(got["codes_dev"], got["fmt_dev"], step, Wd, Xd, dbp.F32, B, n_in, n_out, dX, dW, ws, path,
                            torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        # the products' tolerance: 1e-4 of the sum of the magnitudes of the terms, as for the dithered codes
        absX = step * np.abs(ref.astype(np.float64)) @ np.abs(W.astype(np.float64))
        absW = step * np.abs(ref.astype(np.float64)).T @ np.abs(X.astype(np.float64))
        check_products(dX.cpu().numpy(), dX_ref, absX, "top-k dX path %d" % path)
        check_products(dW.cpu().numpy(), dW_ref, absW, "top-k dW path %d" % path)


@pytest.mark.parametrize("vec_rows", [1, 12])
def test_products_on_top_k_codes_conv_layer(vec_rows):
    # top-k per feature-map plane (vec_rows = 1) or per example (vec_rows = K) of a small convolution's gradient; the
    # codes and the format then feed both kernel families (the gather kernels read the format's entries)
    rng = np.random.default_rng(21 + vec_rows)
    N, C, H, K = 6, 10, 14, 12
    d = rng.laplace(0, 1e-3, size=(N, K, H, H)).astype(np.float32)
    W = (rng.standard_normal((K, C, 3, 3)) * 0.1).astype(np.float32)
    X = np.maximum(rng.standard_normal((N, C, H, H)), 0).astype(np.float32)
    step = float(np.float32(np.abs(d).max() / 127))
    k = 12 if vec_rows == 1 else 150
    got, ref = check(d.reshape(N * K, H * H), N * K, H * H, vec_rows, k, step)
    ref4 = ref.reshape(N, K, H, H)
    dX_ref, dW_ref, _ = O.conv2d_backward(W, X, codes=ref4, step=step, stride=1, pad=1)
    aX, aW, _ = O.conv2d_backward(np.abs(W), np.abs(X), codes=np.abs(ref4), step=step, stride=1, pad=1)
    Wd, Xd = torch.from_numpy(W).to(DEV), torch.from_numpy(X).to(DEV)
    for path in (dbp.PATH_MFMA, dbp.PATH_GATHER):
        dX = torch.full(X.shape, float("nan"), device=DEV)
        dW = torch.full(W.shape, float("nan"), device=DEV)
        ws = torch.empty(dbp.conv2d_workspace_bytes(N, C, H, H, K, 3, 3, 1, 1), dtype=torch.uint8, device=DEV)
        dbp.conv2d_products(got["codes_dev"], got["fmt_dev"], step, Wd, Xd, dbp.F32, N, C, H, H, K, 3, 3, 1, 1, dX, dW, ws, path,
                            torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        check_products(dX.cpu().numpy(), dX_ref, aX, "top-k conv dX path %d" % path)
        check_products(dW.cpu().numpy(), dW_ref, aW, "top-k conv dW path %d" % path)
