"""Helpers of the GPU parity tests: run the HIP library through its C ABI binding on torch-owned
device memory and compare with the CPU oracle.  Tolerance for fp32 products (both readings of the
target "max relative error 1e-4, normalised by the row's l1 norm"):
  (i)  |gpu - ref| <= 1e-4 * sum_r |q_r| |w_r|   over the element's own reduction (the stricter one),
  (ii) |gpu - ref| <= 1e-4 * ||ref row||_1,
and an element whose reduction has no nonzero term must be exactly 0.
"""
import numpy as np
import torch

import paper_2004_04729_amd as dbp
from oracle import oracle as O

TOL = 1e-4
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def stream():
    return torch.cuda.current_stream().cuda_stream


def check_products(got, ref, absref, what=""):
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    bound = TOL * absref
    bad = err > bound
    assert not bad.any(), "%s: %d elements outside 1e-4*sum|q||w| (max ratio %.3g)" % (
        what, int(bad.sum()), float((err / np.maximum(absref, 1e-300)).max()))
    assert np.all(got[absref == 0] == 0), what + ": element with an empty reduction is not exactly 0"
    if ref.ndim >= 2:
        r2 = ref.reshape(ref.shape[0], -1)
        l1 = np.abs(r2).sum(axis=1, keepdims=True)
        assert np.all(err.reshape(r2.shape) <= TOL * l1 + 1e-300), what + ": outside 1e-4 * row l1 norm"
    return float((err / np.maximum(absref, 1e-300)).max())


def run_nsd(delta, rows, cols, step, seed, idx_base=0, with_format=True, with_stats=True):
    d = dev(delta.astype(np.float32).reshape(-1))
    codes = torch.full((rows * cols,), 99, dtype=torch.int8, device=DEV)
    L = dbp.format_layout(rows, cols)
    fmt = torch.full((L["total_bytes"],), 0xFF, dtype=torch.uint8, device=DEV) if with_format else None
    st = torch.full((32,), 0xEE, dtype=torch.uint8, device=DEV) if with_stats else None
    dbp.nsd_quantize(d, rows, cols, step, seed, idx_base, codes, fmt, st, stream())
    torch.cuda.synchronize()
    out = {"codes": codes.cpu().numpy().reshape(rows, cols), "layout": L}
    if with_format:
        raw = fmt.cpu().numpy()
        nt = L["n_tiles"]
        out["bitmap"] = raw[L["bitmap_offset"]:L["bitmap_offset"] + nt * 32].view(np.uint64).reshape(nt, 4)
        out["tile_nnz"] = raw[L["tile_nnz_offset"]:L["tile_nnz_offset"] + nt * 2].view(np.uint16)
        out["entries"] = raw[L["entries_offset"]:L["entries_offset"] + nt * 512].view(np.uint16).reshape(nt, 256)
        out["fmt_dev"] = fmt
    if with_stats:
        out["stats"] = dbp.Stats.from_tensor(st)
    out["codes_dev"] = codes
    return out


def check_nsd_against_oracle(delta, rows, cols, step, seed, idx_base=0):
    got = run_nsd(delta, rows, cols, step, seed, idx_base)
    k_ref, st_ref = O.nsd(delta.reshape(-1), step, seed, idx_base)
    k_ref = k_ref.reshape(rows, cols)
    assert np.array_equal(got["codes"], k_ref), "codes differ at %d of %d elements" % (
        int((got["codes"] != k_ref).sum()), k_ref.size)
    s = got["stats"]
    assert (s.nnz, s.n_saturated, s.n_nonfinite, s.max_abs_code) == (
        st_ref.nnz, st_ref.n_saturated, st_ref.n_nonfinite, st_ref.max_abs_code)
    bm, tn, en = O.tile_format(k_ref, rows, cols)
    assert np.array_equal(got["bitmap"], bm), "bitmap differs"
    assert np.array_equal(got["tile_nnz"], tn), "tile counts differ"
    used = np.arange(256)[None, :] < tn[:, None].astype(np.int64)
    if not np.array_equal(got["entries"][used], en[used]):
        bad = np.argwhere((got["entries"] != en) & used)
        t0 = int(bad[0][0])
        raise AssertionError("compacted entries differ in %d slots of %d tiles; first tile %d (nnz %d): gpu %s ref %s" % (
            len(bad), len(set(bad[:, 0].tolist())), t0, int(tn[t0]), got["entries"][t0, :int(tn[t0]) + 1].tolist(),
            en[t0, :int(tn[t0]) + 1].tolist()))
    return got, k_ref


def run_linear(p, path=dbp.PATH_MFMA, x_i8=None, want_dx=True, want_dw=True, fused=True, codes_np=None):
    """Returns dict(codes, dX, dW) as numpy.  x_i8: int8 X for the 8-bit mode."""
    B, in_, out = p.dims
    i8 = x_i8 is not None
    d, W = dev(p.delta), dev(p.W)
    X = dev(x_i8) if i8 else dev(p.X)
    codes = torch.empty((B, out), dtype=torch.int8, device=DEV)
    dX = torch.full((B, in_), float("nan"), dtype=torch.float32, device=DEV) if want_dx else None
    dW = (torch.full((out, in_), -77, dtype=torch.int32, device=DEV) if i8 else
          torch.full((out, in_), float("nan"), dtype=torch.float32, device=DEV)) if want_dw else None
    xd = dbp.I8 if i8 else dbp.F32
    ws = torch.empty(dbp.linear_workspace_bytes(B, in_, out, xd), dtype=torch.uint8, device=DEV)
    st = None
    if fused:
        st = torch.full((32,), 0xEE, dtype=torch.uint8, device=DEV)
        dbp.dithered_linear_backward(d, W, X, xd, B, in_, out, p.step, p.seed, 0, codes, dX, dW, ws, st, path, stream())
    else:
        L = dbp.format_layout(B, out)
        fmt = torch.empty(L["total_bytes"], dtype=torch.uint8, device=DEV)
        if codes_np is not None:
            codes = dev(codes_np)
            dbp.nsd_quantize(d, B, out, p.step, p.seed, 0, torch.empty_like(codes), fmt, None, stream())
        else:
            dbp.nsd_quantize(d, B, out, p.step, p.seed, 0, codes, fmt, None, stream())
        dbp.linear_products(codes, fmt, p.step, W, X, xd, B, in_, out, dX, dW, ws, path, stream())
    torch.cuda.synchronize()
    return {"codes": codes.cpu().numpy(), "dX": None if dX is None else dX.cpu().numpy(),
            "dW": None if dW is None else dW.cpu().numpy(), "stats": None if st is None else dbp.Stats.from_tensor(st)}


def conv_dims(p):
    N, Cc, H, Wd = p.X.shape
    K, _, R, S = p.W.shape
    return N, Cc, H, Wd, K, R, S


def run_conv(p, path=dbp.PATH_MFMA, want_dx=True, want_dw=True):
    N, Cc, H, Wd, K, R, S = conv_dims(p)
    i8 = p.X.dtype == np.int8
    xd = dbp.I8 if i8 else dbp.F32
    d, W, X = dev(p.delta), dev(p.W), dev(p.X)
    codes = torch.empty(p.delta.shape, dtype=torch.int8, device=DEV)
    dX = torch.full(p.X.shape, float("nan"), dtype=torch.float32, device=DEV) if want_dx else None
    dW = (torch.full(p.W.shape, -77, dtype=torch.int32, device=DEV) if i8 else
          torch.full(p.W.shape, float("nan"), dtype=torch.float32, device=DEV)) if want_dw else None
    ws = torch.empty(dbp.conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, p.stride, p.pad, xd), dtype=torch.uint8, device=DEV)
    st = torch.zeros(32, dtype=torch.uint8, device=DEV)
    dbp.dithered_conv2d_backward(d, W, X, xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, p.step, p.seed, 0,
                                 codes, dX, dW, ws, st, path, stream())
    torch.cuda.synchronize()
    return {"codes": codes.cpu().numpy(), "dX": None if dX is None else dX.cpu().numpy(),
            "dW": None if dW is None else dW.cpu().numpy(), "stats": dbp.Stats.from_tensor(st)}
