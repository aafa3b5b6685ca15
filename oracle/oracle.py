"""ctypes front end of the plain-C oracle in ``dbp_oracle.c`` -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this.  It marshals numpy arrays into the C functions and holds no arithmetic
of the method itself; the C file cites the passages of the paper each function follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dbp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
GCC_FLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *GCC_FLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Stats(C.Structure):
    _fields_ = [("nnz", C.c_uint64), ("n_saturated", C.c_uint64), ("n_nonfinite", C.c_uint64),
                ("max_abs_code", C.c_int32), ("pad_", C.c_int32)]


@dataclass
class Stats:
    nnz: int
    n_saturated: int
    n_nonfinite: int
    max_abs_code: int


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.dbp_oracle_hash.restype = C.c_uint32
        L.dbp_oracle_hash.argtypes = [C.c_uint64, C.c_uint64]
        L.dbp_oracle_dither_u.restype = C.c_float
        L.dbp_oracle_dither_u.argtypes = [C.c_uint64, C.c_uint64]
        L.dbp_oracle_linear_dw_i8.restype = C.c_int64
        L.dbp_oracle_conv2d_dw_i8.restype = C.c_int64
        L.dbp_oracle_max_threads.restype = C.c_int
        L.dbp_oracle_step_size.restype = C.c_float
    return _lib


def max_threads() -> int:
    return int(lib().dbp_oracle_max_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int8)


def hash32(seed: int, counter: int) -> int:
    return int(lib().dbp_oracle_hash(C.c_uint64(seed), C.c_uint64(counter)))


def keys(seed: int):
    k0, k1 = C.c_uint32(), C.c_uint32()
    lib().dbp_oracle_keys(C.c_uint64(seed), C.byref(k0), C.byref(k1))
    return k0.value, k1.value


def dither_u(seed: int, g: int) -> float:
    return float(lib().dbp_oracle_dither_u(C.c_uint64(seed), C.c_uint64(g)))


def nsd(delta, step: float, seed: int, idx_base: int = 0):
    """Codes (int8, same shape as delta) and Stats for Eq. (nsd) applied elementwise."""
    d = _f32(delta)
    codes = np.empty(d.shape, dtype=np.int8)
    st = _Stats()
    lib().dbp_oracle_nsd(_p(d), C.c_int64(d.size), C.c_float(step), C.c_uint64(seed),
                         C.c_uint64(idx_base), _p(codes), C.byref(st))
    return codes, Stats(st.nnz, st.n_saturated, st.n_nonfinite, st.max_abs_code)


def topk_threshold(delta, k: int):
    """k-th largest magnitude of every row of the 2-D `delta` (NaN when k <= 0): top-k sparsifier of Sec. "Comparison to meProp"."""
    d = _f32(delta)
    assert d.ndim == 2
    thr = np.empty(d.shape[0], dtype=np.float32)
    lib().dbp_oracle_topk_threshold(_p(d), C.c_int64(d.shape[0]), C.c_int64(d.shape[1]), C.c_int64(k), _p(thr))
    return thr


def topk_quantize(delta, k: int, step: float):
    """Codes and Stats of the top-k sparsifier: per row of the 2-D `delta` the elements whose magnitude reaches the k-th
    largest are rounded to the nearest level of step `step` (Eq. (nsd) without dither), the others are 0."""
    d = _f32(delta)
    assert d.ndim == 2
    codes = np.empty(d.shape, dtype=np.int8)
    st = _Stats()
    lib().dbp_oracle_topk_quantize(_p(d), C.c_int64(d.shape[0]), C.c_int64(d.shape[1]), C.c_int64(k), C.c_float(step),
                                   _p(codes), C.byref(st))
    return codes, Stats(st.nnz, st.n_saturated, st.n_nonfinite, st.max_abs_code)


def step_size(delta, s: float):
    """(Delta = s*std(delta) as fp32, sigma as fp64): Algorithm 1, population std, radix-16 summation tree."""
    d = _f32(delta)
    sigma = C.c_double(0.0)
    step = lib().dbp_oracle_step_size(_p(d), C.c_int64(d.size), C.c_float(s), C.byref(sigma))
    return float(step), float(sigma.value)


def relu_backward(delta_a, act):
    """delta_z = delta_a (.) f'(z) for the rectifier: delta_a where act > 0, +0.0 elsewhere (exact)."""
    d, a = _f32(delta_a), _f32(act)
    assert d.shape == a.shape
    out = np.empty(d.shape, dtype=np.float32)
    lib().dbp_oracle_relu_backward(_p(d), _p(a), C.c_int64(d.size), _p(out))
    return out


def bias_grad(codes, rows: int, cols: int, per_column: bool, length: int, step: float):
    """(int64 code sums [length], fp32 bias gradient Delta*sum [length]); see dbp_oracle_bias_grad."""
    k = _i8(codes)
    assert k.size == rows * cols
    sums = np.zeros(length, dtype=np.int64)
    grad = np.zeros(length, dtype=np.float32)
    lib().dbp_oracle_bias_grad(_p(k), C.c_int64(rows), C.c_int64(cols), C.c_int(0 if per_column else 1),
                               C.c_int64(length), C.c_float(step), _p(sums), _p(grad))
    return sums, grad


def tile_format(codes, rows: int, cols: int):
    """(bitmap u64 [tiles,4], tile_nnz u16 [tiles], entries u16 [tiles,256]); unused slots are 0xFFFF."""
    k = _i8(codes)
    assert k.size == rows * cols
    tiles = rows * ((cols + 255) // 256)
    bitmap = np.zeros((tiles, 4), dtype=np.uint64)
    tile_nnz = np.zeros(tiles, dtype=np.uint16)
    entries = np.full((tiles, 256), 0xFFFF, dtype=np.uint16)
    lib().dbp_oracle_tile_format(_p(k), C.c_int64(rows), C.c_int64(cols), _p(bitmap), _p(tile_nnz), _p(entries))
    return bitmap, tile_nnz, entries


def _q_args(codes, dense, step):
    if (codes is None) == (dense is None):
        raise ValueError("pass exactly one of codes / dense")
    return _i8(codes), _f32(dense), C.c_double(float(step) if codes is not None else 0.0)


def linear_backward(W, X, *, codes=None, dense=None, step=0.0, want_dx=True, want_dw=True, threads=None):
    """fp64 (dX [B,in], dW [out,in], macs) of Eqs. (qda),(qdw); W [out,in], X [B,in], q [B,out]."""
    W, X = _f32(W), _f32(X)
    out, in_ = W.shape
    B = X.shape[0]
    k, d, s = _q_args(codes, dense, step)
    assert (k if k is not None else d).shape == (B, out) and X.shape == (B, in_)
    dX = np.empty((B, in_), dtype=np.float64) if want_dx else None
    dW = np.empty((out, in_), dtype=np.float64) if want_dw else None
    macs = C.c_uint64(0)
    lib().dbp_oracle_linear_backward(_p(k), _p(d), s, _p(W), _p(X), C.c_int64(B), C.c_int64(in_), C.c_int64(out),
                                     _p(dX), _p(dW), C.c_int(threads or max_threads()), C.byref(macs))
    return dX, dW, macs.value


def linear_dw_i8(codes, X8, threads=None):
    """Exact int32 dW32 [out,in] = codes^T . X8; raises if an element leaves int32."""
    k, x = _i8(codes), _i8(X8)
    B, out = k.shape
    in_ = x.shape[1]
    assert x.shape[0] == B
    dW = np.empty((out, in_), dtype=np.int32)
    bad = lib().dbp_oracle_linear_dw_i8(_p(k), _p(x), C.c_int64(B), C.c_int64(in_), C.c_int64(out), _p(dW),
                                        C.c_int(threads or max_threads()))
    if bad:
        raise OverflowError("%d int32 overflows" % bad)
    return dW


def _conv_dims(Xshape, Wshape, stride, pad):
    N, Cc, H, Wd = Xshape
    K, C2, R, S = Wshape
    assert Cc == C2
    P = (H + 2 * pad - R) // stride + 1
    Q = (Wd + 2 * pad - S) // stride + 1
    return N, Cc, H, Wd, K, R, S, P, Q


def conv2d_forward(X, W, stride=1, pad=0):
    X, W = _f32(X), _f32(W)
    N, Cc, H, Wd, K, R, S, P, Q = _conv_dims(X.shape, W.shape, stride, pad)
    Y = np.empty((N, K, P, Q), dtype=np.float64)
    lib().dbp_oracle_conv2d_forward(_p(X), _p(W), *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad)], _p(Y))
    return Y


def conv2d_backward(W, X, *, codes=None, dense=None, step=0.0, stride=1, pad=0,
                    want_dx=True, want_dw=True, threads=None):
    """fp64 (dX [N,C,H,W], dW [K,C,R,S], macs); q has the layer output's shape [N,K,P,Q]."""
    W, X = _f32(W), _f32(X)
    N, Cc, H, Wd, K, R, S, P, Q = _conv_dims(X.shape, W.shape, stride, pad)
    k, d, s = _q_args(codes, dense, step)
    assert (k if k is not None else d).shape == (N, K, P, Q)
    dX = np.empty(X.shape, dtype=np.float64) if want_dx else None
    dW = np.empty(W.shape, dtype=np.float64) if want_dw else None
    macs = C.c_uint64(0)
    lib().dbp_oracle_conv2d_backward(_p(k), _p(d), s, _p(W), _p(X),
                                     *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad)],
                                     _p(dX), _p(dW), C.c_int(threads or max_threads()), C.byref(macs))
    return dX, dW, macs.value


def conv2d_forward_grouped(X, W, groups, stride=1, pad=0):
    """fp64 Y [N,K,P,Q] of a grouped cross-correlation; X [N,C,H,Wd], W [K,C/groups,R,S]."""
    X, W = _f32(X), _f32(W)
    N, Cc, H, Wd = X.shape
    K, Cg, R, S = W.shape
    assert Cc == Cg * groups and K % groups == 0
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    Y = np.empty((N, K, P, Q), dtype=np.float64)
    lib().dbp_oracle_conv2d_forward_grouped(_p(X), _p(W), *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad, groups)], _p(Y))
    return Y


def conv2d_backward_grouped(W, X, groups, *, codes=None, dense=None, step=0.0, stride=1, pad=0, want_dx=True, want_dw=True,
                            threads=None):
    """fp64 (dX [N,C,H,Wd], dW [K,C/groups,R,S]) of the grouped convolution's Eqs. (qda), (qdw)."""
    X, W = _f32(X), _f32(W)
    N, Cc, H, Wd = X.shape
    K, Cg, R, S = W.shape
    assert Cc == Cg * groups and K % groups == 0
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    k, d, s = _q_args(codes, dense, step)
    assert (k if k is not None else d).shape == (N, K, P, Q)
    dX = np.empty(X.shape, dtype=np.float64) if want_dx else None
    dW = np.empty(W.shape, dtype=np.float64) if want_dw else None
    lib().dbp_oracle_conv2d_backward_grouped(_p(k), _p(d), s, _p(W), _p(X),
                                             *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad, groups)],
                                             _p(dX), _p(dW), C.c_int(threads or max_threads()))
    return dX, dW


def conv2d_dw_i8(codes, X8, R, S, stride=1, pad=0, threads=None):
    k, x = _i8(codes), _i8(X8)
    N, Cc, H, Wd = x.shape
    K = k.shape[1]
    dW = np.empty((K, Cc, R, S), dtype=np.int32)
    bad = lib().dbp_oracle_conv2d_dw_i8(_p(k), _p(x), *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad)],
                                        _p(dW), C.c_int(threads or max_threads()))
    if bad:
        raise OverflowError("%d int32 overflows" % bad)
    return dW


def _idx(idx):
    return np.ascontiguousarray(idx, dtype=np.int64).ravel()


def linear_dx_at(W, idx, *, B, codes=None, dense=None, step=0.0):
    W = _f32(W)
    out, in_ = W.shape
    k, d, s = _q_args(codes, dense, step)
    idx = _idx(idx)
    val = np.empty(idx.size, dtype=np.float64)
    lib().dbp_oracle_linear_dx_at(_p(k), _p(d), s, _p(W), C.c_int64(B), C.c_int64(in_), C.c_int64(out),
                                  _p(idx), C.c_int64(idx.size), _p(val))
    return val


def linear_dw_at(X, idx, *, out, codes=None, dense=None, step=0.0):
    """X float32 [B,in] or int8 (integer mode: returns exact sums as fp64)."""
    X = np.ascontiguousarray(X)
    x8 = X if X.dtype == np.int8 else None
    xf = None if x8 is not None else _f32(X)
    B, in_ = X.shape
    k, d, s = _q_args(codes, dense, step)
    idx = _idx(idx)
    val = np.empty(idx.size, dtype=np.float64)
    lib().dbp_oracle_linear_dw_at(_p(k), _p(d), s, _p(xf), _p(x8), C.c_int64(B), C.c_int64(in_), C.c_int64(out),
                                  _p(idx), C.c_int64(idx.size), _p(val))
    return val


def conv2d_dx_at(W, Xshape, idx, *, codes=None, dense=None, step=0.0, stride=1, pad=0):
    W = _f32(W)
    N, Cc, H, Wd, K, R, S, P, Q = _conv_dims(Xshape, W.shape, stride, pad)
    k, d, s = _q_args(codes, dense, step)
    idx = _idx(idx)
    val = np.empty(idx.size, dtype=np.float64)
    lib().dbp_oracle_conv2d_dx_at(_p(k), _p(d), s, _p(W), *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad)],
                                  _p(idx), C.c_int64(idx.size), _p(val))
    return val


def conv2d_dw_at(X, Wshape, idx, *, codes=None, dense=None, step=0.0, stride=1, pad=0):
    X = np.ascontiguousarray(X)
    x8 = X if X.dtype == np.int8 else None
    xf = None if x8 is not None else _f32(X)
    N, Cc, H, Wd, K, R, S, P, Q = _conv_dims(X.shape, Wshape, stride, pad)
    k, d, s = _q_args(codes, dense, step)
    idx = _idx(idx)
    val = np.empty(idx.size, dtype=np.float64)
    lib().dbp_oracle_conv2d_dw_at(_p(k), _p(d), s, _p(xf), _p(x8),
                                  *[C.c_int64(v) for v in (N, Cc, H, Wd, K, R, S, stride, pad)],
                                  _p(idx), C.c_int64(idx.size), _p(val))
    return val


# ---- full 8-bit backward (Sec. "Quantizing forward pass") ---------------------------------------
def quantize_int8(x):
    """Symmetric per-tensor int8 quantiser (dbp_oracle_quantize_int8): returns (q int8, scale float32, inv float32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.int8)
    scale, inv = C.c_float(0.0), C.c_float(0.0)
    lib().dbp_oracle_quantize_int8(_p(x), C.c_int64(x.size), _p(q), C.byref(scale), C.byref(inv))
    return q, np.float32(scale.value), np.float32(inv.value)


def _as_int32(v, what):
    r = np.rint(v)
    if not np.array_equal(r, v):
        raise ArithmeticError("%s: the fp64 sum of integer products is not an integer" % what)
    if r.size and (r.max() > 2**31 - 1 or r.min() < -2**31):
        raise OverflowError("%s leaves int32" % what)
    return r.astype(np.int32)


def linear_backward_q8(codes, W8, X8, threads=None):
    """Exact (dX32 [B,in], dW32 [out,in]) = (codes . W8, codes^T . X8).  Every term of Eqs. (qda)/(qdw) is an
    integer here, so the fp64 sums of linear_backward (step 1) are exact as long as they stay below 2^53."""
    dX, dW, _ = linear_backward(np.asarray(W8, np.float32), np.asarray(X8, np.float32), codes=codes, step=1.0,
                                threads=threads)
    return _as_int32(dX, "dX32"), _as_int32(dW, "dW32")


def conv2d_backward_q8(codes, W8, X8, stride=1, pad=0, threads=None):
    """Exact int32 (dX32, dW32) of the convolution's adjoints with int8 weights and activations."""
    dX, dW, _ = conv2d_backward(np.asarray(W8, np.float32), np.asarray(X8, np.float32), codes=codes, step=1.0,
                                stride=stride, pad=pad, threads=threads)
    return _as_int32(dX, "dX32"), _as_int32(dW, "dW32")
