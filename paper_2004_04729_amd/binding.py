"""Thin ctypes binding of include/dbp.h: same names, argument marshalling only.

Tensor arguments are anything with ``data_ptr()`` (torch tensors on the GPU) or plain integer
device addresses; torch is used by callers for device memory and streams, never for compute.
The raw C entry points are reachable through :func:`lib` for tests of the error paths.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdbp_hip.so")

F32, I8 = 0, 1
PATH_AUTO, PATH_MFMA, PATH_GATHER = 0, 1, 2
PATH_TWO_PLANES = 0x100      # a flag, OR-ed onto a path: two bf16 planes of the fp32 operand instead of three


class DbpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("dbp status %d: %s" % (code, msg))
        self.code = code


class _Layout(C.Structure):
    _fields_ = [("tiles_per_row", C.c_int64), ("n_tiles", C.c_int64), ("bitmap_offset", C.c_size_t),
                ("tile_nnz_offset", C.c_size_t), ("entries_offset", C.c_size_t), ("scratch_offset", C.c_size_t),
                ("total_bytes", C.c_size_t)]


@dataclass
class Stats:
    nnz: int
    n_saturated: int
    n_nonfinite: int
    max_abs_code: int

    @staticmethod
    def from_tensor(t) -> "Stats":
        """Decode a 32-byte device buffer (any tensor of that size) written by the NSD pass."""
        import struct
        raw = bytes(t.detach().cpu().contiguous().view(-1).view(dtype=__import__("torch").uint8).tolist())
        nnz, sat, nf, mx, _ = struct.unpack("<QQQii", raw[:32])
        return Stats(nnz, sat, nf, mx)


class _Extras(C.Structure):
    _fields_ = [("act", C.c_void_p), ("step_dev", C.c_void_p), ("bias_sums", C.c_void_p), ("bias_grad", C.c_void_p),
                ("bias_mode", C.c_int32), ("bias_len", C.c_int64)]


BIAS_PER_COLUMN, BIAS_PER_ROW_GROUP = 0, 1

_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded C library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("HIP library %s is missing: run `python -c 'import __graft_entry__ as g; g.build()'`"
                              % _LIB_PATH)
        L = C.CDLL(_LIB_PATH)
        vp, i64, u64, f32, sz, ci = C.c_void_p, C.c_int64, C.c_uint64, C.c_float, C.c_size_t, C.c_int
        L.dbp_abi_version.restype = C.c_uint32
        L.dbp_status_string.restype = C.c_char_p
        L.dbp_status_string.argtypes = [ci]
        L.dbp_format_layout_of.argtypes = [i64, i64, C.POINTER(_Layout)]
        L.dbp_linear_workspace_bytes.restype = sz
        L.dbp_linear_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.dbp_conv2d_workspace_bytes.restype = sz
        L.dbp_conv2d_workspace_bytes.argtypes = [i64] * 9 + [ci]
        L.nsd_quantize.argtypes = [vp, i64, i64, f32, u64, u64, vp, vp, sz, vp, vp]
        L.nsd_quantize_static.argtypes = [vp, i64, i64, f32, u64, u64, vp, vp, vp]
        L.dbp_topk_workspace_bytes.restype = sz
        L.dbp_topk_workspace_bytes.argtypes = [i64, i64]
        L.topk_quantize.argtypes = [vp, i64, i64, i64, i64, f32, vp, vp, sz, vp, sz, vp, vp]
        L.topk_quantize.restype = ci
        L.dithered_linear_backward.argtypes = [vp, vp, vp, ci, i64, i64, i64, f32, u64, u64, vp, vp, vp, vp, sz, vp, ci, vp]
        L.dithered_conv2d_backward.argtypes = [vp, vp, vp, ci] + [i64] * 9 + [f32, u64, u64, vp, vp, vp, vp, sz, vp, ci, vp]
        L.dbp_conv2d_grouped_workspace_bytes.restype = sz
        L.dbp_conv2d_grouped_workspace_bytes.argtypes = [i64] * 10 + [ci]
        L.dithered_conv2d_backward_grouped.argtypes = [vp, vp, vp, ci] + [i64] * 10 + [f32, u64, u64, vp, vp, vp, vp, sz, vp, ci, vp]
        L.dithered_conv2d_backward_grouped.restype = ci
        L.dbp_conv2d_products_grouped.argtypes = [vp, vp, f32, vp, vp, ci] + [i64] * 10 + [vp, vp, vp, sz, ci, vp]
        L.dbp_conv2d_products_grouped.restype = ci
        L.dense_linear_backward.argtypes = [vp, vp, vp, ci, i64, i64, i64, vp, vp, vp, sz, vp]
        L.dense_conv2d_backward.argtypes = [vp, vp, vp, ci] + [i64] * 9 + [vp, vp, vp, sz, vp]
        L.dbp_linear_products.argtypes = [vp, vp, f32, vp, vp, ci, i64, i64, i64, vp, vp, vp, sz, ci, vp]
        L.dbp_conv2d_products.argtypes = [vp, vp, f32, vp, vp, ci] + [i64] * 9 + [vp, vp, vp, sz, ci, vp]
        L.dbp_step_size_workspace_bytes.restype = sz
        L.dbp_step_size_workspace_bytes.argtypes = [i64]
        L.dbp_step_size.argtypes = [vp, vp, i64, f32, vp, vp, sz, vp]
        L.nsd_quantize_ex.argtypes = [vp, i64, i64, f32, u64, u64, vp, vp, sz, vp, C.POINTER(_Extras), vp]
        L.dbp_linear_layer_workspace_bytes.restype = sz
        L.dbp_linear_layer_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.dbp_conv2d_layer_workspace_bytes.restype = sz
        L.dbp_conv2d_layer_workspace_bytes.argtypes = [i64] * 9 + [ci]
        L.dithered_linear_layer_backward.argtypes = [vp, vp, vp, vp, ci, i64, i64, i64, f32, u64, u64, vp, vp, vp, vp, vp,
                                                     vp, sz, vp, ci, vp]
        L.dithered_conv2d_layer_backward.argtypes = [vp, vp, vp, vp, ci] + [i64] * 9 + [f32, u64, u64, vp, vp, vp, vp, vp,
                                                                                        vp, sz, vp, ci, vp]
        L.dbp_quantize_int8_workspace_bytes.restype = sz
        L.dbp_quantize_int8_workspace_bytes.argtypes = [i64]
        L.dbp_quantize_int8.argtypes = [vp, i64, vp, vp, vp, sz, vp]
        L.dithered_linear_backward_q8.argtypes = [vp, vp, vp, i64, i64, i64, f32, u64, u64, vp, vp, vp, vp, sz, vp, vp]
        L.dithered_conv2d_backward_q8.argtypes = [vp, vp, vp] + [i64] * 9 + [f32, u64, u64, vp, vp, vp, vp, sz, vp, vp]
        for name in ("dbp_step_size", "nsd_quantize_ex", "dithered_linear_layer_backward", "dithered_conv2d_layer_backward",
                     "dbp_quantize_int8", "dithered_linear_backward_q8", "dithered_conv2d_backward_q8"):
            getattr(L, name).restype = ci
        for name in ("dbp_format_layout_of", "nsd_quantize", "dithered_linear_backward", "dithered_conv2d_backward",
                     "dense_linear_backward", "dense_conv2d_backward", "dbp_linear_products", "dbp_conv2d_products"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _check(code: int):
    if code != 0:
        raise DbpError(code, lib().dbp_status_string(code).decode())


def abi_version() -> int:
    return int(lib().dbp_abi_version())


def status_string(code: int) -> str:
    return lib().dbp_status_string(code).decode()


def format_layout(rows: int, cols: int) -> dict:
    L = _Layout()
    _check(lib().dbp_format_layout_of(rows, cols, C.byref(L)))
    return {f: getattr(L, f) for f, _ in _Layout._fields_}


def linear_workspace_bytes(B: int, in_: int, out: int, x_dtype: int = F32) -> int:
    return int(lib().dbp_linear_workspace_bytes(B, in_, out, x_dtype))


def conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, stride=1, pad=0, x_dtype: int = F32) -> int:
    return int(lib().dbp_conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, stride, pad, x_dtype))


def nsd_quantize(delta, rows, cols, step, seed, idx_base, codes, fmt=None, stats=None, stream=0):
    _check(lib().nsd_quantize(_ptr(delta), rows, cols, step, seed, idx_base, _ptr(codes), _ptr(fmt), _nbytes(fmt),
                              _ptr(stats), stream))


def nsd_quantize_static(delta, rows, cols, step, seed, idx_base, codes, stats, stream=0):
    _check(lib().nsd_quantize_static(_ptr(delta), rows, cols, step, seed, idx_base, _ptr(codes), _ptr(stats), stream))


def topk_workspace_bytes(rows: int, vec_rows: int = 1) -> int:
    return int(lib().dbp_topk_workspace_bytes(rows, vec_rows))


def topk_quantize(delta, rows, cols, vec_rows, k, step, codes, workspace, fmt=None, stats=None, stream=0):
    _check(lib().topk_quantize(_ptr(delta), rows, cols, vec_rows, k, step, _ptr(codes), _ptr(fmt), _nbytes(fmt),
                               _ptr(workspace), _nbytes(workspace), _ptr(stats), stream))


def dithered_linear_backward(delta, W, X, x_dtype, B, in_, out, step, seed, idx_base, codes, dX, dW, workspace,
                             stats=None, path=PATH_AUTO, stream=0):
    _check(lib().dithered_linear_backward(_ptr(delta), _ptr(W), _ptr(X), x_dtype, B, in_, out, step, seed, idx_base,
                                          _ptr(codes), _ptr(dX), _ptr(dW), _ptr(workspace), _nbytes(workspace),
                                          _ptr(stats), path, stream))


def dithered_conv2d_backward(delta, W, X, x_dtype, N, Cc, H, Wd, K, R, S, stride, pad, step, seed, idx_base,
                             codes, dX, dW, workspace, stats=None, path=PATH_AUTO, stream=0):
    _check(lib().dithered_conv2d_backward(_ptr(delta), _ptr(W), _ptr(X), x_dtype, N, Cc, H, Wd, K, R, S, stride, pad,
                                          step, seed, idx_base, _ptr(codes), _ptr(dX), _ptr(dW), _ptr(workspace),
                                          _nbytes(workspace), _ptr(stats), path, stream))


def conv2d_grouped_workspace_bytes(N, Cc, H, Wd, K, R, S, stride, pad, groups, x_dtype: int = F32) -> int:
    return int(lib().dbp_conv2d_grouped_workspace_bytes(N, Cc, H, Wd, K, R, S, stride, pad, groups, x_dtype))


def dithered_conv2d_backward_grouped(delta, W, X, x_dtype, N, Cc, H, Wd, K, R, S, stride, pad, groups, step, seed, idx_base,
                                     codes, dX, dW, workspace, stats=None, path=PATH_AUTO, stream=0):
    _check(lib().dithered_conv2d_backward_grouped(_ptr(delta), _ptr(W), _ptr(X), x_dtype, N, Cc, H, Wd, K, R, S, stride, pad,
                                                  groups, step, seed, idx_base, _ptr(codes), _ptr(dX), _ptr(dW),
                                                  _ptr(workspace), _nbytes(workspace), _ptr(stats), path, stream))


def conv2d_products_grouped(codes, fmt, step, W, X, x_dtype, N, Cc, H, Wd, K, R, S, stride, pad, groups, dX, dW, workspace,
                            path=PATH_AUTO, stream=0):
    _check(lib().dbp_conv2d_products_grouped(_ptr(codes), _ptr(fmt), step, _ptr(W), _ptr(X), x_dtype, N, Cc, H, Wd, K, R, S,
                                             stride, pad, groups, _ptr(dX), _ptr(dW), _ptr(workspace), _nbytes(workspace),
                                             path, stream))


def dense_linear_backward(delta, W, X, x_dtype, B, in_, out, dX, dW, workspace, stream=0):
    _check(lib().dense_linear_backward(_ptr(delta), _ptr(W), _ptr(X), x_dtype, B, in_, out, _ptr(dX), _ptr(dW),
                                       _ptr(workspace), _nbytes(workspace), stream))


def dense_conv2d_backward(delta, W, X, x_dtype, N, Cc, H, Wd, K, R, S, stride, pad, dX, dW, workspace, stream=0):
    _check(lib().dense_conv2d_backward(_ptr(delta), _ptr(W), _ptr(X), x_dtype, N, Cc, H, Wd, K, R, S, stride, pad,
                                       _ptr(dX), _ptr(dW), _ptr(workspace), _nbytes(workspace), stream))


def linear_products(codes, fmt, step, W, X, x_dtype, B, in_, out, dX, dW, workspace, path=PATH_AUTO, stream=0):
    _check(lib().dbp_linear_products(_ptr(codes), _ptr(fmt), step, _ptr(W), _ptr(X), x_dtype, B, in_, out,
                                     _ptr(dX), _ptr(dW), _ptr(workspace), _nbytes(workspace), path, stream))


def conv2d_products(codes, fmt, step, W, X, x_dtype, N, Cc, H, Wd, K, R, S, stride, pad, dX, dW, workspace,
                    path=PATH_AUTO, stream=0):
    _check(lib().dbp_conv2d_products(_ptr(codes), _ptr(fmt), step, _ptr(W), _ptr(X), x_dtype, N, Cc, H, Wd, K, R, S,
                                     stride, pad, _ptr(dX), _ptr(dW), _ptr(workspace), _nbytes(workspace), path, stream))


def step_size_workspace_bytes(n: int) -> int:
    return int(lib().dbp_step_size_workspace_bytes(n))


def step_size(delta, act, n, s, step_out, workspace, stream=0):
    """The step-size computation of Algorithm 1 on the device: step_out[0:2] = {s*std(delta_z), its reciprocal}."""
    _check(lib().dbp_step_size(_ptr(delta), _ptr(act), n, s, _ptr(step_out), _ptr(workspace), _nbytes(workspace), stream))


def nsd_quantize_ex(delta, rows, cols, step, seed, idx_base, codes, fmt=None, stats=None, act=None, step_dev=None,
                    bias_sums=None, bias_grad=None, bias_mode=BIAS_PER_COLUMN, bias_len=0, stream=0):
    ex = _Extras(_ptr(act), _ptr(step_dev), _ptr(bias_sums), _ptr(bias_grad), bias_mode, bias_len)
    _check(lib().nsd_quantize_ex(_ptr(delta), rows, cols, step, seed, idx_base, _ptr(codes), _ptr(fmt), _nbytes(fmt),
                                 _ptr(stats), C.byref(ex), stream))


def linear_layer_workspace_bytes(B: int, in_: int, out: int, x_dtype: int = F32) -> int:
    return int(lib().dbp_linear_layer_workspace_bytes(B, in_, out, x_dtype))


def conv2d_layer_workspace_bytes(N, Cc, H, Wd, K, R, S, stride=1, pad=0, x_dtype: int = F32) -> int:
    return int(lib().dbp_conv2d_layer_workspace_bytes(N, Cc, H, Wd, K, R, S, stride, pad, x_dtype))


def dithered_linear_layer_backward(delta_a, act, W, X, x_dtype, B, in_, out, s, seed, idx_base, codes, dX, dW, db, step_out,
                                   workspace, stats=None, path=PATH_AUTO, stream=0):
    _check(lib().dithered_linear_layer_backward(_ptr(delta_a), _ptr(act), _ptr(W), _ptr(X), x_dtype, B, in_, out, s, seed,
                                                idx_base, _ptr(codes), _ptr(dX), _ptr(dW), _ptr(db), _ptr(step_out),
                                                _ptr(workspace), _nbytes(workspace), _ptr(stats), path, stream))


def dithered_conv2d_layer_backward(delta_a, act, W, X, x_dtype, N, Cc, H, Wd, K, R, S, stride, pad, s, seed, idx_base, codes,
                                   dX, dW, db, step_out, workspace, stats=None, path=PATH_AUTO, stream=0):
    _check(lib().dithered_conv2d_layer_backward(_ptr(delta_a), _ptr(act), _ptr(W), _ptr(X), x_dtype, N, Cc, H, Wd, K, R, S,
                                                stride, pad, s, seed, idx_base, _ptr(codes), _ptr(dX), _ptr(dW), _ptr(db),
                                                _ptr(step_out), _ptr(workspace), _nbytes(workspace), _ptr(stats), path,
                                                stream))


def quantize_int8_workspace_bytes(n):
    return int(lib().dbp_quantize_int8_workspace_bytes(n))


def quantize_int8(x, n, q, scale_out, workspace, stream=0):
    """The forward pass's symmetric int8 quantiser: q[0:n], scale_out[0:2] = {scale, 1/scale}."""
    _check(lib().dbp_quantize_int8(_ptr(x), n, _ptr(q), _ptr(scale_out), _ptr(workspace), _nbytes(workspace), stream))


def dithered_linear_backward_q8(delta, W8, X8, B, in_, out, step, seed, idx_base, codes, dX32, dW32, workspace,
                                stats=None, stream=0):
    _check(lib().dithered_linear_backward_q8(_ptr(delta), _ptr(W8), _ptr(X8), B, in_, out, step, seed, idx_base,
                                             _ptr(codes), _ptr(dX32), _ptr(dW32), _ptr(workspace), _nbytes(workspace),
                                             _ptr(stats), stream))


def dithered_conv2d_backward_q8(delta, W8, X8, N, Cc, H, Wd, K, R, S, stride, pad, step, seed, idx_base, codes, dX32,
                                dW32, workspace, stats=None, stream=0):
    _check(lib().dithered_conv2d_backward_q8(_ptr(delta), _ptr(W8), _ptr(X8), N, Cc, H, Wd, K, R, S, stride, pad, step,
                                             seed, idx_base, _ptr(codes), _ptr(dX32), _ptr(dW32), _ptr(workspace),
                                             _nbytes(workspace), _ptr(stats), stream))
