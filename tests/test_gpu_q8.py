"""GPU parity of the full 8-bit backward: the int8 quantiser of the forward pass and the two products on int8
matrix cores.  Everything here is integer (or a single fp32 operation per element): the bar is bit-exact."""
import numpy as np
import pytest
import torch

import paper_2004_04729_amd as dbp
import workloads
from oracle import oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _quantize_gpu(x):
    n = x.size
    q = torch.full((n,), 77, dtype=torch.int8, device=DEV)
    sc = torch.full((2,), -1.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(dbp.quantize_int8_workspace_bytes(n), dtype=torch.uint8, device=DEV)
    dbp.quantize_int8(_dev(x.reshape(-1)), n, q, sc, ws, _stream())
    torch.cuda.synchronize()
    return q.cpu().numpy().reshape(x.shape), sc.cpu().numpy()


@pytest.mark.parametrize("n,seed", [(1, 0), (7, 1), (4096, 2), (100003, 3), (3 * 1024 * 1024 + 5, 4)])
def test_quantiser_is_bit_exact(n, seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal(n) * np.exp(2 * rng.standard_normal(n))).astype(np.float32)
    q, sc = _quantize_gpu(x)
    q_ref, scale, inv = O.quantize_int8(x)
    assert sc[0] == scale and sc[1] == inv
    assert np.array_equal(q, q_ref)


def test_quantiser_special_values_and_ties():
    x = np.array([np.nan, np.inf, -np.inf, 2.0, -4.0, 1e-30, 0.0, -0.0, 1e-45], dtype=np.float32)
    q, sc = _quantize_gpu(x)
    q_ref, scale, inv = O.quantize_int8(x)
    assert sc[0] == scale and sc[1] == inv and np.array_equal(q, q_ref)
    x = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5], dtype=np.float32)
    q, sc = _quantize_gpu(x)
    assert list(q) == [127, 0, 2, 2, 0, -2, -2, 126] and sc[0] == 1.0 and sc[1] == 1.0
    q, sc = _quantize_gpu(np.zeros(100, dtype=np.float32))
    assert not q.any() and sc[0] == 0.0 and sc[1] == 0.0
    q, sc = _quantize_gpu(np.array([np.nan, np.inf], dtype=np.float32))
    assert list(q) == [0, 127] and sc[0] == 0.0


def _fc(B, in_, out, seed, c=2.0, want_dx=True, want_dw=True):
    rng = np.random.default_rng(seed)
    delta = rng.laplace(size=(B, out)).astype(np.float32) * np.float32(1e-3)
    step = float(np.float32(c * delta.std())) if delta.size > 1 else 1e-3
    W8 = rng.integers(-127, 128, size=(out, in_)).astype(np.int8)
    X8 = np.maximum(rng.integers(-127, 128, size=(B, in_)), 0).astype(np.int8)
    codes = torch.empty((B, out), dtype=torch.int8, device=DEV)
    dX = torch.full((B, in_), 12345, dtype=torch.int32, device=DEV) if want_dx else None
    dW = torch.full((out, in_), 12345, dtype=torch.int32, device=DEV) if want_dw else None
    ws = torch.empty(dbp.linear_workspace_bytes(B, in_, out), dtype=torch.uint8, device=DEV)
    st = torch.zeros(32, dtype=torch.uint8, device=DEV)
    dbp.dithered_linear_backward_q8(_dev(delta), _dev(W8), _dev(X8), B, in_, out, step, seed, 0, codes, dX, dW, ws, st,
                                    _stream())
    torch.cuda.synchronize()
    k_ref, st_ref = O.nsd(delta, step, seed)
    assert np.array_equal(codes.cpu().numpy(), k_ref.reshape(B, out))
    assert dbp.Stats.from_tensor(st).nnz == st_ref.nnz
    dX_ref, dW_ref = O.linear_backward_q8(k_ref.reshape(B, out), W8, X8)
    if want_dx:
        assert np.array_equal(dX.cpu().numpy(), dX_ref)
    if want_dw:
        assert np.array_equal(dW.cpu().numpy(), dW_ref)


@pytest.mark.parametrize("B,in_,out", [(1, 1, 1), (37, 100, 52), (64, 784, 512), (256, 1000, 300), (300, 260, 1030)])
def test_fc_q8_is_bit_exact(B, in_, out):
    _fc(B, in_, out, seed=B + out)


# shapes the role-specialised int8 kernel takes (batch and out above 128, in a multiple of 8), through its edges:
# ragged tiles, reductions that end inside a window of 64, a batch that is not a multiple of 4
@pytest.mark.parametrize("B,in_,out", [(258, 264, 200), (130, 4104, 140), (1000, 136, 260), (512, 512, 392),
                                       (256, 1024, 4096), (256, 4096, 1000),
                                       (256, 4096, 4096)])     # the two products on two groups of workgroups
def test_fc_q8_large_layer_kernel(B, in_, out):
    _fc(B, in_, out, seed=B + in_ + out, c=8.0)
    _fc(B, in_, out, seed=B + in_ + out, c=8.0, want_dw=False)
    _fc(B, in_, out, seed=B + in_ + out, c=8.0, want_dx=False)


def test_fc_q8_single_products_and_dense_codes():
    _fc(70, 130, 90, seed=3, want_dw=False)
    _fc(70, 130, 90, seed=3, want_dx=False)
    _fc(40, 64, 2000, seed=5, c=0.02)                    # nearly every code nonzero, many saturated


CONV_CASES = [  # N, C, H, Wd, K, R, S, pad (, stride)
    (2, 8, 15, 14, 12, 3, 3, 1, 2),
    (2, 16, 14, 14, 24, 1, 1, 0, 2),
    (3, 40, 28, 28, 72, 3, 3, 1, 2),    # strided dX as four stride-1 classes in one launch (P*Q a multiple of 4)
    (2, 16, 16, 16, 24, 1, 1, 0, 2),    # 1x1 / 2: three classes without taps (cleared), one with the single tap
    (2, 8, 15, 17, 8, 3, 3, 1, 2),      # odd image sizes: the classes have different extents
    (2, 6, 11, 13, 9, 3, 3, 0, 3),      # stride 3: nine classes of one tap each
    (16, 64, 28, 28, 128, 3, 3, 1, 2),  # large enough that dW runs as column matrix x int8 fully connected kernel
    (32, 128, 14, 14, 256, 1, 1, 0),    # 1x1, more than 128 output channels: dW by the int8 fully connected kernel on the NCHW tensors
    (4, 36, 14, 14, 130, 1, 1, 0),      # the same with partial tiles
    (1, 1, 1, 1, 1, 1, 1, 0),
    (2, 5, 9, 7, 6, 3, 3, 1),
    (3, 16, 14, 14, 24, 3, 3, 1),
    (2, 33, 14, 14, 20, 1, 1, 0),
    (2, 3, 11, 8, 4, 5, 3, 2),
    (1, 130, 6, 6, 260, 3, 3, 1),
    (2, 64, 30, 30, 40, 3, 3, 1),
]


def _conv_inputs(N, C, H, Wd, K, R, S, pad, seed, c=2.0, stride=1):
    rng = np.random.default_rng(seed)
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    delta = rng.laplace(size=(N, K, P, Q)).astype(np.float32) * np.float32(1e-3)
    step = float(np.float32(c * delta.std())) if delta.size > 1 else 1e-3
    W8 = rng.integers(-127, 128, size=(K, C, R, S)).astype(np.int8)
    X8 = np.maximum(rng.integers(-127, 128, size=(N, C, H, Wd)), 0).astype(np.int8)
    return delta, step, W8, X8, P, Q


def _conv_gpu(delta, step, W8, X8, pad, seed, stride=1):
    N, C, H, Wd = X8.shape
    K, _, R, S = W8.shape
    codes = torch.empty(delta.shape, dtype=torch.int8, device=DEV)
    dX = torch.full(X8.shape, 12345, dtype=torch.int32, device=DEV)
    dW = torch.full(W8.shape, 12345, dtype=torch.int32, device=DEV)
    ws = torch.empty(dbp.conv2d_workspace_bytes(N, C, H, Wd, K, R, S, stride, pad, dbp.I8), dtype=torch.uint8, device=DEV)
    dbp.dithered_conv2d_backward_q8(_dev(delta), _dev(W8), _dev(X8), N, C, H, Wd, K, R, S, stride, pad, step, seed, 0, codes,
                                    dX, dW, ws, None, _stream())
    torch.cuda.synchronize()
    return codes.cpu().numpy(), dX.cpu().numpy(), dW.cpu().numpy()


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_q8_is_bit_exact(case):
    N, C, H, Wd, K, R, S, pad = case[:8]
    stride = case[8] if len(case) > 8 else 1
    delta, step, W8, X8, P, Q = _conv_inputs(*case[:8], seed=N + K, stride=stride)
    codes, dX, dW = _conv_gpu(delta, step, W8, X8, pad, seed=11, stride=stride)
    k_ref, _ = O.nsd(delta, step, 11)
    k_ref = k_ref.reshape(delta.shape)
    assert np.array_equal(codes, k_ref)
    dX_ref, dW_ref = O.conv2d_backward_q8(k_ref, W8, X8, stride=stride, pad=pad)
    assert np.array_equal(dX, dX_ref) and np.array_equal(dW, dW_ref)


def test_conv_q8_config5_full_size_in_full():
    # the 8-bit configuration at its real size: codes and every element of both int32 products
    p = workloads.config5(0.9)
    rng = np.random.default_rng(77)
    W8 = rng.integers(-127, 128, size=p.W.shape).astype(np.int8)
    codes, dX, dW = _conv_gpu(p.delta, p.step, W8, p.X, p.pad, seed=p.seed)
    k_ref, _ = O.nsd(p.delta, p.step, p.seed)
    k_ref = k_ref.reshape(p.delta.shape)
    assert np.array_equal(codes, k_ref)
    dX_ref, dW_ref = O.conv2d_backward_q8(k_ref, W8, p.X, stride=1, pad=p.pad)
    assert np.array_equal(dX, dX_ref) and np.array_equal(dW, dW_ref)
