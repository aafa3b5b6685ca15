"""Pins for the oracle's backward products (CPU only): library routines, brute force in exact
integer arithmetic, algebraic identities and the adjoint property that defines a backward pass."""
import itertools

import numpy as np
import pytest
import torch

from oracle import oracle as O


def _codes(rng, shape, density=0.2, amp=3):
    return (rng.integers(-amp, amp + 1, size=shape) * (rng.random(shape) < density)).astype(np.int8)


# ------------------------------------------------------------------ fully connected
@pytest.mark.parametrize("B,in_,out", [(1, 1, 1), (3, 5, 4), (8, 7, 8), (17, 33, 9)])
def test_fc_brute_force_exact_integers(B, in_, out):
    # Eqs. (qda),(qdw) written out with Python integers: exact, so equality is exact.
    rng = np.random.default_rng(B * 100 + in_)
    k = _codes(rng, (B, out), 0.5)
    W = rng.integers(-9, 10, size=(out, in_)).astype(np.float32)
    X = rng.integers(-9, 10, size=(B, in_)).astype(np.float32)
    step = 0.25
    dX, dW, macs = O.linear_backward(W, X, codes=k, step=step)
    for b, i in itertools.product(range(B), range(in_)):
        assert dX[b, i] == step * sum(int(k[b, o]) * int(W[o, i]) for o in range(out))
    for o, i in itertools.product(range(out), range(in_)):
        assert dW[o, i] == step * sum(int(k[b, o]) * int(X[b, i]) for b in range(B))
    # cost model of Sec. "Computational complexity": p_nz * m*k*n multiply-adds per product
    assert macs == 2 * np.count_nonzero(k) * in_


def test_fc_against_library_matmul_and_special_cases():
    rng = np.random.default_rng(21)
    B, in_, out = 37, 300, 129
    k = _codes(rng, (B, out), 0.15, amp=100)
    W = rng.standard_normal((out, in_)).astype(np.float32)
    X = rng.standard_normal((B, in_)).astype(np.float32)
    step = float(np.float32(3.3e-3))
    dX, dW, _ = O.linear_backward(W, X, codes=k, step=step)
    q = k.astype(np.float64) * step
    np.testing.assert_allclose(dX, q @ W.astype(np.float64), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dW, q.T @ X.astype(np.float64), rtol=1e-12, atol=1e-15)
    # a transposed-operand mistake cannot hide: shapes differ and the values are asymmetric
    assert dX.shape == (B, in_) and dW.shape == (out, in_)
    # identity weights: delta_a = q ; one-hot q picks one row of W / one row of X
    I = np.eye(out, dtype=np.float32)
    dXi, _, _ = O.linear_backward(I, X[:, :out], codes=k, step=step)
    assert np.array_equal(dXi, q)
    one = np.zeros((B, out), dtype=np.int8)
    one[5, 7] = -3
    dX1, dW1, macs = O.linear_backward(W, X, codes=one, step=step)
    assert np.array_equal(dX1[5], -3 * step * W[7].astype(np.float64)) and not dX1[np.arange(B) != 5].any()
    assert np.array_equal(dW1[7], -3 * step * X[5].astype(np.float64)) and not dW1[np.arange(out) != 7].any()
    assert macs == 2 * in_
    # dense (undithered) path, Eqs. (da),(dw)
    d = rng.standard_normal((B, out)).astype(np.float32)
    dXd, dWd, _ = O.linear_backward(W, X, dense=d)
    np.testing.assert_allclose(dXd, d.astype(np.float64) @ W, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dWd, d.astype(np.float64).T @ X, rtol=1e-12, atol=1e-14)


def test_fc_int8_mode_exact_and_overflow_detected():
    rng = np.random.default_rng(22)
    B, in_, out = 50, 40, 30
    k = _codes(rng, (B, out), 0.3, amp=127)
    X8 = rng.integers(-127, 128, size=(B, in_)).astype(np.int8)
    ref = k.astype(np.int64).T @ X8.astype(np.int64)
    assert np.array_equal(O.linear_dw_i8(k, X8), ref.astype(np.int32))
    big_k = np.full((140000, 1), 127, dtype=np.int8)
    big_x = np.full((140000, 1), 127, dtype=np.int8)
    with pytest.raises(OverflowError):
        O.linear_dw_i8(big_k, big_x)


def test_fc_single_output_versions_agree_with_full():
    rng = np.random.default_rng(23)
    B, in_, out = 12, 31, 17
    k = _codes(rng, (B, out), 0.3)
    W = rng.standard_normal((out, in_)).astype(np.float32)
    X = rng.standard_normal((B, in_)).astype(np.float32)
    dX, dW, _ = O.linear_backward(W, X, codes=k, step=0.5)
    ix = rng.integers(0, B * in_, size=64)
    iw = rng.integers(0, out * in_, size=64)
    np.testing.assert_allclose(O.linear_dx_at(W, ix, B=B, codes=k, step=0.5), dX.ravel()[ix], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.linear_dw_at(X, iw, out=out, codes=k, step=0.5), dW.ravel()[iw], rtol=1e-13, atol=1e-15)
    X8 = rng.integers(-127, 128, size=(B, in_)).astype(np.int8)
    assert np.array_equal(O.linear_dw_at(X8, iw, out=out, codes=k), O.linear_dw_i8(k, X8).ravel()[iw].astype(np.float64))


# ------------------------------------------------------------------ convolution
CONV_CASES = [  # N, C, H, Wd, K, R, S, stride, pad
    (2, 3, 6, 7, 4, 3, 3, 1, 1),
    (1, 2, 5, 5, 3, 1, 1, 1, 0),
    (2, 2, 8, 6, 3, 3, 3, 2, 1),
    (1, 3, 7, 7, 2, 5, 3, 1, 2),
    (2, 1, 4, 4, 2, 3, 3, 1, 0),
]


def _conv_inputs(case, seed=0):
    N, C, H, Wd, K, R, S, st, pad = case
    rng = np.random.default_rng(seed + sum(case))
    P, Q = (H + 2 * pad - R) // st + 1, (Wd + 2 * pad - S) // st + 1
    X = rng.standard_normal((N, C, H, Wd)).astype(np.float32)
    W = rng.standard_normal((K, C, R, S)).astype(np.float32)
    k = _codes(rng, (N, K, P, Q), 0.4)
    return X, W, k, st, pad


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_against_library_autograd(case):
    # the library routine: torch's CPU convolution and its autograd, in fp64
    X, W, k, st, pad = _conv_inputs(case)
    step = 0.125
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    Y = torch.nn.functional.conv2d(Xt, Wt, stride=st, padding=pad)
    np.testing.assert_allclose(O.conv2d_forward(X, W, st, pad), Y.detach().numpy(), rtol=1e-12, atol=1e-13)
    Y.backward(torch.tensor(k.astype(np.float64) * step))
    dX, dW, macs = O.conv2d_backward(W, X, codes=k, step=step, stride=st, pad=pad)
    np.testing.assert_allclose(dX, Xt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert macs == 2 * np.count_nonzero(k) * W[0].size


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoint_identity(case):
    # <conv(X,W), Q> = <X, dX(Q,W)> = <W, dW(Q,X)>: what makes dX and dW "the" backward products
    X, W, k, st, pad = _conv_inputs(case, seed=5)
    step = 0.5
    q = k.astype(np.float64) * step
    lhs = float((O.conv2d_forward(X, W, st, pad) * q).sum())
    dX, dW, _ = O.conv2d_backward(W, X, codes=k, step=step, stride=st, pad=pad)
    assert abs(lhs - float((dX * X).sum())) < 1e-9 * max(1.0, abs(lhs))
    assert abs(lhs - float((dW * W).sum())) < 1e-9 * max(1.0, abs(lhs))


def test_conv_1x1_is_a_fully_connected_layer():
    case = (3, 6, 5, 4, 7, 1, 1, 1, 0)
    X, W, k, st, pad = _conv_inputs(case, seed=9)
    N, C, H, Wd, K = case[:5]
    dX, dW, _ = O.conv2d_backward(W, X, codes=k, step=0.25, stride=1, pad=0)
    Xf = X.transpose(0, 2, 3, 1).reshape(-1, C)
    kf = k.transpose(0, 2, 3, 1).reshape(-1, K)
    fX, fW, _ = O.linear_backward(W.reshape(K, C), Xf, codes=kf, step=0.25)
    assert np.array_equal(dX, fX.reshape(N, H, Wd, C).transpose(0, 3, 1, 2))
    np.testing.assert_allclose(dW.reshape(K, C), fW, rtol=1e-13, atol=1e-15)


def test_conv_equals_explicit_im2col_times_fc():
    case = (2, 3, 6, 5, 4, 3, 3, 1, 1)
    X, W, k, st, pad = _conv_inputs(case, seed=13)
    N, C, H, Wd, K, R, S = case[:7]
    P, Q = k.shape[2:]
    Xp = np.pad(X, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    cols = np.empty((N * P * Q, C * R * S), dtype=np.float32)
    for n, p, q in itertools.product(range(N), range(P), range(Q)):
        cols[(n * P + p) * Q + q] = Xp[n, :, p:p + R, q:q + S].ravel()
    kf = k.transpose(0, 2, 3, 1).reshape(-1, K)
    _, fW, _ = O.linear_backward(W.reshape(K, -1), cols, codes=kf, step=0.5, want_dx=False)
    _, dW, _ = O.conv2d_backward(W, X, codes=k, step=0.5, stride=1, pad=pad, want_dx=False)
    np.testing.assert_allclose(dW.reshape(K, -1), fW, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_single_output_versions_and_int8(case):
    X, W, k, st, pad = _conv_inputs(case, seed=17)
    rng = np.random.default_rng(1)
    dX, dW, _ = O.conv2d_backward(W, X, codes=k, step=0.5, stride=st, pad=pad)
    ix = rng.integers(0, X.size, size=80)
    iw = rng.integers(0, W.size, size=80)
    np.testing.assert_allclose(O.conv2d_dx_at(W, X.shape, ix, codes=k, step=0.5, stride=st, pad=pad),
                               dX.ravel()[ix], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.conv2d_dw_at(X, W.shape, iw, codes=k, step=0.5, stride=st, pad=pad),
                               dW.ravel()[iw], rtol=1e-13, atol=1e-15)
    X8 = rng.integers(-127, 128, size=X.shape).astype(np.int8)
    d32 = O.conv2d_dw_i8(k, X8, W.shape[2], W.shape[3], st, pad)
    _, ref, _ = O.conv2d_backward(W, X8.astype(np.float32), codes=k, step=1.0, stride=st, pad=pad, want_dx=False)
    assert np.array_equal(d32.astype(np.float64), ref)          # small integers: fp64 sums are exact
    assert np.array_equal(O.conv2d_dw_at(X8, W.shape, iw, codes=k, stride=st, pad=pad), d32.ravel()[iw].astype(np.float64))


def test_dense_conv_path_against_autograd():
    case = CONV_CASES[0]
    X, W, k, st, pad = _conv_inputs(case, seed=19)
    d = np.random.default_rng(2).standard_normal(k.shape).astype(np.float32)
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.conv2d(Xt, Wt, stride=st, padding=pad).backward(torch.tensor(d, dtype=torch.float64))
    dX, dW, _ = O.conv2d_backward(W, X, dense=d, stride=st, pad=pad)
    np.testing.assert_allclose(dX, Xt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-12, atol=1e-13)
