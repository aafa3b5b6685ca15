"""Pins of the oracle's grouped convolution (the layer type of the CNNs of Sec. "Experiments") against things that are
not the oracle: torch's fp64 grouped convolution and its autograd, the adjoint identities that define Eqs. (qda)/(qdw)
for any linear layer, the reduction to the ungrouped functions, and a hand-computed depthwise case."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle

CASES = [  # N, C, H, Wd, K, R, S, stride, pad, groups
    (2, 4, 7, 6, 6, 3, 3, 1, 1, 2),
    (1, 6, 9, 9, 3, 3, 2, 2, 0, 3),
    (2, 8, 5, 5, 8, 3, 3, 1, 1, 8),          # depthwise
    (1, 4, 8, 7, 8, 5, 5, 3, 2, 4),          # depthwise with a channel multiplier of 2
    (3, 6, 6, 6, 4, 1, 1, 1, 0, 2),
]


def _rand(case, seed=0):
    N, C, H, Wd, K, R, S, st, pad, g = case
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, C, H, Wd)).astype(np.float32)
    W = rng.standard_normal((K, C // g, R, S)).astype(np.float32)
    P, Q = (H + 2 * pad - R) // st + 1, (Wd + 2 * pad - S) // st + 1
    codes = rng.integers(-127, 128, size=(N, K, P, Q)).astype(np.int8)
    codes[rng.random(codes.shape) < 0.6] = 0
    return X, W, codes


@pytest.mark.parametrize("case", CASES)
def test_forward_and_both_gradients_match_torch_fp64(case):
    N, C, H, Wd, K, R, S, st, pad, g = case
    X, W, codes = _rand(case)
    step = 0.37
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    Y = F.conv2d(Xt, Wt, stride=st, padding=pad, groups=g)
    np.testing.assert_allclose(oracle.conv2d_forward_grouped(X, W, g, st, pad), Y.detach().numpy(), rtol=1e-12, atol=1e-12)
    Y.backward(torch.tensor(codes.astype(np.float64) * step))
    dX, dW = oracle.conv2d_backward_grouped(W, X, g, codes=codes, step=step, stride=st, pad=pad)
    np.testing.assert_allclose(dX, Xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identities(case):
    # <q, conv(X', W)> = <dX, X'> for any X', and <q, conv(X, W')> = <dW, W'> for any W': the definition of the two products
    N, C, H, Wd, K, R, S, st, pad, g = case
    X, W, codes = _rand(case, 1)
    dense = (codes.astype(np.float32) * np.float32(0.5))
    dX, dW = oracle.conv2d_backward_grouped(W, X, g, dense=dense, stride=st, pad=pad)
    rng = np.random.default_rng(2)
    X2 = rng.standard_normal(X.shape).astype(np.float32)
    W2 = rng.standard_normal(W.shape).astype(np.float32)
    lhs_x = float((dense.astype(np.float64) * oracle.conv2d_forward_grouped(X2, W, g, st, pad)).sum())
    lhs_w = float((dense.astype(np.float64) * oracle.conv2d_forward_grouped(X, W2, g, st, pad)).sum())
    assert abs(lhs_x - float((dX * X2).sum())) <= 1e-9 * (np.abs(dX) * np.abs(X2)).sum()
    assert abs(lhs_w - float((dW * W2).sum())) <= 1e-9 * (np.abs(dW) * np.abs(W2)).sum()


def test_one_group_is_the_plain_convolution():
    case = (2, 5, 7, 8, 4, 3, 3, 2, 1, 1)
    X, W, codes = _rand(case, 3)
    dX, dW = oracle.conv2d_backward_grouped(W, X, 1, codes=codes, step=0.25, stride=2, pad=1)
    dX1, dW1, _ = oracle.conv2d_backward(W, X, codes=codes, step=0.25, stride=2, pad=1)
    np.testing.assert_array_equal(dX, dX1)
    np.testing.assert_array_equal(dW, dW1)
    np.testing.assert_array_equal(oracle.conv2d_forward_grouped(X, W, 1, 2, 1), oracle.conv2d_forward(X, W, 2, 1))


def test_groups_are_independent_convolutions_on_channel_blocks():
    case = (2, 6, 6, 5, 9, 3, 3, 1, 1, 3)
    X, W, codes = _rand(case, 4)
    dX, dW = oracle.conv2d_backward_grouped(W, X, 3, codes=codes, step=0.5, stride=1, pad=1)
    for j in range(3):
        dXj, dWj, _ = oracle.conv2d_backward(W[3 * j:3 * j + 3], np.ascontiguousarray(X[:, 2 * j:2 * j + 2]),
                                             codes=np.ascontiguousarray(codes[:, 3 * j:3 * j + 3]), step=0.5, stride=1, pad=1)
        np.testing.assert_array_equal(dX[:, 2 * j:2 * j + 2], dXj)
        np.testing.assert_array_equal(dW[3 * j:3 * j + 3], dWj)


def test_hand_computed_depthwise_1x1():
    # groups = C = K, 1x1 kernel: dX[n,c] = step*code[n,c]*w[c] pointwise, dW[c] = step * sum code[n,c]*X[n,c]
    X = np.arange(2 * 3 * 2 * 2, dtype=np.float32).reshape(2, 3, 2, 2)
    W = np.array([2.0, -1.0, 0.5], dtype=np.float32).reshape(3, 1, 1, 1)
    codes = (np.arange(24).reshape(2, 3, 2, 2) % 5 - 2).astype(np.int8)
    dX, dW = oracle.conv2d_backward_grouped(W, X, 3, codes=codes, step=0.5)
    np.testing.assert_array_equal(dX, 0.5 * codes * W.reshape(1, 3, 1, 1).astype(np.float64))
    np.testing.assert_array_equal(dW.ravel(), 0.5 * (codes.astype(np.float64) * X).sum(axis=(0, 2, 3)))
