"""Pins for the oracle of the full 8-bit backward (CPU only): the forward pass's int8 quantiser against
hand-computed values and its defining properties, the integer products against numpy's integer matmul
and against sums written out with Python integers."""
import itertools

import numpy as np
import pytest

from oracle import oracle as O


def test_quantiser_hand_computed_values():
    # amax = 1 -> inv = 127 exactly: 0.5*127 = 63.5 and 0.1968503937..*127 = 24.99999.. / 25.0 decide by fp32 rounding
    x = np.array([1.0, -1.0, 0.5, -0.5, 0.25, 0.0, 3.0 / 127.0, 2.5 / 127.0], dtype=np.float32)
    q, scale, inv = O.quantize_int8(x)
    assert inv == np.float32(127.0) and scale == np.float32(1.0) / np.float32(127.0)
    # 63.5 -> 64 (half to even), 31.75 -> 32; 2.5/127 is not exact in fp32: its product with 127 is taken as computed
    t = np.float32(np.float32(2.5 / 127.0) * np.float32(127.0))
    assert list(q[:7]) == [127, -127, 64, -64, 32, 0, 3]
    assert q[7] == int(np.rint(t))


def test_quantiser_ties_go_to_even_and_scale_is_a_division():
    x = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5], dtype=np.float32)     # amax 127 -> inv = 1 exactly
    q, scale, inv = O.quantize_int8(x)
    assert inv == np.float32(1.0) and scale == np.float32(1.0)
    assert list(q) == [127, 0, 2, 2, 0, -2, -2, 126]
    x3 = np.array([3.0, 1.0], dtype=np.float32)
    _, s3, i3 = O.quantize_int8(x3)
    assert s3 == np.float32(3.0) / np.float32(127.0) and i3 == np.float32(127.0) / np.float32(3.0)


def test_quantiser_special_values():
    x = np.array([np.nan, np.inf, -np.inf, 2.0, -4.0, 1e-30], dtype=np.float32)
    q, scale, inv = O.quantize_int8(x)
    assert scale == np.float32(4.0) / np.float32(127.0)                  # the infinities do not set the scale
    assert list(q) == [0, 127, -127, 64, -127, 0]                        # 2*31.75 = 63.5 -> 64
    q0, s0, i0 = O.quantize_int8(np.zeros(5, dtype=np.float32))
    assert s0 == 0 and i0 == 0 and not q0.any()
    qn, sn, _ = O.quantize_int8(np.array([np.nan, np.inf], dtype=np.float32))
    assert sn == 0 and list(qn) == [0, 127]


def test_quantiser_properties_on_random_data():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(20000) * np.exp(rng.standard_normal(20000))).astype(np.float32)
    q, scale, inv = O.quantize_int8(x)
    assert np.abs(q).max() == 127 and q[np.argmax(np.abs(x))] in (127, -127)
    # reconstruction error at most half a step (plus the fp32 rounding of the product), sign preserved, monotone
    err = np.abs(q.astype(np.float64) * float(scale) - x.astype(np.float64))
    assert err.max() <= 0.5 * float(scale) * (1 + 1e-5)
    assert np.all(np.sign(q[q != 0]) == np.sign(x[q != 0]))
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(q[order].astype(np.int32)) >= 0)
    # scale invariance: a power of two in, the same codes out
    q2, scale2, _ = O.quantize_int8(x * np.float32(8.0))
    assert np.array_equal(q, q2) and scale2 == scale * np.float32(8.0)


@pytest.mark.parametrize("B,in_,out", [(1, 1, 1), (5, 7, 3), (16, 33, 20)])
def test_fc_q8_against_integer_matmul(B, in_, out):
    rng = np.random.default_rng(B + in_)
    k = (rng.integers(-127, 128, size=(B, out)) * (rng.random((B, out)) < 0.3)).astype(np.int8)
    W8 = rng.integers(-127, 128, size=(out, in_)).astype(np.int8)
    X8 = rng.integers(-127, 128, size=(B, in_)).astype(np.int8)
    dX, dW = O.linear_backward_q8(k, W8, X8)
    assert dX.dtype == np.int32 and dW.dtype == np.int32
    assert np.array_equal(dX, k.astype(np.int64) @ W8.astype(np.int64))
    assert np.array_equal(dW, k.astype(np.int64).T @ X8.astype(np.int64))
    assert np.array_equal(dW, O.linear_dw_i8(k, X8))                   # the 8-bit mode's own routine agrees


def test_fc_q8_extreme_values_and_overflow_is_reported():
    B, in_, out = 4, 3, 2048
    k = np.full((B, out), 127, dtype=np.int8)
    W8 = np.full((out, in_), -127, dtype=np.int8)
    X8 = np.full((B, in_), 127, dtype=np.int8)
    dX, dW = O.linear_backward_q8(k, W8, X8)
    assert np.all(dX == -127 * 127 * out) and np.all(dW == 127 * 127 * B)
    big = 140000                                                        # 140000 * 127 * 127 > 2^31
    with pytest.raises(OverflowError):
        O.linear_backward_q8(np.full((1, big), 127, np.int8), np.full((big, 1), 127, np.int8), np.zeros((1, 1), np.int8))


def test_conv_q8_brute_force():
    rng = np.random.default_rng(9)
    N, C, H, Wd, K, R, S, pad = 2, 3, 5, 4, 2, 3, 2, 1
    P, Q = H + 2 * pad - R + 1, Wd + 2 * pad - S + 1
    k = (rng.integers(-127, 128, size=(N, K, P, Q)) * (rng.random((N, K, P, Q)) < 0.5)).astype(np.int8)
    W8 = rng.integers(-127, 128, size=(K, C, R, S)).astype(np.int8)
    X8 = rng.integers(-127, 128, size=(N, C, H, Wd)).astype(np.int8)
    dX, dW = O.conv2d_backward_q8(k, W8, X8, stride=1, pad=pad)
    ex = np.zeros((N, C, H, Wd), dtype=object)
    ew = np.zeros((K, C, R, S), dtype=object)
    for n, kk, p, q, c, r, s in itertools.product(range(N), range(K), range(P), range(Q), range(C), range(R), range(S)):
        h, w = p + r - pad, q + s - pad
        if 0 <= h < H and 0 <= w < Wd:
            ex[n, c, h, w] += int(k[n, kk, p, q]) * int(W8[kk, c, r, s])
            ew[kk, c, r, s] += int(k[n, kk, p, q]) * int(X8[n, c, h, w])
    assert np.array_equal(dX, ex.astype(np.int64)) and np.array_equal(dW, ew.astype(np.int64))
    assert np.array_equal(dW, O.conv2d_dw_i8(k, X8, R, S, stride=1, pad=pad))
