"""Pins of the oracle's top-k sparsifier (Sec. "Comparison to meProp": keep the k largest-magnitude elements of each
gradient vector) against things that are not the oracle: a counting definition written out in Python on tiny inputs,
numpy's partition on tie-free inputs, hand-computed roundings, and the degenerate cases."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle


def _kept_by_counting(row, k):
    # the definition itself: kept iff fewer than k elements are strictly larger in magnitude (NaN counts as 0)
    mag = [0.0 if np.isnan(v) else abs(float(v)) for v in row]
    return [sum(1 for o in mag if o > m) < k for m in mag]


def _round_half_up(x, step):
    # floor(x/step + 1/2) in exact rational arithmetic
    q = Fraction(float(x)) / Fraction(float(step)) + Fraction(1, 2)
    return q.numerator // q.denominator


@pytest.mark.parametrize("k", [0, 1, 2, 5, 6, 7, 100])
def test_selection_matches_the_counting_definition_on_tiny_rows(k):
    rng = np.random.default_rng(3)
    d = rng.integers(-4, 5, size=(9, 6)).astype(np.float32) * 0.25        # many ties, zeros included
    d[2, 3] = np.nan
    d[4, 0] = -np.inf
    step = 0.25
    codes, st = oracle.topk_quantize(d, k, step)
    for r in range(d.shape[0]):
        keep = _kept_by_counting(d[r], k)
        for c in range(d.shape[1]):
            v = d[r, c]
            if not keep[c] or np.isnan(v):
                want = 0
            elif np.isinf(v):
                want = 127 if v > 0 else -127
            else:
                want = max(-127, min(127, _round_half_up(v, step)))
            assert codes[r, c] == want, (r, c, v, keep[c])
    assert st.nnz == int(np.count_nonzero(codes))


def test_without_ties_exactly_the_k_largest_survive():
    rng = np.random.default_rng(11)
    rows, cols, k = 7, 1000, 37
    d = rng.standard_normal((rows, cols)).astype(np.float32)
    assert all(len(np.unique(np.abs(d[r]))) == cols for r in range(rows))
    step = float(np.abs(d).max()) / 127 * 1.0001
    thr = oracle.topk_threshold(d, k)
    codes, _ = oracle.topk_quantize(d, k, step)
    for r in range(rows):
        top = np.argpartition(-np.abs(d[r]), k - 1)[:k]
        assert thr[r] == np.abs(d[r])[top].min()
        others = np.setdiff1d(np.arange(cols), top)
        assert not codes[r, others].any()
        # every survivor is far above half a step here (the 37 largest of 1000 normals), so none rounds to 0
        assert np.count_nonzero(codes[r, top]) == k
        want = np.floor(d[r, top].astype(np.float64) / step + 0.5)
        assert np.abs(codes[r, top] - want).max() <= 1          # fp32 fma against fp64: at most one level at a rounding boundary
        assert np.count_nonzero(codes[r, top] != want) <= 1


def test_rounding_is_to_the_nearest_level_halves_upward():
    step = 0.5                                                             # x/step exact in fp32
    x = np.array([[0.25, -0.25, 0.2499, -0.2501, 0.74, 0.75, -0.75, -0.76, 63.4, 63.5, 64.0, -63.5, -63.8, -64.0, 1e9, -1e9]],
                 dtype=np.float32)
    want = np.array([[1, 0, 0, -1, 1, 2, -1, -2, 127, 127, 127, -127, -127, -127, 127, -127]], dtype=np.int8)
    codes, st = oracle.topk_quantize(x, x.shape[1], step)
    np.testing.assert_array_equal(codes, want)
    # |floor| > 127: 64.0/0.5 + 0.5 -> 128, +-1e9, -64.0 -> floor(-127.5) = -128, -63.8 -> floor(-127.1) = -128
    assert st.n_saturated == 5 and st.max_abs_code == 127 and st.n_nonfinite == 0


def test_ties_at_the_threshold_are_all_kept():
    d = np.array([[3.0, -3.0, 3.0, 1.0, 0.0, -2.0]], dtype=np.float32)
    codes, st = oracle.topk_quantize(d, 2, 1.0)
    np.testing.assert_array_equal(codes, [[3, -3, 3, 0, 0, 0]])
    codes, _ = oracle.topk_quantize(d, 4, 1.0)
    np.testing.assert_array_equal(codes, [[3, -3, 3, 0, 0, -2]])
    assert oracle.topk_threshold(d, 4)[0] == 2.0


def test_degenerate_k():
    rng = np.random.default_rng(5)
    d = rng.standard_normal((4, 33)).astype(np.float32)
    none, st0 = oracle.topk_quantize(d, 0, 0.1)
    assert not none.any() and st0.nnz == 0
    assert np.isnan(oracle.topk_threshold(d, 0)).all()
    everything, _ = oracle.topk_quantize(d, 33, 0.1)
    more, _ = oracle.topk_quantize(d, 10 ** 6, 0.1)
    np.testing.assert_array_equal(everything, more)
    want = np.floor(d.astype(np.float64) / np.float64(np.float32(0.1)) + 0.5)
    assert np.count_nonzero(everything != want) <= 1


def test_rows_are_independent_and_sparsity_is_k_over_len():
    rng = np.random.default_rng(9)
    d = (rng.standard_normal((16, 500)) * np.logspace(-3, 3, 16)[:, None]).astype(np.float32)   # rows of very different scale
    k = 25
    for r in range(16):
        step = float(np.abs(d[r]).max()) / 127
        whole, _ = oracle.topk_quantize(d, k, step)
        alone, _ = oracle.topk_quantize(d[r:r + 1], k, step)
        np.testing.assert_array_equal(whole[r], alone[0])
        assert np.count_nonzero(alone) <= k
