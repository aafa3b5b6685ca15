"""Pins for the oracle's NSD quantiser (CPU only).

Each test checks the oracle against something other than itself: frozen vectors, the laws
the paper states for non-subtractive dither (unbiased error, bounded variance, open dither
interval, the sparsity integral), hand-built special cases, or brute force.
"""
import math

import numpy as np
import pytest
from scipy import integrate, special, stats as sps

from oracle import oracle as O

SEED = 1


# ------------------------------------------------------------------ frozen vectors
def test_hash_and_keys_match_frozen_vectors(golden):
    g = golden("dither_vectors.txt")
    seed = int(g["seed"][0][0])
    assert O.keys(seed) == (int(g["k0"][0][0], 16), int(g["k1"][0][0], 16))
    for ctr, word in g["hash"]:
        assert O.hash32(seed, int(ctr)) == int(word, 16)


def test_dither_values_and_worked_example(golden):
    g = golden("dither_vectors.txt")
    seed = int(g["seed"][0][0])
    for idx, num in g["u_num"]:
        assert O.dither_u(seed, int(idx)) == int(num) / 131072.0
    delta = np.array([float(v) for v in g["example_delta"][0]], dtype=np.float32)
    codes, st = O.nsd(delta, float(g["example_step"][0][0]), seed)
    assert codes.tolist() == [int(v) for v in g["example_codes"][0]]
    assert st.nnz == 3 and st.max_abs_code == 2 and st.n_saturated == 0


def test_hash_uses_all_64_bits_of_seed_and_counter():
    base = O.hash32(5, 7)
    assert O.hash32(5 + (1 << 32), 7) != base
    assert O.hash32(5, 7 + (1 << 32)) != base
    assert O.hash32(6, 7) != base and O.hash32(5, 8) != base


# ------------------------------------------------------------------ law of the dither
def _u(n, seed=SEED, base=0):
    # u is recovered through the quantiser itself: with delta = 0 and step = 1, t = u in (0,1),
    # so instead read it from the public scalar function on a sample and in bulk via codes below.
    return np.array([O.dither_u(seed, base + g) for g in range(n)], dtype=np.float64)


def test_dither_is_on_open_interval_and_on_the_17_bit_grid():
    u = _u(200_000)
    assert u.min() >= 2.0 ** -17 and u.max() <= 1.0 - 2.0 ** -17     # never 0 or 1: open interval
    k = u * 131072.0
    assert np.all(k == np.round(k)) and np.all(k.astype(np.int64) % 2 == 1)


def test_dither_is_uniform_and_uncorrelated():
    n = 1 << 18
    u = _u(n)
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 1e-3
    cnt, _ = np.histogram(u, bins=256, range=(0, 1))
    chi2 = ((cnt - n / 256) ** 2 / (n / 256)).sum()
    assert sps.chi2.sf(chi2, 255) > 1e-4
    assert sps.kstest(u, "uniform").pvalue > 1e-4
    c = u - 0.5
    lim = 5 / math.sqrt(n) * (1 / 12)
    # the two halves of one hash word (g even / g odd), neighbours, and long lags
    assert abs(np.mean(c[0::2] * c[1::2])) < lim * math.sqrt(2)
    for lag in (1, 2, 3, 64, 256, 300, 1024, 4096):
        assert abs(np.mean(c[:-lag] * c[lag:])) < lim
    v = _u(n // 4, seed=2) - 0.5
    assert abs(np.mean(c[: n // 4] * v)) < lim * 2


def test_low_bits_of_dither_are_uniform_too():
    u = _u(1 << 17)
    low = ((u * 131072.0).astype(np.int64) >> 1) & 0xFF
    cnt = np.bincount(low, minlength=256)
    chi2 = ((cnt - len(u) / 256) ** 2 / (len(u) / 256)).sum()
    assert sps.chi2.sf(chi2, 255) > 1e-4


# ------------------------------------------------------------------ Eq. (nsd): invariants
def test_code_is_floor_or_floor_plus_one_and_error_below_step():
    rng = np.random.default_rng(3)
    step = np.float32(0.0037)
    d = (rng.standard_normal(300_000) * 0.004).astype(np.float32)
    k, st = O.nsd(d, float(step), SEED)
    s = d.astype(np.float64) / np.float64(step)
    # the fp32 product d*inv may sit an ulp beside the exact ratio: allow that sliver
    eps = 1e-6 * np.abs(s) + 1e-9
    assert np.all(k >= np.floor(s - eps)) and np.all(k <= np.floor(s + eps) + 1)
    assert np.all(np.abs(k * np.float64(step) - d) < np.float64(step) * (1 + 1e-5))
    assert st.nnz == np.count_nonzero(k) and st.max_abs_code == np.abs(k).max()


def test_matches_direct_evaluation_of_eq_nsd_in_exact_arithmetic():
    # Delta * floor((x + nu)/Delta + 1/2) with nu = (u - 1/2) Delta, in fp64 on inputs chosen as
    # multiples of 2^-10 with Delta = 2^-3, so every fp32 step of the oracle is exact.
    rng = np.random.default_rng(11)
    step = 0.125
    d = (rng.integers(-4000, 4000, size=50_000) / 1024.0).astype(np.float32)
    k, _ = O.nsd(d, step, SEED, idx_base=12345)
    u = np.array([O.dither_u(SEED, 12345 + g) for g in range(d.size)])
    nu = (u - 0.5) * step
    q = step * np.floor((d.astype(np.float64) + nu) / step + 0.5)
    assert np.array_equal(k.astype(np.float64) * step, q)


@pytest.mark.parametrize("s", [0.0, 0.003, 0.25, 0.5, 0.731, -0.4, -1.25, 3.9, -17.5])
def test_unbiased_with_variance_f_times_one_minus_f(s):
    # E[eps] = 0 and E[eps^2] < Delta^2/4 (Sec. "Non-subtractive dithered quantization");
    # for uniform dither the exact variance is Delta^2 f (1-f), f = frac(x/Delta).
    n = 1_000_000
    step = 0.01
    d = np.full(n, s * step, dtype=np.float32)
    k, _ = O.nsd(d, step, SEED, idx_base=777)
    s_eff = float(np.float32(s * step)) / float(np.float32(step))
    f = s_eff - math.floor(s_eff)
    assert abs(k.mean() - s_eff) < 4 * 0.5 / math.sqrt(n)          # 2e-3
    assert abs(k.var() - f * (1 - f)) < 2e-3
    assert k.var() <= 0.25 + 1e-3
    assert set(np.unique(k).tolist()) <= {math.floor(s_eff), math.floor(s_eff) + 1}


def test_probability_of_nonzero_code_is_abs_delta_over_step():
    n = 400_000
    step = 0.02
    for r in (0.01, 0.1, 0.37, 0.5, 0.9, 0.99):
        for sign in (1, -1):
            d = np.full(n, sign * r * step, dtype=np.float32)
            k, st = O.nsd(d, step, SEED, idx_base=31)
            assert abs(st.nnz / n - r) < 4 * math.sqrt(r * (1 - r) / n) + 2e-5
            assert set(np.unique(k).tolist()) <= {0, sign}
    for r in (1.0, 1.5, 7.25):
        d = np.full(1000, -r * step, dtype=np.float32)
        assert O.nsd(d, step, SEED)[1].nnz == 1000                # |delta| >= Delta: never zero


# ------------------------------------------------------------------ sparsity model
def _paper_sparsity_integral(s):
    """P(0) = int_{-D/2}^{D/2} (G_sigma * U_D)(t) dt with D = s*sigma, sigma = 1, by quadrature.

    (G*U)(t) = [Phi(t + D/2) - Phi(t - D/2)] / D.  Sec. "Effects of applying NSD to the gradients".
    """
    D = float(s)
    f = lambda t: (sps.norm.cdf(t + D / 2) - sps.norm.cdf(t - D / 2)) / D
    return integrate.quad(f, -D / 2, D / 2, epsabs=1e-12)[0]


@pytest.mark.parametrize("s,expect", [(1, 0.3688), (2, 0.6096), (4, 0.8005), (8, 0.9003)])
def test_gaussian_sparsity_matches_the_papers_integral(s, expect):
    closed = special.erf(s / math.sqrt(2)) - 2 / (s * math.sqrt(2 * math.pi)) * (1 - math.exp(-s * s / 2))
    assert abs(_paper_sparsity_integral(s) - closed) < 1e-9
    assert abs(closed - expect) < 5e-4
    rng = np.random.default_rng(5)
    d = rng.standard_normal(1_000_000).astype(np.float32) * 0.003
    step = float(np.float32(s * d.astype(np.float64).std()))
    _, st = O.nsd(d, step, SEED)
    assert abs(1 - st.nnz / d.size - closed) < 5e-3


@pytest.mark.parametrize("c,expect", [(2, 0.667), (4, 0.824), (8, 0.912)])
def test_laplace_sparsity_closed_form(c, expect):
    # E max(0, 1-|x|/D) for x ~ Laplace(b), t = D/b:  1 - (1 - e^-t)/t ;  D = c*std = c*b*sqrt(2)
    t = c * math.sqrt(2)
    closed = 1 - (1 - math.exp(-t)) / t
    assert abs(closed - expect) < 1e-3
    rng = np.random.default_rng(6)
    d = rng.laplace(0, 1e-3, size=1_000_000).astype(np.float32)
    step = float(np.float32(c * d.astype(np.float64).std()))
    _, st = O.nsd(d, step, SEED)
    assert abs(1 - st.nnz / d.size - closed) < 5e-3


def test_sparsity_grows_and_code_width_shrinks_with_step():
    rng = np.random.default_rng(7)
    d = rng.laplace(0, 1e-3, size=200_000).astype(np.float32)
    last_nnz, last_max = d.size + 1, 1 << 30
    for c in (0.25, 0.5, 1, 2, 4, 8, 16):
        _, st = O.nsd(d, c * 1.414e-3, SEED)
        assert st.nnz < last_nnz and st.max_abs_code <= last_max
        last_nnz, last_max = st.nnz, st.max_abs_code


# ------------------------------------------------------------------ special cases
def test_saturation_nonfinite_and_zero_inputs():
    step = 0.5
    d = np.array([200 * step, -200 * step, np.inf, -np.inf, np.nan, 0.0, -0.0, 126.2 * step, -127.9 * step, 1e-45],
                 dtype=np.float32)
    k, st = O.nsd(d, step, SEED)
    assert k[:5].tolist() == [127, -127, 127, -127, 0]
    assert k[5] in (0,) and k[6] in (0,)
    assert k[7] in (126, 127) and k[8] in (-127,) and k[9] == 0
    assert st.n_nonfinite == 3
    assert st.n_saturated == 4 + int(math.floor(np.float32(-127.9) + O.dither_u(SEED, 8)) < -127)
    assert st.max_abs_code == 127


def test_index_base_shifts_the_counter():
    rng = np.random.default_rng(8)
    d = rng.laplace(0, 1e-3, size=5001).astype(np.float32)
    full, _ = O.nsd(d, 2e-3, 9, idx_base=10)
    for a in (1, 2, 777, 4096):
        part, _ = O.nsd(d[a:], 2e-3, 9, idx_base=10 + a)
        assert np.array_equal(part, full[a:])
    other, _ = O.nsd(d, 2e-3, 10, idx_base=10)
    assert not np.array_equal(other, full)


# ------------------------------------------------------------------ tile-sparse format
@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 255), (2, 256), (5, 300), (4, 1000), (2, 513)])
def test_tile_format_decodes_back_to_the_code_plane(rows, cols):
    rng = np.random.default_rng(rows * 1000 + cols)
    codes = (rng.integers(-3, 4, size=(rows, cols)) * (rng.random((rows, cols)) < 0.2)).astype(np.int8)
    codes[0, 0] = -128 + 1
    bitmap, tile_nnz, entries = O.tile_format(codes, rows, cols)
    tpr = (cols + 255) // 256
    dec = np.zeros_like(codes)
    for r in range(rows):
        for s in range(tpr):
            t = r * tpr + s
            bits = sum(bin(int(w)).count("1") for w in bitmap[t])
            assert bits == tile_nnz[t]
            prev = -1
            for i in range(int(tile_nnz[t])):
                e = int(entries[t, i])
                c, v = e >> 8, np.int8(np.uint8(e & 0xFF))
                assert c > prev and (int(bitmap[t, c & 3]) >> (c >> 2)) & 1
                prev = c
                dec[r, s * 256 + c] = v
            assert np.all(entries[t, int(tile_nnz[t]):] == 0xFFFF)          # untouched slots
    assert np.array_equal(dec, codes)


# ---- the step before the quantiser and its by-product (delta_z = delta_a (.) f'(z); delta_b = sum q) ----

def test_relu_backward_is_the_hadamard_product_with_the_step_function():
    from oracle import oracle as O
    # worked by hand: f'(z) = [z > 0]; -0.0, 0.0 and NaN mask the element
    da = np.array([1.5, -2.0, 3.0, 4.0, 5.0, -6.0], dtype=np.float32)
    z = np.array([0.1, -0.1, 0.0, -0.0, np.nan, 7.0], dtype=np.float32)
    assert O.relu_backward(da, z).tolist() == [1.5, 0.0, 0.0, 0.0, 0.0, -6.0]
    rng = np.random.default_rng(3)
    da = rng.standard_normal((37, 129)).astype(np.float32)
    z = rng.standard_normal((37, 129)).astype(np.float32)
    got = O.relu_backward(da, z)
    assert np.array_equal(got, da * (z > 0))                       # Hadamard product with the 0/1 derivative
    assert np.array_equal(got, O.relu_backward(da, np.maximum(z, 0)))   # a = f(z) carries the same sign information


def test_bias_gradient_is_the_batch_sum_of_the_quantised_gradient():
    from oracle import oracle as O
    # worked by hand, FC: codes [3 x 2], Delta = 0.5: column sums (1-2+4, 0+5-1) = (3, 4) -> (1.5, 2.0)
    k = np.array([[1, 0], [-2, 5], [4, -1]], dtype=np.int8)
    s, g = O.bias_grad(k, 3, 2, True, 2, 0.5)
    assert s.tolist() == [3, 4] and g.tolist() == [1.5, 2.0]
    # conv: rows are (n, ch) with ch fastest; N = 2, K = 3, 2 pixels: channel sums over n and pixels
    k = np.array([[1, 2], [3, 4], [5, 6], [-1, -2], [-3, -5], [7, 0]], dtype=np.int8)
    s, g = O.bias_grad(k, 6, 2, False, 3, 2.0)
    assert s.tolist() == [0, -1, 18] and g.tolist() == [0.0, -2.0, 36.0]
    # against numpy on random codes, and against the float sum of q = k*Delta (exact here: small integers, Delta = 2^-3)
    rng = np.random.default_rng(5)
    k = rng.integers(-127, 128, size=(64, 300)).astype(np.int8)
    s, g = O.bias_grad(k, 64, 300, True, 300, 0.125)
    assert np.array_equal(s, k.astype(np.int64).sum(axis=0))
    assert np.array_equal(g, (k.astype(np.float64) * 0.125).sum(axis=0).astype(np.float32))
    k4 = rng.integers(-127, 128, size=(5, 7, 3, 4)).astype(np.int8)               # N, K, P, Q
    s, _ = O.bias_grad(k4, 35, 12, False, 7, 1.0)
    assert np.array_equal(s, k4.astype(np.int64).sum(axis=(0, 2, 3)))
    # the sum over the batch of an unbiased quantiser is unbiased for the true bias gradient (Eq. (unbiased))
    d = rng.laplace(0, 1e-3, size=(4096, 8)).astype(np.float32)
    step = 4e-3
    kk, _ = O.nsd(d, step, 11)
    _, g = O.bias_grad(kk, 4096, 8, True, 8, step)
    true = d.astype(np.float64).sum(axis=0)
    # variance of one element's error <= Delta^2/4 (Eq. (bounded variance)): 5 sigma of the sum
    assert np.all(np.abs(g - true) < 5 * np.sqrt(4096 * step * step / 4))


# ---- step size of a layer: Algorithm 1, sigma = std(delta_z), Delta = s*sigma ----

def test_step_size_is_s_times_the_population_standard_deviation():
    from oracle import oracle as O
    # closed forms: +-a in equal numbers -> sigma = a;  0..n-1 -> sqrt((n^2-1)/12);  constant -> 0
    x = np.array([0.25, -0.25] * 500, dtype=np.float32)
    step, sigma = O.step_size(x, 4)
    assert sigma == 0.25 and step == 1.0
    n = 1000
    step, sigma = O.step_size(np.arange(n, dtype=np.float32), 1)
    assert abs(sigma - np.sqrt((n * n - 1) / 12.0)) < 1e-9
    assert O.step_size(np.full(77, 3.5, dtype=np.float32), 8) == (0.0, 0.0)
    # worked by hand: (1, 2, 3, 6): mean 3, squared deviations 4+1+0+9 = 14, variance 3.5
    step, sigma = O.step_size(np.array([1, 2, 3, 6], dtype=np.float32), 2)
    assert sigma == np.sqrt(3.5) and step == np.float32(2 * np.sqrt(3.5))
    # against numpy's two-pass fp64 std on the workloads' gradient laws, any size (ragged groups of the tree)
    rng = np.random.default_rng(7)
    for size in (1, 15, 16, 17, 255, 4097, 70001):
        d = rng.laplace(0, 1e-3, size=size).astype(np.float32)
        step, sigma = O.step_size(d, 8)
        ref = np.std(d.astype(np.float64))
        assert abs(sigma - ref) <= 1e-12 * max(ref, 1e-30) + 1e-18
        assert step == np.float32(8 * sigma)
    # a shifted distribution (mean >> sigma) still resolves sigma: fp64 sums of fp32 values
    d = (1.0 + rng.standard_normal(50000) * 1e-3).astype(np.float32)
    _, sigma = O.step_size(d, 1)
    assert abs(sigma - np.std(d.astype(np.float64))) < 1e-9
    # scaling the data by a power of two scales Delta exactly (no dependence on magnitude)
    d = rng.laplace(0, 1e-3, size=5000).astype(np.float32)
    assert O.step_size(d * 8, 4)[0] == 8 * O.step_size(d, 4)[0]


def test_step_size_summation_order_is_the_radix16_tree():
    from oracle import oracle as O
    # Values for which the ORDER of the fp64 additions changes the sum of squares: 2^54 absorbs a following 1.0
    # (spacing 4 up there) but not a following 16.0.  x = (2^27, then 31 ones): the tree sums group 0 of the
    # squares to 2^54 (its 15 ones absorbed one by one) and group 1 to 16 exactly, total 2^54 + 16; a plain
    # left-to-right sum absorbs all 31 ones (2^54); a pairwise tree gives 2^54 + 28 (two ones paired with each
    # other first everywhere but next to the big value).  S1 = 2^27 + 31 exactly in every order.
    def sigma_of(s1, s2, n):
        return float(np.sqrt((np.float64(s2) - np.float64(s1) * np.float64(s1) / np.float64(n)) / np.float64(n)))
    x = np.array([2.0 ** 27] + [1.0] * 31, dtype=np.float32)
    _, sigma = O.step_size(x, 1)
    s1 = 2.0 ** 27 + 31.0
    tree, sequential = sigma_of(s1, 2.0 ** 54 + 16.0, 32), sigma_of(s1, 2.0 ** 54, 32)
    assert tree != sequential
    assert sigma == tree
    # second level of the tree: 17 groups; group 0 = 2^54 (15 ones absorbed), groups 1..16 = 16 each;
    # level 2: 2^54 + 15*16 (exact, multiples of 4), then + 16
    y = np.array([2.0 ** 27] + [1.0] * (15 + 16 * 16), dtype=np.float32)
    _, sigma = O.step_size(y, 1)
    assert sigma == sigma_of(2.0 ** 27 + 271.0, 2.0 ** 54 + 256.0, y.size)
    assert sigma != sigma_of(2.0 ** 27 + 271.0, 2.0 ** 54, y.size)


def test_tile_format_matches_the_hand_written_tile(golden):
    # pins the bit order of the bitmap and the entry encoding with a tile written out by hand (tests/golden)
    g = golden("tile_format_example.txt")
    rows, cols = int(g["rows"][0][0]), int(g["cols"][0][0])
    codes = np.array([int(v) for v in g["codes"][0]], dtype=np.int8)
    bitmap, tile_nnz, entries = O.tile_format(codes, rows, cols)
    assert [int(w) for w in bitmap[0]] == [int(v, 16) for v in g["bitmap"][0]]
    assert int(tile_nnz[0]) == int(g["tile_nnz"][0][0])
    assert [int(e) for e in entries[0, :int(tile_nnz[0])]] == [int(v, 16) for v in g["entries"][0]]
