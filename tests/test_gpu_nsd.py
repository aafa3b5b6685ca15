"""GPU parity of the NSD pass against the CPU oracle: codes, statistics and the tile-sparse format,
all bit-exact (integer work)."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1), (1, 3), (3, 5), (2, 255), (2, 256), (3, 257), (64, 300), (7, 1000), (5, 1023), (16, 4096),
          (33, 196), (9, 777), (1, 70001), (300, 12)]


@pytest.mark.parametrize("rows,cols", SHAPES)
def test_codes_stats_and_format_match_oracle(rows, cols):
    from gpu_util import check_nsd_against_oracle
    rng = np.random.default_rng(rows * 7919 + cols)
    d = rng.laplace(0, 1e-3, size=(rows, cols)).astype(np.float32)
    step = float(np.float32((2.0 + (rows % 3) * 3) * 1.414e-3))
    check_nsd_against_oracle(d, rows, cols, step, seed=1 + rows)


@pytest.mark.parametrize("idx_base", [0, 1, 2, 3, 255, (1 << 32) - 6, (1 << 33) + 1, (1 << 40) + 123457])
def test_index_base_and_64_bit_counters(idx_base):
    from gpu_util import check_nsd_against_oracle
    rng = np.random.default_rng(5)
    d = rng.laplace(0, 1e-3, size=(6, 1000)).astype(np.float32)
    check_nsd_against_oracle(d, 6, 1000, 2e-3, seed=(7 << 35) + 11, idx_base=idx_base)
    d2 = d[:, :999].copy()
    check_nsd_against_oracle(d2, 6, 999, 2e-3, seed=3, idx_base=idx_base)


def test_special_values_saturation_and_tiny_steps():
    from gpu_util import check_nsd_against_oracle
    rng = np.random.default_rng(6)
    d = rng.laplace(0, 1.0, size=(4, 512)).astype(np.float32)
    d[0, :8] = [np.inf, -np.inf, np.nan, 0.0, -0.0, 1e30, -1e30, 3.0e38]
    d[1, 5] = np.nan
    d[2, 100:110] = 1e-42                      # subnormal inputs
    for step in (0.5, 1e-3, 1e-30, 3e37, 1.0):
        check_nsd_against_oracle(d, 4, 512, step, seed=9)


def test_dense_small_steps_use_the_whole_code_range():
    from gpu_util import check_nsd_against_oracle
    rng = np.random.default_rng(8)
    d = rng.standard_normal((8, 2048)).astype(np.float32)
    got, k = check_nsd_against_oracle(d, 8, 2048, 0.03, seed=2)
    assert got["stats"].max_abs_code == 127 and got["stats"].n_saturated > 0
    assert (k == 0).mean() < 0.05


def test_codes_only_mode_and_determinism():
    from gpu_util import run_nsd
    from oracle import oracle as O
    rng = np.random.default_rng(10)
    d = rng.laplace(0, 1e-3, size=(10, 3000)).astype(np.float32)
    a = run_nsd(d, 10, 3000, 4e-3, 1, with_format=False, with_stats=False)
    b = run_nsd(d, 10, 3000, 4e-3, 1)
    c = run_nsd(d, 10, 3000, 4e-3, 1)
    k_ref, _ = O.nsd(d.ravel(), 4e-3, 1)
    assert np.array_equal(a["codes"].ravel(), k_ref) and np.array_equal(b["codes"], a["codes"])
    assert np.array_equal(b["bitmap"], c["bitmap"]) and np.array_equal(b["tile_nnz"], c["tile_nnz"])
    used = np.arange(256)[None, :] < b["tile_nnz"][:, None].astype(np.int64)      # later slots are undefined
    assert np.array_equal(b["entries"][used], c["entries"][used])


def test_observed_sparsity_matches_prediction_on_the_configs():
    from gpu_util import run_nsd
    for p in [workloads.config1()] + workloads.config2(8.0) + [workloads.config3(N=8), workloads.config4a(N=8)]:
        rows = int(np.prod(p.delta.shape[:-2])) if p.delta.ndim == 4 else p.delta.shape[0]
        cols = p.delta.size // rows
        got = run_nsd(p.delta, rows, cols, p.step, p.seed, with_format=False)
        sparsity = 1 - got["stats"].nnz / p.delta.size
        assert abs(sparsity - p.predicted_sparsity) < 5e-3, (p.name, sparsity, p.predicted_sparsity)
        assert got["stats"].n_saturated == 0 and got["stats"].n_nonfinite == 0
