"""The entry point that allocates nothing (nsd_quantize_static: its scratch is a device array inside the library) against
the entry point it is a variant of (nsd_quantize with a caller's buffer), through the C ABI: codes and statistics bit for
bit, on two calls in a row, the second on a smaller input (the shared scratch keeps the first call's records)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _both(delta, rows, cols, step, seed, idx_base):
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream
    d = dev(delta.reshape(-1))
    L = dbp.format_layout(rows, cols)
    out = []
    for static in (False, True):
        codes = torch.full((rows * cols,), 99, dtype=torch.int8, device="cuda:0")
        st = torch.full((32,), 0xEE, dtype=torch.uint8, device="cuda:0")
        if static:
            dbp.nsd_quantize_static(d, rows, cols, step, seed, idx_base, codes, st, stream())
        else:
            fmt = torch.full((L["total_bytes"],), 0xFF, dtype=torch.uint8, device="cuda:0")
            dbp.nsd_quantize(d, rows, cols, step, seed, idx_base, codes, fmt, st, stream())
        torch.cuda.synchronize()
        s = dbp.Stats.from_tensor(st)
        out.append((codes.cpu().numpy(), (s.nnz, s.n_saturated, s.n_nonfinite, s.max_abs_code)))
    return out


def test_static_scratch_entry_point_matches_nsd_quantize_twice_in_a_row():
    import paper_2004_04729_amd as dbp
    rng = np.random.default_rng(2024)
    # first a tensor large enough for thousands of workgroup records, then a small ragged one
    for rows, cols in ((3000, 4100), (37, 301)):
        d = rng.laplace(0, 1e-3, size=(rows, cols)).astype(np.float32)
        d.reshape(-1)[::997] = 1.0          # saturating values
        d.reshape(-1)[5::4999] = np.nan
        (k_ref, s_ref), (k, s) = _both(d, rows, cols, 4e-3, 7, 123456789)
        assert s_ref[0] > 0 and s_ref[1] > 0 and s_ref[2] > 0
        assert np.array_equal(k, k_ref)
        assert s == s_ref
    # sizes beyond the stated maximum and missing statistics are rejected before any launch
    with pytest.raises(dbp.DbpError) as e:
        dbp.nsd_quantize_static(0x10000, 1 << 20, 1 << 13, 1.0, 1, 0, 0x10000, 0x10000)
    assert e.value.code == 2
    with pytest.raises(dbp.DbpError) as e:
        dbp.nsd_quantize_static(0x10000, 4, 4, 1.0, 1, 0, 0x10000, None)
    assert e.value.code == 1
