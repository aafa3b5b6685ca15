"""GPU parity of the convolutional backward products (implicit-im2col GEMMs) against the CPU oracle."""
import numpy as np
import pytest

import workloads
from workloads import ConvProblem

pytestmark = pytest.mark.gpu


def _problem(N, C, H, Wd, K, R, S, pad, c=4.0, seed=0, i8=False, stride=1):
    rng = np.random.default_rng(seed + N * 131 + C * 17 + H * 5 + K)
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    X = workloads.int8_relu_uniform(rng, (N, C, H, Wd)) if i8 else workloads.relu_normal(rng, (N, C, H, Wd))
    W = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
    d = rng.laplace(0, 5e-4, size=(N, K, P, Q)).astype(np.float32)
    return ConvProblem("t_n%d_c%d_%dx%d_k%d_%dx%d_p%d_s%d" % (N, C, H, Wd, K, R, S, pad, stride), d, W, X,
                       float(np.float32(c * 7.071e-4)), stride, pad)


def _check(p, res):
    """Codes, statistics and every element of both products against the oracle."""
    from gpu_util import check_products
    from oracle import oracle as O
    k_ref, st = O.nsd(p.delta, p.step, p.seed)
    assert np.array_equal(res["codes"], k_ref)
    if res.get("stats") is not None:
        assert res["stats"].nnz == st.nnz and res["stats"].max_abs_code == st.max_abs_code
    i8 = p.X.dtype == np.int8
    Xf = p.X.astype(np.float32)
    kw = dict(stride=p.stride, pad=p.pad)
    rX, rW, _ = O.conv2d_backward(p.W, Xf, codes=k_ref, step=p.step, want_dw=not i8, **kw)
    aX, aW, _ = O.conv2d_backward(np.abs(p.W), np.abs(Xf), codes=np.abs(k_ref), step=p.step, want_dw=not i8, **kw)
    if res["dX"] is not None:
        check_products(res["dX"], rX, aX, p.name + " dX")
    if res["dW"] is not None:
        if i8:
            assert np.array_equal(res["dW"], O.conv2d_dw_i8(k_ref, p.X, p.W.shape[2], p.W.shape[3], p.stride, p.pad))
        else:
            check_products(res["dW"], rW, aW, p.name + " dW")


CASES = [  # N, C, H, Wd, K, R, S, pad
    (1, 1, 1, 1, 1, 1, 1, 0),
    (2, 5, 9, 7, 6, 3, 3, 1),
    (3, 16, 14, 14, 24, 3, 3, 1),
    (2, 33, 14, 14, 20, 1, 1, 0),
    (2, 3, 11, 8, 4, 5, 3, 2),
    (2, 8, 10, 10, 9, 3, 3, 0),
    (5, 40, 12, 20, 70, 3, 3, 1),
    (1, 130, 6, 6, 260, 3, 3, 1),
    (2, 7, 12, 9, 5, 5, 3, 2),          # R != S, wide padding
    (1, 4, 6, 6, 3, 3, 3, 3),           # padding beyond the kernel extent
    (2, 64, 30, 30, 40, 3, 3, 1),       # several pixel tiles per image, tile borders inside a row
    (2, 6, 12, 9, 10, 3, 3, 1),         # odd row length: element-wise scatter into the staging buffers
    (17, 70, 8, 8, 130, 3, 3, 1),       # more images than one reduction split takes, partial channel tiles
    (2, 16, 12, 12, 24, 1, 3, 0),       # three taps in a row: the three-set weight ring with one turn per chunk
    (2, 40, 12, 12, 24, 3, 1, 1),       # three taps in a column, output wider than the input (padding on a 1-wide kernel)
    (2, 16, 12, 12, 40, 2, 3, 1),       # six taps
    (2, 16, 13, 12, 24, 3, 2, 1),       # six taps the other way round, odd height
    (32, 256, 48, 48, 16, 3, 3, 1),     # 704 workgroups: two rounds over the chip, the second one partly filled
    (2, 24, 16, 16, 40, 3, 3, 0),       # 14-wide code rows under 16-wide image rows: the dW stager's half-piece path for the codes alone
    (3, 70, 18, 18, 130, 3, 3, 1),      # 18-wide rows (even, not a multiple of 4): half-piece path for both operands, partial tiles
    (2, 64, 10, 14, 64, 3, 3, 1),       # the same on whole tiles, more rows than columns
]


@pytest.mark.parametrize("case", CASES)
def test_conv_products_match_oracle(case):
    from gpu_util import run_conv
    p = _problem(*case)
    _check(p, run_conv(p))


@pytest.mark.parametrize("case", CASES[1:])
def test_conv_int8_mode_is_bit_exact(case):
    from gpu_util import run_conv
    p = _problem(*case, c=1.0, i8=True)
    _check(p, run_conv(p))


GATHER = [  # N, C, H, Wd, K, R, S, pad, stride: the kernels that walk the nonzero entries of the tile-sparse format
    (2, 5, 9, 7, 6, 3, 3, 1, 1),
    (3, 16, 14, 14, 24, 3, 3, 1, 1),
    (2, 33, 14, 14, 20, 1, 1, 0, 1),        # 1x1: 64 channels per wavefront
    (2, 3, 11, 8, 4, 5, 3, 2, 1),           # 15 taps: 4 channels per wavefront, wide padding
    (2, 8, 23, 20, 8, 7, 7, 3, 2),          # 49 taps: one channel per wavefront; stride 2
    (4, 64, 28, 28, 40, 3, 3, 1, 2),
    (2, 40, 20, 24, 70, 3, 3, 1, 1),        # planes of more than one 256-pixel tile
    (1, 30, 40, 40, 8, 3, 3, 1, 1),         # input planes too large for seven per wavefront: fewer channels per workgroup
    # the kernels that scan the code planes (3x3 and 1x1, planes a multiple of 4 bytes; dX: stride 1)
    (3, 70, 14, 14, 130, 3, 3, 1, 1),       # two channel blocks and five plane blocks, both ragged; dW summed over shares of the images
    (2, 64, 56, 56, 40, 3, 3, 1, 1),        # several row bands per image on both products
    (2, 20, 12, 12, 40, 3, 3, 0, 1),        # no padding: the output is smaller than the input
    (2, 20, 12, 12, 36, 3, 3, 2, 1),        # padding 2: code rows and columns beyond the image on every side
    (2, 96, 16, 16, 48, 1, 1, 0, 1),        # 1x1
    (9, 16, 6, 6, 8, 3, 3, 1, 1),           # tiny planes (36 codes): one dword pass covers several rows
    (2, 24, 20, 100, 8, 3, 3, 1, 1),        # wide rows: two dword passes per plane in the dX kernel
]


@pytest.mark.parametrize("case", GATHER)
def test_conv_gather_path_matches_oracle(case):
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    p = _problem(*case[:8], stride=case[8])
    _check(p, run_conv(p, path=dbp.PATH_GATHER))
    p8 = _problem(*case[:8], c=1.0, i8=True, stride=case[8])      # int8 X: exact int32 dW
    _check(p8, run_conv(p8, path=dbp.PATH_GATHER))


def test_conv_gather_very_sparse_and_empty_planes():
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    p = _problem(3, 20, 16, 16, 12, 3, 3, 1, c=40.0)               # step 40 sigma: almost every plane is empty
    _check(p, run_conv(p, path=dbp.PATH_GATHER))
    mf = run_conv(p, path=dbp.PATH_MFMA)
    assert np.array_equal(mf["codes"], run_conv(p, path=dbp.PATH_GATHER)["codes"])


I8_ROWS = [  # 3x3, padding 1, rows of a multiple of 4 pixels: the int8 dW kernel that loads whole 16-pixel cells
    (2, 64, 16, 16, 64, 3, 3, 1),       # one full cell per row, a whole image per unit
    (2, 70, 32, 32, 130, 3, 3, 1),      # two full cells; partial channel tiles on both sides
    (3, 24, 17, 44, 40, 3, 3, 1),       # a partly filled last cell; image rows not a multiple of the unit
    (1, 8, 5, 100, 16, 3, 3, 1),        # wide rows, few rows per unit
    (2, 16, 9, 224, 8, 3, 3, 1),        # widest rows served: single-row units
    (1, 8, 1, 16, 8, 3, 3, 1),          # an image of one row
    (9, 64, 28, 28, 64, 3, 3, 1),       # a single tile: the reduction split over many units
    (2, 32, 56, 56, 32, 3, 3, 1),       # the row geometry of the 8-bit VGG layer
    (1, 16, 20, 228, 16, 3, 3, 1),      # rows too wide for it: the other kernels serve
]


@pytest.mark.parametrize("case", I8_ROWS)
def test_conv_int8_whole_cell_rows_bit_exact(case):
    from gpu_util import run_conv
    p = _problem(*case, c=1.0, i8=True)
    _check(p, run_conv(p))


LOWERED = [  # N, C, H, Wd, K, R, S, pad, stride: large enough that dW runs as column matrix x fully connected kernels
    (32, 128, 14, 14, 256, 1, 1, 0, 1),     # 1x1: the column matrix is the transposed activations
    (16, 64, 28, 28, 128, 3, 3, 1, 2),      # 3x3 / 2
    (8, 32, 20, 20, 96, 5, 5, 2, 1),        # 5x5, several bands of rows per image
    (16, 64, 15, 15, 128, 3, 3, 1, 1),      # rows of 15 pixels: codes re-laid a byte at a time
    (64, 132, 24, 20, 264, 1, 1, 0, 2),     # 1x1 / 2, channel counts that are not tile multiples
]


@pytest.mark.parametrize("case", LOWERED)
def test_conv_dw_lowered_to_fc_kernels(case):
    from gpu_util import run_conv
    p = _problem(*case[:8], stride=case[8])
    _check(p, run_conv(p))
    p8 = _problem(*case[:8], c=1.0, i8=True, stride=case[8])      # int8 X: the same lowering on the int8 kernels, exact int32
    _check(p8, run_conv(p8))


ONE_BY_ONE = [  # N, C, H, Wd, K: 1x1, stride 1, no padding, more than 128 output channels: dW straight from the NCHW tensors
    (4, 36, 14, 14, 130),       # 196 pixels: six windows of 32 and one that overlaps; partial row and column tiles
    (3, 64, 8, 8, 200),         # 64 pixels: whole windows only
    (5, 16, 6, 6, 140),         # 36 pixels: the second window repeats 28 indices of the first
    (70, 128, 14, 14, 256),     # the reduction split over groups of images
    (2, 260, 10, 10, 300),      # several column tiles, two row tiles
    (6, 96, 12, 12, 64),        # 64 output channels: a quarter of the 256-row tile, the fewest this kernel takes
    (4, 200, 8, 16, 100),       # 100 output channels, ragged against every tile size
]


@pytest.mark.parametrize("case", ONE_BY_ONE)
def test_conv_1x1_dw_batched_fc_kernel(case):
    from gpu_util import run_conv
    N, C, H, Wd, K = case
    p = _problem(N, C, H, Wd, K, 1, 1, 0)
    _check(p, run_conv(p))


ONE_BY_ONE_I8 = [  # the same with int8 activations: windows of 64 pixels
    (4, 36, 14, 14, 130),       # 196 pixels: three windows and one that overlaps; partial row and column tiles
    (3, 64, 8, 8, 200),         # 64 pixels: one whole window per image
    (5, 16, 10, 10, 140),       # 100 pixels: the second window repeats 28 indices of the first
    (70, 128, 14, 14, 256),     # the reduction split over groups of images
    (2, 260, 10, 10, 300),      # several column tiles, two row tiles
    (3, 16, 6, 6, 140),         # 36 pixels, less than a window: the other kernels serve
    (6, 96, 12, 12, 64),        # 64 output channels: a quarter of the row tile
    (4, 200, 8, 16, 100),       # 100 output channels
]


@pytest.mark.parametrize("case", ONE_BY_ONE_I8)
def test_conv_1x1_dw_batched_fc_kernel_int8_bit_exact(case):
    from gpu_util import run_conv
    N, C, H, Wd, K = case
    p = _problem(N, C, H, Wd, K, 1, 1, 0, c=1.0, i8=True)
    _check(p, run_conv(p))


STRIDED = [  # N, C, H, Wd, K, R, S, pad, stride  (the strided layers of a ResNet: 3x3/2, 1x1/2 shortcuts, 7x7/2 stem)
    (2, 5, 9, 7, 6, 3, 3, 1, 2),
    (3, 16, 14, 14, 24, 3, 3, 1, 2),
    (2, 33, 14, 14, 20, 1, 1, 0, 2),
    (2, 3, 23, 20, 8, 7, 7, 3, 2),
    (2, 8, 11, 13, 9, 3, 3, 0, 3),       # stride 3, sizes that leave a remainder
    (4, 64, 28, 28, 128, 3, 3, 1, 2),
    # strided dX as st*st stride-1 problems in one launch (taken when P*Q is a multiple of 4):
    (2, 33, 16, 16, 20, 1, 1, 0, 2),     # 1x1 / 2: three classes without taps (cleared), one with the single tap
    (2, 16, 12, 20, 24, 3, 3, 1, 2),
    (2, 8, 15, 17, 8, 3, 3, 1, 2),       # odd image sizes: the classes have different extents
    (2, 8, 16, 16, 8, 2, 2, 0, 2),       # even kernel: every class has exactly one tap
    (1, 130, 8, 8, 70, 3, 3, 1, 2),      # partial channel blocks
    (3, 12, 20, 24, 10, 5, 5, 2, 2),     # 5x5 / 2: classes of 3x3, 3x2, 2x3, 2x2 taps
    (1, 8, 17, 17, 8, 3, 3, 1, 4),       # stride 4: more classes than one launch takes, generic kernel
]


@pytest.mark.parametrize("case", STRIDED)
def test_conv_strided_matches_oracle(case):
    from gpu_util import run_conv
    p = _problem(*case[:8], stride=case[8])
    _check(p, run_conv(p))
    p8 = _problem(*case[:8], c=1.0, i8=True, stride=case[8])
    _check(p8, run_conv(p8))


def test_conv_dense_codes_and_structured_zeros():
    from gpu_util import run_conv
    p = _problem(2, 12, 10, 10, 40, 3, 3, 1, c=0.02)
    res = run_conv(p)
    assert np.abs(res["codes"]).max() == 127
    _check(p, res)
    p = _problem(4, 12, 16, 16, 40, 3, 3, 1, c=8.0)
    p.delta[:] = workloads.structured_planes(p.delta, 0.5)
    _check(p, run_conv(p))
    p.delta[:] = 0
    res = run_conv(p)
    assert not res["dX"].any() and not res["dW"].any()


def test_conv_single_products_and_determinism():
    from gpu_util import run_conv
    p = _problem(3, 16, 14, 14, 24, 3, 3, 1)
    a = run_conv(p)
    b = run_conv(p)
    assert a["dX"].tobytes() == b["dX"].tobytes() and a["dW"].tobytes() == b["dW"].tobytes()
    only_dx = run_conv(p, want_dw=False)
    only_dw = run_conv(p, want_dx=False)
    assert only_dx["dX"].tobytes() == a["dX"].tobytes() and only_dw["dW"].tobytes() == a["dW"].tobytes()


def test_dense_conv_baseline_matches_oracle():
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream, check_products, conv_dims
    from oracle import oracle as O
    for case in (CASES[1], CASES[2], CASES[3]):
        p = _problem(*case)
        N, Cc, H, Wd, K, R, S = conv_dims(p)
        dX = torch.empty(p.X.shape, dtype=torch.float32, device="cuda:0")
        dW = torch.empty(p.W.shape, dtype=torch.float32, device="cuda:0")
        ws = torch.empty(dbp.conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, 1, p.pad), dtype=torch.uint8, device="cuda:0")
        dbp.dense_conv2d_backward(dev(p.delta), dev(p.W), dev(p.X), dbp.F32, N, Cc, H, Wd, K, R, S, 1, p.pad, dX, dW, ws, stream())
        torch.cuda.synchronize()
        rX, rW, _ = O.conv2d_backward(p.W, p.X, dense=p.delta, pad=p.pad)
        aX, aW, _ = O.conv2d_backward(np.abs(p.W), np.abs(p.X), dense=np.abs(p.delta), pad=p.pad)
        check_products(dX.cpu().numpy(), rX, aX, "dense conv dX")
        check_products(dW.cpu().numpy(), rW, aW, "dense conv dW")


def test_config3_reduced_batch_in_full():
    from gpu_util import run_conv
    p = workloads.config3(N=4)
    _check(p, run_conv(p))


# The configurations at their real sizes, every output element of both products against the oracle (the launch
# geometry of the benchmark: all tiles, split-K slots and workgroup numberings of the full grid are covered).
@pytest.mark.parametrize("make", [workloads.config3, workloads.config4a, workloads.config4b])
def test_fp32_conv_configs_full_size_in_full(make):
    from gpu_util import run_conv
    p = make()
    res = run_conv(p)
    assert abs(1 - res["stats"].nnz / p.delta.size - p.predicted_sparsity) < 5e-3
    assert res["stats"].n_saturated == 0
    _check(p, res)


@pytest.mark.parametrize("target", [0.5, 0.9, 0.99])
def test_config5_int8_full_size_in_full(target):
    from gpu_util import run_conv
    p = workloads.config5(target)
    res = run_conv(p)
    assert abs(1 - res["stats"].nnz / p.delta.size - target) < 5e-3
    assert res["stats"].n_saturated == 0
    _check(p, res)


def _auto_conv(p, want_dx=True, stats=True, path=None):
    """dithered_conv2d_backward with DBP_PATH_AUTO; returns the results and the three density flags the device wrote."""
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream, conv_dims
    N, Cc, H, Wd, K, R, S = conv_dims(p)
    codes = torch.empty(p.delta.shape, dtype=torch.int8, device="cuda:0")
    dX = torch.full(p.X.shape, float("nan"), dtype=torch.float32, device="cuda:0") if want_dx else None
    i8 = p.X.dtype == np.int8
    xd = dbp.I8 if i8 else dbp.F32
    dW = torch.full(p.W.shape, -77, dtype=torch.int32, device="cuda:0") if i8 else torch.full(p.W.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.zeros(dbp.conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, p.stride, p.pad, xd), dtype=torch.uint8, device="cuda:0")
    off = dbp.format_layout(N * K, p.delta.shape[2] * p.delta.shape[3])["scratch_offset"] + 16384 * 16
    ws[off:off + 12] = 255                                     # reads back as -1 unless a gated call writes the flags
    st = torch.zeros(32, dtype=torch.uint8, device="cuda:0") if stats else None
    dbp.dithered_conv2d_backward(dev(p.delta), dev(p.W), dev(p.X), xd, N, Cc, H, Wd, K, R, S, p.stride, p.pad, p.step, p.seed, 0,
                                 codes, dX, dW, ws, st, dbp.PATH_AUTO if path is None else path, stream())
    torch.cuda.synchronize()
    flags = [int(v) for v in ws[off:off + 12].cpu().numpy().view(np.int32)]
    res = {"codes": codes.cpu().numpy(), "dX": dX.cpu().numpy() if want_dx else None, "dW": dW.cpu().numpy(),
           "stats": dbp.Stats.from_tensor(st) if stats else None}
    return res, flags


@pytest.mark.parametrize("target,expect", [(0.92, [0, 0, 1]), (0.985, [0, 1, 0]), (0.999, [0, 1, 0])])
def test_conv_auto_dispatches_by_density_on_the_device(target, expect):
    # the ResNet-stage layer behind the density gate, decided on the device from the quantiser's nonzero count: matrix cores
    # at 92 % zeros; matrix cores for dX and the plane-scanning gather kernel for dW beyond ~97 %.
    # Flags: [whole gather family, dW on the gather kernel, matrix cores].
    p = workloads.config4a(target)
    res, flags = _auto_conv(p)
    assert flags == expect
    _check(p, res)


@pytest.mark.parametrize("target,expect", [(0.92, [0, 0, 1]), (0.999, [1, 0, 0])])
def test_conv_auto_whole_gather_family_with_int8_activations(target, expect):
    # int8 activations: dW stays on the int8 matrix cores at every density the plane-scanning kernel could take, so the gate
    # has its other state -- both products on the kernels that walk the format's entries, beyond ~99.8 % zeros
    p = _problem(64, 256, 14, 14, 256, 3, 3, 1, i8=True)
    p.step = float(np.float32(workloads.step_for_sparsity(p.delta, target)))
    res, flags = _auto_conv(p)
    assert flags == expect
    _check(p, res)


@pytest.mark.parametrize("target,expect", [(0.9, [0, 0, 1]), (0.99, [0, 1, 0])])
@pytest.mark.parametrize("want_dx,stats,two", [(True, True, False), (False, True, False), (True, False, True)])
def test_conv_auto_dw_alone_on_the_gather_kernel(target, expect, want_dx, stats, two):
    # a layer where only the middle state is armed (planes too large for the entry-walking kernels to win): the flags ride
    # in the dX kernel's weight preparation, or, without dX, in a launch of their own; also without a statistics
    # argument (the sum then goes to the workspace) and with the two-plane operands
    import paper_2004_04729_amd as dbp
    p = _problem(16, 128, 56, 56, 128, 3, 3, 1, c=4.0)
    p.step = float(np.float32(workloads.step_for_sparsity(p.delta, target)))
    res, flags = _auto_conv(p, want_dx=want_dx, stats=stats, path=(dbp.PATH_AUTO | dbp.PATH_TWO_PLANES) if two else None)
    # (two planes make the matrix-core dW a third cheaper: on this layer the state is then not worth its launches and the
    # gate is not armed at all)
    assert flags == ([-1, -1, -1] if two else expect)
    if stats:
        assert abs(1 - res["stats"].nnz / p.delta.size - target) < 2e-2
    _check(p, res)                                             # the two-plane bound (1.5e-5) lies inside the tolerance


@pytest.mark.parametrize("target", [0.92, 0.99])
def test_config4a_gather_kernels_full_size_in_full(target):
    # the plane-scanning gather kernels in the launch shape the bench times (256 workgroups of 14 output rows for dX; 256
    # workgroups of 64 planes x 64 channels and a sum over 16 shares of the images for dW): every element against the oracle
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    p = workloads.config4a(target)
    _check(p, run_conv(p, path=dbp.PATH_GATHER))


def test_conv_gather_without_a_workspace_and_products_alone():
    # dbp_conv2d_products with path GATHER: with a workspace the plane-scanning kernels run (prepared weights and partial sums
    # live there); without one dX runs on the kernel that walks the format's entries and dW unsplit; same oracle, same
    # tolerance, int8 X bit-exact
    import torch
    import paper_2004_04729_amd as dbp
    from gpu_util import dev, stream, conv_dims, run_nsd, check_products
    from oracle import oracle as O
    for i8 in (False, True):
        p = _problem(3, 40, 14, 14, 48, 3, 3, 1, c=1.0 if i8 else 4.0, i8=i8)
        N, Cc, H, Wd, K, R, S = conv_dims(p)
        xd = dbp.I8 if i8 else dbp.F32
        q = run_nsd(p.delta.reshape(N * K, -1), N * K, H * Wd, p.step, p.seed)
        k_ref, _ = O.nsd(p.delta, p.step, p.seed)
        assert np.array_equal(q["codes"].reshape(p.delta.shape), k_ref)
        Xf = p.X.astype(np.float32)
        rX, rW, _ = O.conv2d_backward(p.W, Xf, codes=k_ref, step=p.step, stride=1, pad=1)
        aX, aW, _ = O.conv2d_backward(np.abs(p.W), np.abs(Xf), codes=np.abs(k_ref), step=p.step, stride=1, pad=1)
        codes = dev(k_ref)
        for ws in (None, torch.empty(dbp.conv2d_workspace_bytes(N, Cc, H, Wd, K, R, S, 1, 1, xd), dtype=torch.uint8, device="cuda:0")):
            dX = torch.full(p.X.shape, float("nan"), dtype=torch.float32, device="cuda:0")
            dW = torch.full(p.W.shape, -77, dtype=torch.int32, device="cuda:0") if i8 else torch.full(p.W.shape, float("nan"), device="cuda:0")
            dbp.conv2d_products(codes, q["fmt_dev"], p.step, dev(p.W), dev(p.X), xd, N, Cc, H, Wd, K, R, S, 1, 1, dX, dW, ws, dbp.PATH_GATHER, stream())
            torch.cuda.synchronize()
            check_products(dX.cpu().numpy(), rX, aX, "gather dX, workspace %s" % (ws is not None))
            if i8:
                assert np.array_equal(dW.cpu().numpy(), O.conv2d_dw_i8(k_ref, p.X, R, S, 1, 1))
            else:
                check_products(dW.cpu().numpy(), rW, aW, "gather dW, workspace %s" % (ws is not None))


def _random_gather_case(seed):
    """A small random layer the plane-scanning gather kernels can take (3x3 or 1x1, planes a multiple of 4 bytes)."""
    rng = np.random.default_rng(7000 + seed)
    while True:
        R = int(rng.choice([1, 3])); pad = int(rng.integers(0, 3)); st = int(rng.choice([1, 1, 1, 2]))
        H = int(rng.integers(2, 41)); Wd = int(rng.integers(2, 61))
        if H + 2 * pad < R or Wd + 2 * pad < R:
            continue
        P, Q = (H + 2 * pad - R) // st + 1, (Wd + 2 * pad - R) // st + 1
        if (P * Q) % 4 or Q < 2:
            continue
        N = int(rng.integers(1, 5)); C = int(rng.integers(1, 141)); K = int(rng.integers(1, 141))
        return (N, C, H, Wd, K, R, R, pad), st, bool(rng.integers(0, 2)), float(rng.choice([1.0, 4.0, 12.0]))


@pytest.mark.parametrize("seed", range(24))
def test_conv_gather_random_small_layers(seed):
    # shapes nobody picked by hand: ragged channel and plane blocks, bands that end inside the image, rows that straddle dwords
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    case, st, i8, c = _random_gather_case(seed)
    p = _problem(*case, c=1.0 if i8 else c, i8=i8, stride=st, seed=seed)
    _check(p, run_conv(p, path=dbp.PATH_GATHER))


@pytest.mark.parametrize("seed", range(24))
def test_conv_matrix_core_random_small_layers(seed):
    # random kernel sizes, strides, paddings, channel counts and operand types over the matrix-core kernels and their fallbacks,
    # half of them with the two-plane operand split
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    rng = np.random.default_rng(9000 + seed)
    while True:
        R = int(rng.choice([1, 3, 3, 3, 5])); S = int(rng.choice([R, R, 3 if R != 3 else 1]))
        pad = int(rng.integers(0, 3)); st = int(rng.choice([1, 1, 1, 2, 3]))
        H = int(rng.integers(1, 40)); Wd = int(rng.integers(1, 60))
        if H + 2 * pad < R or Wd + 2 * pad < S:
            continue
        N = int(rng.integers(1, 6)); C = int(rng.integers(1, 200)); K = int(rng.integers(1, 200))
        i8 = bool(rng.integers(0, 2)); two = bool(rng.integers(0, 2))
        P, Q = (H + 2 * pad - R) // st + 1, (Wd + 2 * pad - S) // st + 1
        if i8 and N * P * Q * 127 * 127 >= 2 ** 31:
            continue
        break
    p = _problem(N, C, H, Wd, K, R, S, pad, c=1.0 if i8 else 4.0, i8=i8, stride=st, seed=seed)
    _check(p, run_conv(p, path=dbp.PATH_MFMA | (dbp.PATH_TWO_PLANES if two else 0)))
