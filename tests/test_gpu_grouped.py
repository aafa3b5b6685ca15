"""GPU parity of the grouped convolution's backward products against the CPU oracle's grouped convolution: every element,
on every kernel family a group's problem can land on (the fast stride-1 dX kernel, its strided form, the generic
implicit-im2col kernel, the 3x3 dW kernel, the 1x1 dW form, the lowered dW, the int8 dW kernels, the gather kernels)."""
import numpy as np
import pytest
import torch

import paper_2004_04729_amd as dbp
import workloads
from gpu_util import check_products
from oracle import oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(N, C, H, Wd, K, R, S, stride, pad, groups, path, i8=False, seed=0, c=4.0):
    rng = np.random.default_rng(seed + N * 131 + C * 17 + H * 5 + K + groups)
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    Cg = C // groups
    X = workloads.int8_relu_uniform(rng, (N, C, H, Wd)) if i8 else workloads.relu_normal(rng, (N, C, H, Wd))
    W = (rng.standard_normal((K, Cg, R, S)) * np.sqrt(2.0 / (Cg * R * S))).astype(np.float32)
    d = rng.laplace(0, 5e-4, size=(N, K, P, Q)).astype(np.float32)
    step = float(np.float32(c * 7.071e-4))
    xd = dbp.I8 if i8 else dbp.F32
    dd, Wd_, Xd = (torch.from_numpy(a).to(DEV) for a in (d, W, X))
    codes = torch.empty(d.shape, dtype=torch.int8, device=DEV)
    dX = torch.full(X.shape, float("nan"), dtype=torch.float32, device=DEV)
    dW = torch.full(W.shape, -77, dtype=torch.int32, device=DEV) if i8 else torch.full(W.shape, float("nan"), device=DEV)
    ws = torch.empty(dbp.conv2d_grouped_workspace_bytes(N, C, H, Wd, K, R, S, stride, pad, groups, xd), dtype=torch.uint8, device=DEV)
    st = torch.zeros(32, dtype=torch.uint8, device=DEV)
    dbp.dithered_conv2d_backward_grouped(dd, Wd_, Xd, xd, N, C, H, Wd, K, R, S, stride, pad, groups, step, 5, 0, codes, dX, dW, ws, st,
                                         path, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    k_ref, s_ref = O.nsd(d, step, 5)
    assert np.array_equal(codes.cpu().numpy(), k_ref)
    assert dbp.Stats.from_tensor(st).nnz == s_ref.nnz
    Xf = X.astype(np.float32)
    rX, rW = O.conv2d_backward_grouped(W, Xf, groups, codes=k_ref, step=step, stride=stride, pad=pad)
    aX, aW = O.conv2d_backward_grouped(np.abs(W), np.abs(Xf), groups, codes=np.abs(k_ref), step=step, stride=stride, pad=pad)
    name = "grouped n%d c%d %dx%d k%d %dx%d s%d p%d g%d path%d" % (N, C, H, Wd, K, R, S, stride, pad, groups, path)
    check_products(dX.cpu().numpy(), rX, aX, name + " dX")
    if i8:
        want = np.rint(rW / step).astype(np.int64)               # exact integers: sums of code * int8 activation
        assert np.array_equal(dW.cpu().numpy().astype(np.int64), want), name + " dW32"
    else:
        check_products(dW.cpu().numpy(), rW, aW, name + " dW")


CASES = [  # N, C, H, Wd, K, R, S, stride, pad, groups
    (2, 8, 9, 7, 6, 3, 3, 1, 1, 2),             # tiny: generic / fast kernels on ragged tiles
    (3, 64, 14, 14, 96, 3, 3, 1, 1, 2),         # the two-tower AlexNet pattern: fast dX and 3x3 dW kernels per group
    (2, 128, 28, 28, 128, 3, 3, 1, 1, 4),       # ResNeXt-like block, 32 channels per group
    (2, 96, 12, 12, 192, 1, 1, 1, 0, 3),        # 1x1 layer: dW on the fully connected form, images strided by the whole tensor
    (2, 32, 13, 13, 64, 3, 3, 2, 1, 2),         # strided: dX as stride-1 problems per pixel class, dW lowered or generic
    (2, 16, 12, 12, 16, 1, 1, 2, 0, 4),         # 1x1 with stride 2: three of four pixel classes get no tap (dX cleared once)
    (4, 24, 7, 7, 48, 3, 3, 1, 1, 3),           # 7x7 planes: codes copied into padded planes for the dX kernel
    (2, 12, 10, 10, 12, 3, 3, 1, 1, 12),        # depthwise
    (1, 8, 6, 6, 16, 5, 5, 3, 2, 8),            # depthwise with a channel multiplier, stride 3
    (2, 70, 8, 8, 130, 3, 3, 1, 1, 1),          # one group: the ungrouped layer through this entry point
    # 64 and more channels per group: the groups run one after the other on channel blocks of the tensors (fewer: one
    # ungrouped layer with block-diagonal weights)
    (3, 128, 14, 14, 192, 3, 3, 1, 1, 2),       # fast dX kernel and 3x3 dW kernel per group
    (2, 192, 12, 12, 384, 1, 1, 1, 0, 3),       # 1x1: dW on the fully connected form, images strided by the whole tensor
    (2, 128, 13, 13, 128, 3, 3, 2, 1, 2),       # strided: dX per pixel class, dW lowered or generic
    (2, 128, 12, 12, 256, 1, 1, 2, 0, 2),       # 1x1 with stride 2: pixel classes without taps, dX cleared once
    (4, 128, 7, 7, 256, 3, 3, 1, 1, 2),         # 7x7 planes: codes copied into padded planes, planes strided by the whole tensor
    (2, 130, 9, 11, 70, 5, 3, 1, 2, 2),         # odd sizes: generic kernels
]


@pytest.mark.parametrize("case", CASES)
def test_grouped_conv_matrix_core_path_matches_oracle(case):
    _run(*case, path=dbp.PATH_MFMA)


@pytest.mark.parametrize("case", [CASES[0], CASES[1], CASES[4], CASES[7], CASES[10], CASES[12]])
def test_grouped_conv_gather_path_matches_oracle(case):
    _run(*case, path=dbp.PATH_GATHER, c=8.0)


@pytest.mark.parametrize("case", [CASES[1], CASES[2], CASES[3], CASES[4], CASES[7], CASES[10], CASES[11], CASES[12], CASES[14]])
def test_grouped_conv_int8_activations(case):
    _run(*case, path=dbp.PATH_MFMA, i8=True)


def test_auto_is_the_matrix_core_path_and_bad_groups_are_rejected():
    _run(*CASES[1], path=dbp.PATH_AUTO)
    z = torch.zeros(16, device=DEV)
    for groups in (0, -2, 3, 5):                   # 3 and 5 divide neither 8 nor 6 together
        with pytest.raises(dbp.DbpError):
            dbp.dithered_conv2d_backward_grouped(z, z, z, dbp.F32, 2, 8, 9, 7, 6, 3, 3, 1, 1, groups, 0.1, 1, 0, z, z, z, z)
        assert dbp.conv2d_grouped_workspace_bytes(2, 8, 9, 7, 6, 3, 3, 1, 1, groups) == 0
