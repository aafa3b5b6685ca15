"""Host-side walk of the launch plans (no GPU): for a grid of layer shapes, the planning code of the fast kernels must hand
out every work item exactly once, keep every tile / split / class index in range and every partial-sum buffer inside
the workspace size the library reports.  This is the arithmetic a GPU fault would come from."""
import ctypes as C
import itertools

import pytest

import paper_2004_04729_amd as dbp


def _lib():
    L = dbp.lib()
    L.dbp_plan_check_linear.argtypes = [C.c_int64] * 3
    L.dbp_plan_check_conv2d.argtypes = [C.c_int64] * 9
    return L


FC_DIMS = [1, 2, 3, 4, 31, 32, 33, 64, 100, 127, 128, 129, 255, 256, 257, 300, 511, 512, 513, 784, 1000, 1024, 1030, 2048, 4096, 4100, 8192]


def test_fc_plans_cover_every_item_once_and_stay_in_bounds():
    L = _lib()
    bad = []
    for B, in_, out in itertools.product(FC_DIMS, FC_DIMS, FC_DIMS):
        e = L.dbp_plan_check_linear(B, in_, out)
        if e:
            bad.append((B, in_, out, e))
    assert not bad, bad[:10]
    # the configurations and a few very large layers
    for B, in_, out in [(64, 784, 300), (256, 1024, 4096), (256, 4096, 4096), (256, 4096, 1000), (256, 8192, 8192), (300, 4096, 4000),
                        (2048, 2048, 2048), (256, 4096, 16384), (65536, 65536, 8), (8, 65536, 65536), (4096, 16384, 16384)]:
        assert L.dbp_plan_check_linear(B, in_, out) == 0, (B, in_, out)
    assert L.dbp_plan_check_linear(0, 4, 4) == -1


CONV = [  # N, C, H, Wd, K, R, S, stride, pad
    (128, 64, 32, 32, 64, 3, 3, 1, 1), (64, 256, 14, 14, 256, 3, 3, 1, 1), (64, 1024, 14, 14, 256, 1, 1, 1, 0), (32, 256, 56, 56, 256, 3, 3, 1, 1),
    (64, 128, 28, 28, 256, 3, 3, 2, 1), (64, 256, 14, 14, 512, 3, 3, 2, 1), (64, 3, 224, 224, 64, 7, 7, 2, 3), (32, 64, 15, 15, 64, 3, 3, 1, 1),
    (16, 512, 7, 7, 512, 3, 3, 1, 1), (8, 96, 27, 27, 256, 5, 5, 1, 2), (1, 1, 1, 1, 1, 1, 1, 1, 0), (2, 5, 9, 7, 6, 3, 3, 1, 1),
    (64, 132, 24, 20, 264, 1, 1, 2, 0), (1, 8, 17, 17, 8, 3, 3, 4, 1), (2, 16, 9, 224, 8, 3, 3, 1, 1), (1, 16, 20, 228, 16, 3, 3, 1, 1),
]


def test_conv_plans_stay_in_bounds():
    L = _lib()
    for case in CONV:
        assert L.dbp_plan_check_conv2d(*case) == 0, case
    bad = []
    for N, C_, H, K, (R, st, pad) in itertools.product([1, 3, 32, 70], [1, 3, 16, 33, 64, 130, 256], [1, 5, 7, 8, 14, 15, 28, 31, 56],
                                                        [1, 8, 20, 64, 130, 260], [(1, 1, 0), (3, 1, 1), (3, 1, 0), (3, 2, 1), (5, 1, 2), (7, 2, 3), (2, 2, 0), (3, 3, 0)]):
        for Wd in {H, H + 3, 4 * ((H + 3) // 4)}:
            if H + 2 * pad < R or Wd + 2 * pad < R:
                continue
            e = L.dbp_plan_check_conv2d(N, C_, H, Wd, K, R, R, st, pad)
            if e:
                bad.append((N, C_, H, Wd, K, R, st, pad, e))
    assert not bad, bad[:10]
    assert L.dbp_plan_check_conv2d(1, 1, 2, 2, 1, 5, 5, 1, 0) == -1


def test_conv_gather_plans_stay_in_bounds():
    # the gather kernels that scan the code planes: bands, tiles, LDS sizes, the reciprocals that replace divisions
    L = dbp.lib()
    L.dbp_plan_check_conv2d_gather.argtypes = [C.c_int64] * 9 + [C.c_int, C.c_size_t]
    big = 1 << 30
    for case in CONV:
        for i8 in (0, 1):
            for scratch in (0, 1 << 20, big):
                assert L.dbp_plan_check_conv2d_gather(*case, i8, scratch) == 0, (case, i8, scratch)
    bad = []
    for N, C_, H, K, (R, st, pad) in itertools.product([1, 3, 32, 70], [1, 16, 33, 64, 130, 256], [1, 2, 4, 6, 8, 14, 16, 28, 30, 56, 112],
                                                        [1, 8, 33, 64, 130, 260], [(1, 1, 0), (3, 1, 1), (3, 1, 0), (3, 2, 1), (3, 1, 2), (1, 2, 0)]):
        for Wd in {H, H + 2, 4 * ((H + 3) // 4), 200, 252}:
            if H + 2 * pad < R or Wd + 2 * pad < R:
                continue
            for i8 in (0, 1):
                e = L.dbp_plan_check_conv2d_gather(N, C_, H, Wd, K, R, R, st, pad, i8, big)
                if e:
                    bad.append((N, C_, H, Wd, K, R, st, pad, i8, e))
    assert not bad, bad[:10]
    assert L.dbp_plan_check_conv2d_gather(1, 1, 2, 2, 1, 5, 5, 1, 0, 0, 0) == -1


def test_conv_auto_plan_arms_what_the_measurements_say():
    """The host's cost models behind DBP_PATH_AUTO on the layer shapes they were calibrated on (measured on MI355X: where the
    plane-scanning gather kernel for dW beats the matrix cores below 2-4 % nonzeros it is armed, with a threshold in that
    range; where it never does, or the gate's empty launches would cost more than it can win, nothing is armed)."""
    L = _lib()
    L.dbp_plan_auto_conv2d.argtypes = [C.c_int64] * 9 + [C.c_int] * 4 + [C.POINTER(C.c_uint64)] * 2
    L.dbp_plan_auto_conv2d.restype = C.c_int

    def plan(N, C_, H, K, R, pad, i8=0, dx=1, dw=1, two=0, stride=1):
        g, d = C.c_uint64(7), C.c_uint64(7)
        kind = L.dbp_plan_auto_conv2d(N, C_, H, H, K, R, R, stride, pad, i8, dx, dw, two, C.byref(g), C.byref(d))
        codes = N * K * ((H + 2 * pad - R) // stride + 1) ** 2
        return kind, g.value / codes, d.value / codes

    # dW alone on the gather kernel: armed, switching between 1.5 % and 5 % nonzeros (measured crossovers: 3-4 %)
    for shape in [(64, 256, 14, 256), (64, 512, 14, 512), (32, 256, 28, 256), (16, 128, 56, 128), (256, 128, 16, 128)]:
        kind, g, d = plan(*shape, 3, 1)
        assert kind == 2 and g == 0 and 0.015 < d < 0.05, (shape, kind, g, d)
        assert plan(*shape, 3, 1, dx=0)[0] == 2                         # also for a call that asks for dW alone
        assert plan(*shape, 3, 1, dw=0)[0] in (0, 1)                    # and never for one that asks for dX alone
    # too little to win (64-channel layers, config 3's shape among them; 1x1 layers): no gate, or the whole-family one
    for shape, r, pad in [((128, 64, 32, 64), 3, 1), ((32, 64, 56, 64), 3, 1), ((64, 1024, 14, 256), 1, 0), ((32, 512, 28, 128), 1, 0)]:
        kind, g, d = plan(*shape, r, pad)
        assert kind in (0, 1) and d == 0, (shape, kind, d)
    # int8 activations keep dW on the int8 matrix cores: config 5 no gate at all, the 14x14 layer the whole-family gate beyond 99.5 % zeros
    assert plan(32, 256, 56, 256, 3, 1, i8=1)[0] == 0
    kind, g, d = plan(64, 256, 14, 256, 3, 1, i8=1)
    assert kind == 1 and d == 0 and 0 < g < 0.005, (kind, g, d)
    # shapes the kernels decline (stride 2; 5x5) and invalid ones
    assert plan(64, 256, 28, 256, 3, 1, stride=2)[0] in (0, 1) and plan(16, 64, 28, 64, 5, 2)[0] in (0, 1)
    assert L.dbp_plan_auto_conv2d(1, 1, 2, 2, 1, 5, 5, 1, 0, 0, 1, 1, 0, None, None) == -1
    assert L.dbp_plan_auto_conv2d(4, 8, 8, 8, 8, 3, 3, 1, 1, 0, 0, 0, 0, None, None) == -1


def test_fc_auto_plan_arms_the_wide_layer_only():
    """Fully connected layers: the gather family's fixed cost (streaming the dense operand, writing dW) is what the matrix
    cores pay too, so the gate is armed only where a layer is wide enough for the nonzero-proportional part to matter:
    256x4096x16384 (measured: gather wins from ~98.5 % zeros), not the 4096-wide layers of the MLP or 2048^3."""
    L = _lib()
    L.dbp_plan_auto_linear.argtypes = [C.c_int64] * 3 + [C.c_int] * 4 + [C.POINTER(C.c_uint64)]
    L.dbp_plan_auto_linear.restype = C.c_int
    g = C.c_uint64(7)
    assert L.dbp_plan_auto_linear(256, 4096, 16384, 0, 1, 1, 0, C.byref(g)) == 1
    assert 0.005 < g.value / (256 * 16384) < 0.03, g.value
    for B, in_, out in [(256, 4096, 4096), (256, 784, 4096), (256, 4096, 1000), (2048, 2048, 2048), (64, 784, 300)]:
        assert L.dbp_plan_auto_linear(B, in_, out, 0, 1, 1, 0, C.byref(g)) == 0 and g.value == 0, (B, in_, out)
    assert L.dbp_plan_auto_linear(0, 4, 4, 0, 1, 1, 0, None) == -1
