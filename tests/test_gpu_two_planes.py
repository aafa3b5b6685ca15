"""The DBP_PATH_TWO_PLANES flag: the matrix-core kernels cut the fp32 operand into two bf16 planes (rounded to nearest, 16
significant bits) instead of three exact ones.  Checked against the same oracle, to the same 1e-4 tolerance, and to the
flag's own bound: 2^-16 * sum|q||w| for the operand's rounding, on top of the fp32 accumulation error the three-plane
kernels have as well (about 1e-6 of sum|q||w| on these sizes)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

OPERAND = 2.0 ** -16          # |w - hi - lo| <= 2^-16 |w|
ACCUM = 4e-6                  # fp32 accumulation, observed <= 1.5e-6 with three planes on every case below


def _two(path):
    import paper_2004_04729_amd as dbp
    return path | dbp.PATH_TWO_PLANES


def _ratio(got, ref, absref):
    return float((np.abs(np.asarray(got, dtype=np.float64) - ref) / np.maximum(absref, 1e-300)).max())


# shape, and whether the layer runs on the large-layer kernel, which has the two-plane form (None: one product does, or neither)
FC = [(256, 1024, 1000, True), (384, 512, 640, True), (300, 520, 1030, None), (260, 384, 515, None), (37, 301, 129, False)]


@pytest.mark.parametrize("B,in_,out,applies", FC)
def test_fc_two_planes(B, in_, out, applies):
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    from oracle import oracle as O
    from test_gpu_linear import _problem, _check_fp32
    p = _problem(B, in_, out)
    res = run_linear(p, path=_two(dbp.PATH_MFMA))
    assert _check_fp32(p, res) < 1e-4
    k_ref, _ = O.nsd(p.delta, p.step, p.seed)
    rX, rW, _ = O.linear_backward(p.W, p.X, codes=k_ref, step=p.step)
    aX, aW, _ = O.linear_backward(np.abs(p.W), np.abs(p.X), codes=np.abs(k_ref), step=p.step)
    assert _ratio(res["dX"], rX, aX) <= OPERAND + ACCUM and _ratio(res["dW"], rW, aW) <= OPERAND + ACCUM
    three = run_linear(p, path=dbp.PATH_MFMA)
    if applies is True:                             # the flag must have changed the arithmetic
        assert not np.array_equal(three["dX"], res["dX"]) and not np.array_equal(three["dW"], res["dW"])
    elif applies is False:                          # kernels without the form ignore it
        assert np.array_equal(three["dX"], res["dX"]) and np.array_equal(three["dW"], res["dW"])


def test_fc_two_planes_extreme_values_and_separate_calls():
    import paper_2004_04729_amd as dbp
    from gpu_util import run_linear
    from test_gpu_linear import _problem, _check_fp32
    p = _problem(192, 200, 260, c=0.02, x_zero_frac=0)       # dense codes up to +-127
    p.W[::3] *= 1e4
    p.W[1::3] *= 1e-6
    p.W[5, 7] = np.float32(3.38e38)                         # just inside the bf16 range
    p.delta[:, 5] = np.float32(0.9 * p.step) * np.sign(p.delta[:, 5])      # codes 0 and +-1 only, so that its products stay finite
    p.W[6, 9] = np.float32(1e-40)                           # subnormal
    two = run_linear(p, path=_two(dbp.PATH_MFMA))
    _check_fp32(p, two)
    assert not np.array_equal(two["dX"], run_linear(p, path=dbp.PATH_MFMA)["dX"])     # the large-layer kernel: the flag is honoured
    _check_fp32(p, run_linear(p, path=_two(dbp.PATH_MFMA), fused=False, want_dw=False))
    _check_fp32(p, run_linear(p, path=_two(dbp.PATH_MFMA), fused=False, want_dx=False))
    # the gather kernels have no planes, the flag changes nothing there; AUTO accepts it too
    a, b = run_linear(p, path=dbp.PATH_GATHER), run_linear(p, path=_two(dbp.PATH_GATHER))
    assert np.array_equal(a["dX"], b["dX"]) and np.array_equal(a["dW"], b["dW"])
    _check_fp32(p, run_linear(p, path=_two(dbp.PATH_AUTO)))


CONV = [  # N, C, H, Wd, K, R, S, pad, stride
    (2, 5, 9, 7, 6, 3, 3, 1, 1),
    (5, 40, 12, 20, 70, 3, 3, 1, 1),
    (1, 130, 6, 6, 260, 3, 3, 1, 1),
    (2, 64, 30, 30, 40, 3, 3, 1, 1),            # several pixel tiles per image
    (2, 33, 14, 14, 20, 1, 1, 0, 1),            # 1x1: the two-set weight ring; dW on the fully connected kernels
    (3, 140, 14, 14, 260, 1, 1, 0, 1),          # 1x1 with more than 128 output channels: dW straight on the NCHW tensors
    (2, 16, 12, 12, 40, 2, 3, 1, 1),            # six taps
    (2, 8, 10, 10, 9, 3, 3, 0, 1),              # no padding (the other dW instantiation)
    (4, 64, 28, 28, 40, 3, 3, 1, 2),            # stride 2: the classes in one launch
    (2, 3, 11, 8, 4, 5, 3, 2, 1),               # 15 taps
    (17, 70, 8, 8, 130, 3, 3, 1, 1),
]


@pytest.mark.parametrize("case", CONV)
def test_conv_two_planes(case):
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    from oracle import oracle as O
    from test_gpu_conv import _problem, _check
    p = _problem(*case[:8], stride=case[8])
    res = run_conv(p, path=_two(dbp.PATH_MFMA))
    _check(p, res)
    k_ref, _ = O.nsd(p.delta, p.step, p.seed)
    kw = dict(stride=p.stride, pad=p.pad)
    rX, rW, _ = O.conv2d_backward(p.W, p.X, codes=k_ref, step=p.step, **kw)
    aX, aW, _ = O.conv2d_backward(np.abs(p.W), np.abs(p.X), codes=np.abs(k_ref), step=p.step, **kw)
    assert _ratio(res["dX"], rX, aX) <= OPERAND + ACCUM and _ratio(res["dW"], rW, aW) <= OPERAND + ACCUM
    three = run_conv(p, path=dbp.PATH_MFMA)
    assert _ratio(three["dX"], rX, aX) <= ACCUM and _ratio(three["dW"], rW, aW) <= ACCUM
    assert not np.array_equal(three["dX"], res["dX"])        # every case above runs dX on the kernel with prepared weights


def test_conv_two_planes_int8_activations_and_groups():
    import paper_2004_04729_amd as dbp
    from gpu_util import run_conv
    from test_gpu_conv import _problem, _check
    p8 = _problem(3, 24, 17, 44, 40, 3, 3, 1, c=1.0, i8=True)     # int8 X: dW is exact int32 whatever the flag says
    res = run_conv(p8, path=_two(dbp.PATH_MFMA))
    _check(p8, res)
    assert np.array_equal(res["dW"], run_conv(p8, path=dbp.PATH_MFMA)["dW"])
    from test_gpu_grouped import _run
    _run(4, 128, 12, 12, 128, 3, 3, 1, 1, 2, path=_two(dbp.PATH_MFMA))     # 64 channels per group: group by group
    _run(4, 32, 12, 12, 64, 3, 3, 1, 1, 4, path=_two(dbp.PATH_MFMA))       # block-diagonal form
