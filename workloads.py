"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the CPU oracle's tests and the HIP path's tests/benchmark.  It
holds none of the method's arithmetic (no dither, no quantiser, no products): it only
draws tensors and picks the step size Delta that is handed to either side as an input.

The paper trains LeNet/AlexNet/VGG11/ResNet18 on MNIST/CIFAR/ImageNet (Sec. "Experiments");
none of those datasets or weights is available here, so every tensor is synthetic and
stands in for them: layer shapes and batch sizes follow the paper's models, the
preactivation gradient follows a Laplace (or heavy-tailed Laplace mixture) law, inputs
are ReLU outputs.  Data seed = 1000 + config number (+ layer number); dither seed = 1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

DITHER_SEED = 1


# --------------------------------------------------------------------------- step size
def step_from_std(delta: np.ndarray, c: float) -> float:
    """Delta = c * std(delta) (Algorithm 1, steps 2-3): population std about the mean, in fp64."""
    return float(np.float32(c * np.std(delta.astype(np.float64))))


def expected_sparsity(delta: np.ndarray, step: float) -> float:
    """Exact expectation over the dither of the fraction of zero codes: mean max(0, 1-|x|/Delta)."""
    a = np.abs(delta.astype(np.float64)) / float(step)
    return float(np.mean(np.maximum(0.0, 1.0 - a)))


def step_for_sparsity(delta: np.ndarray, target: float) -> float:
    """Bisect Delta so that expected_sparsity(delta, Delta) == target (monotone in Delta)."""
    sample = delta.ravel()
    if sample.size > (1 << 22):
        sample = sample[:: sample.size // (1 << 22)]
    lo, hi = 1e-12, float(np.max(np.abs(sample))) * 1e4 + 1e-6
    for _ in range(100):
        mid = np.sqrt(lo * hi)
        if expected_sparsity(sample, mid) < target:
            lo = mid
        else:
            hi = mid
    return float(np.float32(np.sqrt(lo * hi)))


# --------------------------------------------------------------------------- draws
def laplace(rng, b, shape):
    return rng.laplace(0.0, b, size=shape).astype(np.float32)


def laplace_mixture(rng, shape, b_small=1e-4, b_large=1e-2, frac_large=0.05):
    small = rng.laplace(0.0, b_small, size=shape)
    large = rng.laplace(0.0, b_large, size=shape)
    pick = rng.random(size=shape) < frac_large
    return np.where(pick, large, small).astype(np.float32)


def relu_normal(rng, shape):
    return np.maximum(rng.standard_normal(size=shape), 0.0).astype(np.float32)


def int8_relu_uniform(rng, shape):
    """Uniform on [-127,127] clipped at 0 from below: about half zeros, int8."""
    return np.maximum(rng.integers(-127, 128, size=shape), 0).astype(np.int8)


# --------------------------------------------------------------------------- problems
@dataclass
class LinearProblem:
    name: str
    delta: np.ndarray          # [B, out] fp32
    W: np.ndarray              # [out, in] fp32
    X: np.ndarray              # [B, in] fp32 or int8
    step: float
    seed: int = DITHER_SEED
    predicted_sparsity: Optional[float] = None

    @property
    def dims(self):
        return self.X.shape[0], self.W.shape[1], self.W.shape[0]   # B, in, out


@dataclass
class ConvProblem:
    name: str
    delta: np.ndarray          # [N, K, P, Q] fp32
    W: np.ndarray              # [K, C, R, S] fp32
    X: np.ndarray              # [N, C, H, W] fp32 or int8
    step: float
    stride: int = 1
    pad: int = 1
    seed: int = DITHER_SEED
    predicted_sparsity: Optional[float] = None


def config1(c: float = 4.0) -> LinearProblem:
    """Single FC layer (LeNet-300-100's first layer shape): batch 64, 784 -> 300."""
    rng = np.random.default_rng(1001)
    X = rng.standard_normal((64, 784)).astype(np.float32)
    W = (0.05 * rng.standard_normal((300, 784))).astype(np.float32)
    d = laplace(rng, 1e-3, (64, 300))
    step = step_from_std(d, c)
    return LinearProblem("cfg1_fc_64x784x300_c%g" % c, d, W, X, step, predicted_sparsity=expected_sparsity(d, step))


MLP_WIDTHS = (1024, 4096, 4096, 1000)


def config2(c: float = 8.0, batch: int = 256, widths=MLP_WIDTHS) -> list:
    """Three-layer MLP backward chain, returned in backward order (last layer first)."""
    layers = []
    nl = len(widths) - 1
    for l in range(nl, 0, -1):
        rng = np.random.default_rng(1002 + 10 * l)
        fan_in, fan_out = widths[l - 1], widths[l]
        X = relu_normal(rng, (batch, fan_in))
        W = (rng.standard_normal((fan_out, fan_in)) / np.sqrt(fan_in)).astype(np.float32)
        b = 10.0 ** rng.uniform(-4.0, -2.0)
        d = laplace(rng, b, (batch, fan_out))
        step = step_from_std(d, c)
        layers.append(LinearProblem("cfg2_L%d_%dx%dx%d_c%g" % (l, batch, fan_in, fan_out, c), d, W, X, step,
                                    predicted_sparsity=expected_sparsity(d, step)))
    return layers


def _conv(name, seed, N, C, K, H, R, pad, delta_fn, x_fn, w_std, step_fn, stride=1):
    rng = np.random.default_rng(seed)
    P = (H + 2 * pad - R) // stride + 1
    X = x_fn(rng, (N, C, H, H))
    W = (w_std * rng.standard_normal((K, C, R, R))).astype(np.float32)
    d = delta_fn(rng, (N, K, P, P))
    step = step_fn(d)
    return ConvProblem(name, d, W, X, step, stride, pad, predicted_sparsity=expected_sparsity(d, step))


def config3(c: float = 4.0, N: int = 128) -> ConvProblem:
    """CIFAR-shaped 3x3 conv, 64 -> 64 channels, 32x32."""
    return _conv("cfg3_conv3x3_n%d_64x64_32x32_c%g" % (N, c), 1003, N, 64, 64, 32, 3, 1,
                 lambda r, s: laplace(r, 5e-4, s), relu_normal, np.sqrt(2.0 / 576.0),
                 lambda d: step_from_std(d, c))


def resnet_downsample(target: float = 0.92, N: int = 64) -> ConvProblem:
    """The strided 3x3 convolution that opens a ResNet-18 stage: 128 -> 256 channels, 28x28 -> 14x14, stride 2."""
    return _conv("resnet_conv3x3s2_n%d_128x256_28x28_s%g" % (N, target), 1006, N, 128, 256, 28, 3, 1,
                 laplace_mixture, relu_normal, np.sqrt(2.0 / 1152.0), lambda d: step_for_sparsity(d, target), stride=2)


def config4a(target: float = 0.92, N: int = 64) -> ConvProblem:
    """ImageNet ResNet-stage 3x3 conv, 256 -> 256 channels, 14x14, heavy-tailed gradient."""
    return _conv("cfg4a_conv3x3_n%d_256x256_14x14_s%g" % (N, target), 1004, N, 256, 256, 14, 3, 1,
                 laplace_mixture, relu_normal, np.sqrt(2.0 / 2304.0), lambda d: step_for_sparsity(d, target))


def config4b(target: float = 0.92, N: int = 64) -> ConvProblem:
    """1x1 conv, 1024 -> 256 channels, 14x14, same gradient law."""
    return _conv("cfg4b_conv1x1_n%d_1024x256_14x14_s%g" % (N, target), 1014, N, 1024, 256, 14, 1, 0,
                 laplace_mixture, relu_normal, np.sqrt(2.0 / 1024.0), lambda d: step_for_sparsity(d, target))


def config5(target: float = 0.90, N: int = 32, C: int = 256, H: int = 56) -> ConvProblem:
    """8-bit mode, VGG-16 conv3-shaped layer: int8 X, fp32 W, int32 dW."""
    return _conv("cfg5_conv3x3_i8_n%d_%dx%d_%dx%d_s%g" % (N, C, C, H, H, target), 1005, N, C, C, H, 3, 1,
                 lambda r, s: laplace(r, 1e-3, s), int8_relu_uniform, 0.02, lambda d: step_for_sparsity(d, target))


def structured_planes(delta: np.ndarray, frac_dead: float = 0.5, seed: int = 77) -> np.ndarray:
    """Zero a fraction of (n, k) planes (or rows) entirely: mimics dead ReLU channels."""
    rng = np.random.default_rng(seed)
    d = delta.copy()
    lead = d.shape[:2] if d.ndim == 4 else d.shape[:1]
    dead = rng.random(size=lead) < frac_dead
    d[dead] = 0.0
    return d
