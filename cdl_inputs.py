"""Seeded synthetic inputs for the CDL quantized-layer step.

This module only draws random tensors and names the five workloads; it holds
none of the method's arithmetic, so both the CPU oracle's tests and the HIP
path's tests/benchmark can take their inputs from it without sharing code.

The workloads stand in for the CNN / transformer layers the paper trains
(Section V: ResNet-18/34 on ImageNet, ResNet-20..110 on CIFAR-100): same
tensor shapes and value distributions, random values.  Step sizes follow the
paper's initialisation rule (Section V-B, "Common hyper-parameters"):
step = 2 * mean|tensor| / sqrt(2^(b-1)), evaluated in closed form for the
stated distribution.  Sharpness defaults to kappa = alpha * step^2 = 4, the
middle of the range the paper plots in Figs. 1-2 (alpha*q^2 in {1, 3, 5, 7});
`alpha_paper` is the paper's literal initial value 500.

Every tensor comes from its own numpy Generator seeded with
(seed, workload number, tensor number), so one tensor can be drawn without
drawing the others.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

_SQRT_2_OVER_PI = math.sqrt(2.0 / math.pi)  # mean |N(0,1)|

ALPHA_PAPER = 500.0  # Section V-B: alpha^0 = beta^0 = 500


@dataclass(frozen=True)
class QuantSpec:
    """Level set {lo, ..., lo + n_levels - 1}, step size and sharpness."""
    lo: int
    n_levels: int
    delta: float
    alpha: float

    @property
    def hi(self) -> int:
        return self.lo + self.n_levels - 1

    def with_alpha(self, alpha: float) -> "QuantSpec":
        return QuantSpec(self.lo, self.n_levels, self.delta, float(np.float32(alpha)))

    def with_kappa(self, kappa: float) -> "QuantSpec":
        return self.with_alpha(kappa / (self.delta * self.delta))


def _f32(x: float) -> float:
    """Round a Python float to the nearest fp32 so every consumer sees one value."""
    return float(np.float32(x))


def _spec(lo: int, n_levels: int, delta: float, kappa: float = 4.0) -> QuantSpec:
    d = _f32(delta)
    return QuantSpec(lo, n_levels, d, _f32(kappa / (d * d)))


@dataclass(frozen=True)
class Workload:
    """One layer-shaped problem: Y[M,N] = X[M,K] . W[N,K]^T over quantized operands."""
    number: int                 # 1-based, as in the list of five
    name: str
    M: int
    N: int
    K: int
    w_sigma: float
    x_kind: str                 # "halfnormal" | "normal_outliers" | "none"
    w_spec: QuantSpec
    x_spec: Optional[QuantSpec]
    flat_n: int = 0             # > 0: a single flat weight tensor, no GEMM
    note: str = ""

    @property
    def has_gemm(self) -> bool:
        return self.flat_n == 0

    @property
    def w_shape(self) -> Tuple[int, ...]:
        return (self.flat_n,) if self.flat_n else (self.N, self.K)

    @property
    def x_shape(self) -> Tuple[int, ...]:
        return (self.M, self.K)

    @property
    def g_shape(self) -> Tuple[int, ...]:
        return (self.flat_n,) if self.flat_n else (self.M, self.N)


def _init_step(mean_abs: float, bits: int) -> float:
    return 2.0 * mean_abs / math.sqrt(2.0 ** (bits - 1))


def _make_workloads():
    wl = {}
    # 1: tiny quantized linear (all values given explicitly)
    wl[1] = Workload(1, "tiny_linear", M=32, N=128, K=256, w_sigma=0.05, x_kind="halfnormal",
                     w_spec=_spec(-7, 15, 0.02), x_spec=_spec(0, 16, 0.25),
                     note="oracle finishes in well under a second")
    # 2: CIFAR ResNet-20-shaped 3x3 conv 16->16 at 32x32, batch 128, as an im2col GEMM
    s2 = math.sqrt(2.0 / 144.0)
    wl[2] = Workload(2, "resnet20_conv_im2col", M=131072, N=16, K=144, w_sigma=s2, x_kind="halfnormal",
                     w_spec=_spec(-7, 15, _init_step(s2 * _SQRT_2_OVER_PI, 4)),
                     x_spec=_spec(0, 16, _init_step(_SQRT_2_OVER_PI, 4)))
    # 3: ImageNet ResNet-18 layer3-shaped 3x3 conv 256->256 at 14x14, batch 256
    s3 = math.sqrt(2.0 / 2304.0)
    wl[3] = Workload(3, "resnet18_layer3_conv", M=50176, N=256, K=2304, w_sigma=s3, x_kind="halfnormal",
                     w_spec=_spec(-7, 15, _init_step(s3 * _SQRT_2_OVER_PI, 4)),
                     x_spec=_spec(0, 16, _init_step(_SQRT_2_OVER_PI, 4)))
    # 4: quantizer-only bandwidth test, one flat ResNet-50-sized weight tensor
    wl[4] = Workload(4, "flat_weights_25M", M=0, N=0, K=0, w_sigma=0.02, x_kind="none",
                     w_spec=_spec(-15, 31, 0.004), x_spec=None, flat_n=25_600_000)
    # 5: transformer MLP-shaped linear, 8-bit, 1% outliers x8 in the activations
    mean_abs_x5 = 0.99 * _SQRT_2_OVER_PI + 0.01 * 8.0 * _SQRT_2_OVER_PI
    wl[5] = Workload(5, "transformer_mlp", M=65536, N=3072, K=768, w_sigma=0.02, x_kind="normal_outliers",
                     w_spec=_spec(-127, 255, _init_step(0.02 * _SQRT_2_OVER_PI, 8)),
                     x_spec=_spec(-127, 255, _init_step(mean_abs_x5, 8)))
    return wl


WORKLOADS = _make_workloads()


def workload(number: int) -> Workload:
    return WORKLOADS[number]


def _rng(seed: int, number: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([seed, number, tensor])


def _normal(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    out = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    return out


def draw_w(wl: Workload, seed: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """Weight tensor [N,K] (or flat [n] for the flat workload), fp32, ~N(0, w_sigma^2).

    `rows` keeps only the first `rows` rows (flat: elements) of the same stream.
    """
    shape = list(wl.w_shape)
    if rows is not None:
        shape[0] = min(rows, shape[0])
    return _normal(_rng(seed, wl.number, 0), tuple(shape), wl.w_sigma)


def draw_x(wl: Workload, seed: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """Activation tensor [M,K], fp32: |N(0,1)| (post-ReLU-like) or N(0,1) with 1% of entries x8."""
    if wl.x_kind == "none":
        raise ValueError("workload %d has no activation tensor" % wl.number)
    shape = list(wl.x_shape)
    if rows is not None:
        shape[0] = min(rows, shape[0])
    rng = _rng(seed, wl.number, 1)
    x = rng.standard_normal(tuple(shape), dtype=np.float32)
    if wl.x_kind == "halfnormal":
        np.abs(x, out=x)
    elif wl.x_kind == "normal_outliers":
        # each entry independently, with probability 0.01, multiplied by 8
        mask = _rng(seed, wl.number, 3).random(tuple(shape), dtype=np.float32) < np.float32(0.01)
        x[mask] *= np.float32(8.0)
    return x


def draw_g(wl: Workload, seed: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """Upstream gradient [M,N] (flat workload: [n]), fp32, ~N(0,1)."""
    shape = list(wl.g_shape)
    if rows is not None:
        shape[0] = min(rows, shape[0])
    return _normal(_rng(seed, wl.number, 2), tuple(shape), 1.0)


def draw_tensor(n: int, kind: str, sigma: float = 1.0, seed: int = 0, stream: int = 100) -> np.ndarray:
    """A free-standing flat fp32 tensor for parity sweeps: 'normal', 'halfnormal' or 'uniform' in [-sigma, sigma]."""
    rng = np.random.default_rng([seed, 0, stream])
    if kind == "uniform":
        return ((rng.random(n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)) * np.float32(sigma))
    x = rng.standard_normal(n, dtype=np.float32)
    if kind == "halfnormal":
        np.abs(x, out=x)
    elif kind != "normal":
        raise ValueError(kind)
    x *= np.float32(sigma)
    return x


def draw_indices(shape, lo: int, hi: int, seed: int = 0, stream: int = 200) -> np.ndarray:
    """Uniform random int8 level indices in [lo, hi] for GEMM-only tests."""
    rng = np.random.default_rng([seed, 0, stream])
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)
