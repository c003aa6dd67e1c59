"""Seeded synthetic convolution workloads (inputs only, none of the method's arithmetic).

The paper drives its measurements with activation maps produced by ImageNet images inside
trained CNNs (Experiments section); neither is available here, so every layer gets a seeded
synthetic stand-in with the same shapes (SI layer tables), zero fractions (density statistics
of the Introduction and Experiments sections) and structure (i.i.d. or spatially clustered
zeros, all-zero channels).  This module is shared by the CPU oracle's tests, the GPU parity
tests and the benchmark; it imports neither of the two implementations.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20210408


@dataclasses.dataclass(frozen=True)
class LayerSpec:
    """One convolution layer of a workload (batch 1, fp32, one stride; `pad` rows above and below
    and as many columns left and right, unless `pad_w` gives the columns their own padding)."""

    name: str
    config: int          # workload number, 1..5
    layer: int           # index of the layer inside the workload
    C: int
    H: int
    W: int
    K: int
    kh: int
    kw: int
    stride: int
    pad: int
    kind: str            # "relu_gauss" | "clustered" | "bernoulli_halfnormal" | "dense"
    zero_frac: float     # targeted fraction of zeros among live channels
    zero_channels: int   # number of channels forced to all-zero
    pad_w: Optional[int] = None

    @property
    def Ih(self) -> int:
        return self.H + 2 * self.pad

    @property
    def Iw(self) -> int:
        return self.W + 2 * (self.pad if self.pad_w is None else self.pad_w)

    @property
    def Oh(self) -> int:
        return (self.Ih - self.kh) // self.stride + 1

    @property
    def Ow(self) -> int:
        return (self.Iw - self.kw) // self.stride + 1

    @property
    def shape_tuple(self) -> Tuple[int, ...]:
        base = (self.C, self.H, self.W, self.K, self.kh, self.kw, self.stride, self.pad)
        return base if self.pad_w is None else base + (self.pad_w,)

    @property
    def s_im2col(self) -> int:
        """Element count of the im2col lowered matrix (SI, space complexity of im2col)."""
        return self.C * self.kh * self.kw * self.Oh * self.Ow

    @property
    def dense_flops(self) -> int:
        return 2 * self.K * self.s_im2col


def _norm_ppf(p: float) -> float:
    """Inverse standard-normal CDF by bisection on erf (avoids a scipy dependency here)."""
    lo, hi = -10.0, 10.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if 0.5 * (1.0 + math.erf(mid / math.sqrt(2.0))) < p:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _cfg5_layers() -> List[LayerSpec]:
    out: List[LayerSpec] = []
    out.append(LayerSpec("cfg5.stem7x7s2", 5, 0, 3, 224, 224, 64, 7, 7, 2, 3, "dense", 0.0, 0))
    body = (
        [(64, 56, 1)] * 3
        + [(128, 56, 2)] + [(128, 28, 1)] * 3
        + [(256, 28, 2)] + [(256, 14, 1)] * 5
        + [(512, 14, 2)] + [(512, 7, 1)] * 2
    )
    for i, (ch, hw, s) in enumerate(body, start=1):
        z = 0.40 + 0.45 * (i - 1) / 15.0
        out.append(
            LayerSpec(f"cfg5.l{i:02d}.{ch}@{hw}s{s}", 5, i, ch, hw, hw, ch, 3, 3, s, 1,
                      "relu_gauss", z, int(0.05 * ch))
        )
    return out


def layers(config: int) -> List[LayerSpec]:
    """The layers of one of the five workloads (7: the supplementary 1 x n / n x 1 layers)."""
    if config == 1:
        return [LayerSpec("cfg1.16@28", 1, 0, 16, 28, 28, 16, 3, 3, 1, 1, "relu_gauss", 0.5, 2)]
    if config == 2:
        return [LayerSpec("cfg2.128@56", 2, 0, 128, 56, 56, 128, 3, 3, 1, 1, "relu_gauss", 0.6, 0)]
    if config == 3:
        return [LayerSpec("cfg3.256@14", 3, 0, 256, 14, 14, 256, 3, 3, 1, 1, "clustered", 0.7, 25)]
    if config == 4:
        return [
            LayerSpec("cfg4a.5x5.64@27", 4, 0, 64, 27, 27, 192, 5, 5, 1, 2,
                      "bernoulli_halfnormal", 0.5, 0),
            LayerSpec("cfg4b.3x3s2.128@56", 4, 1, 128, 56, 56, 256, 3, 3, 2, 1, "clustered", 0.65, 0),
        ]
    if config == 5:
        return _cfg5_layers()
    if config == 7:
        return line_layers()
    raise ValueError(f"unknown workload {config}")


def all_layers() -> List[LayerSpec]:
    return [spec for cfg in (1, 2, 3, 4, 5) for spec in layers(cfg)]


def line_layers() -> List[LayerSpec]:
    """Layers with 1 x n and n x 1 kernels, shaped like those of the SI's layer tables (17 x 17
    maps with 128 to 192 channels under 1 x 7 / 7 x 1 kernels, 8 x 8 maps with 384 channels under
    1 x 3 / 3 x 1), padded in the kernel's direction only so that the map keeps its size.  A
    supplement to the five workloads (number 7): ReLU-Gaussian inputs, 60 to 80 % zeros."""
    rows = [
        ("1x7.128to128@17", 128, 17, 128, 1, 7, 0.60), ("7x1.128to192@17", 128, 17, 192, 7, 1, 0.60),
        ("1x7.160to160@17", 160, 17, 160, 1, 7, 0.65), ("7x1.160to192@17", 160, 17, 192, 7, 1, 0.65),
        ("1x7.192to192@17", 192, 17, 192, 1, 7, 0.70), ("7x1.192to192@17", 192, 17, 192, 7, 1, 0.70),
        ("1x3.384to384@8", 384, 8, 384, 1, 3, 0.80), ("3x1.384to384@8", 384, 8, 384, 3, 1, 0.80),
    ]
    return [LayerSpec("line." + name, 7, i, C, hw, hw, K, kh, kw, 1, kh // 2, "relu_gauss", z, int(0.05 * C),
                      pad_w=kw // 2) for i, (name, C, hw, K, kh, kw, z) in enumerate(rows)]


def layer_seed(spec: LayerSpec, m: int = 0) -> int:
    return BASE_SEED + 100 * spec.config + spec.layer + 1000003 * m


def _clustered_channel(rng: np.random.Generator, H: int, W: int, zero_frac: float) -> np.ndarray:
    from scipy.ndimage import gaussian_filter

    g = gaussian_filter(rng.standard_normal((H, W)), sigma=2.0, mode="reflect")
    tau = np.quantile(g, zero_frac)
    a = np.maximum(g - tau, 0.0)
    sd = a.std()
    return a / sd if sd > 0 else a


def make_activation(spec: LayerSpec, m: int = 0) -> np.ndarray:
    """Activation map C x H x W, fp32, C-contiguous."""
    rng = np.random.default_rng(layer_seed(spec, m))
    C, H, W = spec.C, spec.H, spec.W
    if spec.kind == "dense":
        act = rng.standard_normal((C, H, W))
    elif spec.kind == "relu_gauss":
        mu = _norm_ppf(1.0 - spec.zero_frac)
        act = np.maximum(rng.standard_normal((C, H, W)) + mu, 0.0)
    elif spec.kind == "bernoulli_halfnormal":
        keep = rng.random((C, H, W)) >= spec.zero_frac
        act = keep * np.abs(rng.standard_normal((C, H, W)))
    elif spec.kind == "clustered":
        act = np.stack([_clustered_channel(rng, H, W, spec.zero_frac) for _ in range(C)])
    else:
        raise ValueError(spec.kind)
    if spec.zero_channels:
        dead = rng.choice(C, size=spec.zero_channels, replace=False)
        act[dead] = 0.0
    return np.ascontiguousarray(act, dtype=np.float32)


def make_weights(spec: LayerSpec) -> np.ndarray:
    """He-normal weights K x C x kh x kw, fp32."""
    rng = np.random.default_rng(layer_seed(spec) + 7919)
    sigma = math.sqrt(2.0 / (spec.C * spec.kh * spec.kw))
    w = rng.standard_normal((spec.K, spec.C, spec.kh, spec.kw)) * sigma
    return np.ascontiguousarray(w, dtype=np.float32)


def make_layer(spec: LayerSpec, m: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    return make_activation(spec, m), make_weights(spec)


def random_case(seed: int, C: int, H: int, W: int, K: int, kh: int, kw: int, stride: int,
                pad: int, zero_frac: float, zero_channels: int = 0, integer: bool = False,
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Small ad-hoc case for edge-case tests.  ``integer=True`` draws small integers so that
    fp32 sums are exact whatever the order of additions."""
    rng = np.random.default_rng(seed)
    keep = rng.random((C, H, W)) >= zero_frac
    if integer:
        vals = rng.integers(1, 8, size=(C, H, W)).astype(np.float64)
        vals *= rng.choice([-1.0, 1.0], size=(C, H, W))
        w = rng.integers(-4, 5, size=(K, C, kh, kw)).astype(np.float64)
    else:
        vals = rng.standard_normal((C, H, W))
        vals[vals == 0.0] = 1.0
        w = rng.standard_normal((K, C, kh, kw)) * math.sqrt(2.0 / (C * kh * kw))
    act = keep * vals
    if zero_channels:
        dead = rng.choice(C, size=min(zero_channels, C), replace=False)
        act[dead] = 0.0
    return (np.ascontiguousarray(act, dtype=np.float32), np.ascontiguousarray(w, dtype=np.float32))


# --- a chained network: the 3x3 layers of workload 5 joined end to end -------------------------
def chain_specs() -> List[LayerSpec]:
    """Workload 5's sixteen 3x3 layers as ONE network: every layer takes the output of the layer
    before it, so the strided layers read the narrower map (64 -> 128, 128 -> 256, 256 -> 512
    channels, as in the residual networks of the SI layer tables).  ``zero_frac`` is the zero
    fraction the bias in front of the layer aims at; ``zero_channels`` channels get a bias that
    switches them off."""
    out: List[LayerSpec] = []
    prev_k, hw = 64, 56
    for spec in _cfg5_layers()[1:]:
        out.append(LayerSpec(f"chain.l{spec.layer:02d}.{prev_k}to{spec.K}@{hw}s{spec.stride}", 6, spec.layer,
                             prev_k, hw, hw, spec.K, 3, 3, spec.stride, 1, "relu_gauss", spec.zero_frac,
                             int(0.05 * prev_k)))
        prev_k, hw = spec.K, out[-1].Oh
    return out


def _relu_gauss_second_moment(mean: float, sd: float) -> float:
    """E[max(0, X)^2] for X ~ N(mean, sd^2)."""
    t = mean / sd
    cdf = 0.5 * (1.0 + math.erf(t / math.sqrt(2.0)))
    pdf = math.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)
    return (mean * mean + sd * sd) * cdf + mean * sd * pdf


def make_chain(m: int = 0):
    """Input map of the first layer, the weights of every layer and the bias in front of every
    layer but the first.  With He-normal weights a layer's output is close to N(0, 2 E[a^2]) for
    an input a (less what dead channels and padding take away), so the bias that leaves a fraction z of zeros after the ReLU is sd * ppf(1 - z);
    it gets a 10 % per-channel jitter, and ``zero_channels`` channels are pushed 8 sd below zero."""
    specs = chain_specs()
    first = specs[0]
    act = make_activation(dataclasses.replace(first, zero_channels=0), m)
    weights, biases = [], []
    mean, sd = _norm_ppf(1.0 - first.zero_frac), 1.0
    for i, spec in enumerate(specs):
        rng = np.random.default_rng(layer_seed(spec) + 104729)
        if i == 0:
            biases.append(None)
        else:
            # spread of the previous layer's output: its live input channels, the taps that fall on
            # the map rather than on the padding, the jitter of the bias in front of it
            prev = specs[i - 1]
            live = 1.0 - (prev.zero_channels if i > 1 else 0) / prev.C
            on_map = ((3.0 * prev.H - 2.0) / (3.0 * prev.H)) ** 2 if prev.stride == 1 else 1.0
            jitter = 1.01 if i > 1 else 1.0
            sd = math.sqrt(2.0 * live * on_map * _relu_gauss_second_moment(mean, sd * math.sqrt(jitter)))
            mean = sd * _norm_ppf(1.0 - spec.zero_frac)
            b = mean + 0.1 * sd * rng.standard_normal(spec.C)
            dead = rng.choice(spec.C, size=spec.zero_channels, replace=False)
            b[dead] = -8.0 * sd
            biases.append(np.ascontiguousarray(b, dtype=np.float32))
        weights.append(make_weights(spec))
    return act, weights, biases
