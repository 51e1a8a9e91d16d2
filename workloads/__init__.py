"""Seeded synthetic inputs shaped like the paper's ViT and ResNet layers.

This module serves both the CPU oracle's tests and the HIP library's tests and benchmark.  It
holds none of the method's arithmetic: it only draws fp32 tensors (activations, a separate
calibration draw, weights) and lists layer shapes.  Quantisation, channel ordering, extraction
positions and the products themselves are computed independently by each side.

Stand-in statement: the paper measures on ImageNet/CIFAR images through pretrained ViT and ResNet
models (Section 8).  Neither datasets nor checkpoints are used here; the tensors below reproduce
the layer shapes and the property the method exploits -- input channels whose value ranges differ
by orders of magnitude, with a few outlier channels.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 251002822
CAL_ROWS = 256          # calibration sample count used in the paper's Table 1 is 128-256


def _rng(config: int, layer: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + layer + stream))


@dataclass
class LinearCase:
    name: str
    M: int
    K: int
    N: int
    group_size: int
    ratios: Tuple[float, ...]
    X: np.ndarray        # fp32 [M][K]
    Xcal: np.ndarray     # fp32 [CAL_ROWS][K], independent draw from the same channel scales
    W: np.ndarray        # fp32 [N][K]
    bias: np.ndarray     # fp32 [N]


@dataclass
class ConvCase:
    name: str
    B: int
    H: int
    Wd: int
    C: int
    N: int
    R: int
    S: int
    stride: int
    pad: int
    group_size: int
    ratios: Tuple[float, ...]
    X: np.ndarray        # fp32 NHWC [B][H][Wd][C]
    Xcal: np.ndarray     # fp32 [CAL_ROWS][C]
    W: np.ndarray        # fp32 [N][R][S][C]
    bias: np.ndarray     # fp32 [N]

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.Wd + 2 * self.pad - self.S) // self.stride + 1


def _channel_scales(rng, K: int, outlier_frac: float) -> np.ndarray:
    s = rng.lognormal(0.0, 1.0, size=K).astype(np.float32)
    if outlier_frac > 0:
        n_out = max(1, int(round(outlier_frac * K)))
        idx = rng.choice(K, size=n_out, replace=False)
        s[idx] *= 20.0
    return s


def make_linear(name: str, config: int, layer: int, M: int, K: int, N: int, group_size: int,
                ratios=(0.0, 0.25, 0.5, 0.75, 1.0), outlier_frac: float = 0.0, relu: bool = False) -> LinearCase:
    """X[m,k] ~ N(0, s_k^2) with s_k ~ LogNormal(0,1) (optionally 2% of channels at 20x scale);
    W ~ N(0, 0.02^2); bias ~ N(0, 0.1^2).  Draw order: scales, X, W, bias; calibration rows come
    from a second generator (seed + 500) so that the test rows can exceed the calibrated range."""
    rng = _rng(config, layer)
    s = _channel_scales(rng, K, outlier_frac)
    X = rng.standard_normal((M, K), dtype=np.float32) * s[None, :]
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    bias = rng.standard_normal(N, dtype=np.float32) * np.float32(0.1)
    Xcal = _rng(config, layer, 500).standard_normal((CAL_ROWS, K), dtype=np.float32) * s[None, :]
    if relu:
        X = np.abs(X)
        Xcal = np.abs(Xcal)
    return LinearCase(name, M, K, N, group_size, tuple(ratios), X, Xcal, W, bias)


def make_conv(name: str, config: int, layer: int, B: int, H: int, Wd: int, C: int, N: int, R: int, S: int,
              stride: int, pad: int, group_size: int, ratios=(0.0, 0.5, 1.0)) -> ConvCase:
    """Post-ReLU activations |N(0, s_c^2)|, s_c ~ LogNormal(0,1); weights N(0, 0.02^2)."""
    rng = _rng(config, layer)
    s = _channel_scales(rng, C, 0.0)
    X = np.abs(rng.standard_normal((B, H, Wd, C), dtype=np.float32)) * s
    W = rng.standard_normal((N, R, S, C), dtype=np.float32) * np.float32(0.02)
    bias = rng.standard_normal(N, dtype=np.float32) * np.float32(0.1)
    Xcal = np.abs(_rng(config, layer, 500).standard_normal((CAL_ROWS, C), dtype=np.float32)) * s
    return ConvCase(name, B, H, Wd, C, N, R, S, stride, pad, group_size, tuple(ratios), X, Xcal, W, bias)


# ---- the benchmark configurations -----------------------------------------------------------------

def config0() -> LinearCase:
    """Oracle-sized single linear layer: M=64, K=256, N=256, group size 32."""
    return make_linear("cfg0_linear", 0, 0, 64, 256, 256, 32)


def config1(which: str, M: int = 32 * 197) -> LinearCase:
    """ViT-B/16 MLP linears, batch 32 at 224 px (M = 32*197): fc1 768->3072, fc2 3072->768."""
    if which == "fc1":
        return make_linear("vitb_fc1", 1, 0, M, 768, 3072, 32, outlier_frac=0.02)
    return make_linear("vitb_fc2", 1, 1, M, 3072, 768, 32, outlier_frac=0.02)


def config2(B: int = 64) -> ConvCase:
    """ResNet-50-style 3x3 conv: NHWC [64,14,14,256] -> 256 channels, stride 1, pad 1."""
    return make_conv("resnet_3x3_256", 2, 0, B, 14, 14, 256, 256, 3, 3, 1, 1, 32)


def config3(which: str, M: int = 64 * 197) -> LinearCase:
    """ViT-L/16 MLP linears, batch 64 at 224 px (M = 64*197), group size 64."""
    if which == "fc1":
        return make_linear("vitl_fc1", 3, 0, M, 1024, 4096, 64, ratios=(0.0, 0.5, 1.0), outlier_frac=0.02)
    return make_linear("vitl_fc2", 3, 1, M, 4096, 1024, 64, ratios=(0.0, 0.5, 1.0), outlier_frac=0.02)


@dataclass
class ConvShape:
    name: str
    count: int
    HW: int      # input height = width
    C: int
    N: int
    R: int       # square filter
    stride: int

    @property
    def pad(self):
        return self.R // 2


def resnet50_shapes() -> List[ConvShape]:
    """Unique conv shapes of ResNet-50 stages 1-4 (bottleneck blocks, stride on the 3x3), with how
    often each occurs.  The 7x7 stem and the classifier stay at 8 bits in the paper and are left out."""
    return [
        ConvShape("s1_1x1_64_64", 1, 56, 64, 64, 1, 1),
        ConvShape("s1_3x3_64_64", 3, 56, 64, 64, 3, 1),
        ConvShape("s1_1x1_64_256", 4, 56, 64, 256, 1, 1),
        ConvShape("s1_1x1_256_64", 2, 56, 256, 64, 1, 1),
        ConvShape("s2_1x1_256_128", 1, 56, 256, 128, 1, 1),
        ConvShape("s2_3x3_128_128_s2", 1, 56, 128, 128, 3, 2),
        ConvShape("s2_1x1_128_512", 4, 28, 128, 512, 1, 1),
        ConvShape("s2_ds_1x1_256_512_s2", 1, 56, 256, 512, 1, 2),
        ConvShape("s2_1x1_512_128", 3, 28, 512, 128, 1, 1),
        ConvShape("s2_3x3_128_128", 3, 28, 128, 128, 3, 1),
        ConvShape("s3_1x1_512_256", 1, 28, 512, 256, 1, 1),
        ConvShape("s3_3x3_256_256_s2", 1, 28, 256, 256, 3, 2),
        ConvShape("s3_1x1_256_1024", 6, 14, 256, 1024, 1, 1),
        ConvShape("s3_ds_1x1_512_1024_s2", 1, 28, 512, 1024, 1, 2),
        ConvShape("s3_1x1_1024_256", 5, 14, 1024, 256, 1, 1),
        ConvShape("s3_3x3_256_256", 5, 14, 256, 256, 3, 1),
        ConvShape("s4_1x1_1024_512", 1, 14, 1024, 512, 1, 1),
        ConvShape("s4_3x3_512_512_s2", 1, 14, 512, 512, 3, 2),
        ConvShape("s4_1x1_512_2048", 3, 7, 512, 2048, 1, 1),
        ConvShape("s4_ds_1x1_1024_2048_s2", 1, 14, 1024, 2048, 1, 2),
        ConvShape("s4_1x1_2048_512", 2, 7, 2048, 512, 1, 1),
        ConvShape("s4_3x3_512_512", 2, 7, 512, 512, 3, 1),
    ]


def config4_layer(index: int, B: int = 128) -> ConvCase:
    sh = resnet50_shapes()[index]
    return make_conv(sh.name, 4, index, B, sh.HW, sh.HW, sh.C, sh.N, sh.R, sh.R, sh.stride, sh.pad, 32,
                     ratios=(0.0, 0.25, 0.5, 0.75, 1.0))


def config4_ratio_schedule(n_calls: int) -> np.ndarray:
    """Seeded per-call low-bit ratios for the runtime-switching configuration."""
    return _rng(4, 900).choice(np.array([0.0, 0.25, 0.5, 0.75, 1.0]), size=n_calls)
