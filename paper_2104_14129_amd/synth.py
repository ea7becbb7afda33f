"""Seeded synthetic workloads: shapes, value laws, widths and sensitivities.

This module only *makes inputs*.  It contains none of the quantizer's or the
allocator's arithmetic, and it is the one module that both the GPU tests and
the CPU oracle's tests draw their inputs from.

The tensors stand in for the activations the paper trains on (ImageNet
ResNet-50, detection / segmentation backbones), which are not available here:
shapes follow the public ResNet-50 v1.5 and FPN geometry, value laws are
post-ReLU Gaussians or heavy-tailed Laplace values with per-channel scales.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

G_DEFAULT = 256


@dataclass
class Workload:
    name: str
    shape: tuple            # (N, C, H, W)
    dtype: str              # "f32" | "f16"
    bits: np.ndarray        # uint8 [N]
    data_seed: int
    philox_seed: int
    tag: int = 0
    G: int = G_DEFAULT
    law: str = "relu_normal"     # see make_input
    law_args: dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(self.shape[0])

    @property
    def D(self) -> int:
        return int(np.prod(self.shape[1:]))

    @property
    def ng(self) -> int:
        return (self.D + self.G - 1) // self.G

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


def shuffled_multiset(counts: dict, seed: int) -> np.ndarray:
    """Widths with exact multiplicities, e.g. {1: 80, 2: 24, 4: 16, 8: 8}, in seeded order."""
    vals = np.concatenate([np.full(c, b, dtype=np.uint8) for b, c in sorted(counts.items())])
    rng = np.random.default_rng(seed)
    rng.shuffle(vals)
    return vals


def make_input(wl: Workload) -> np.ndarray:
    """Host tensor of wl.shape / wl.np_dtype drawn from wl.law with wl.data_seed."""
    rng = np.random.default_rng(wl.data_seed)
    N, C, H, W = wl.shape
    if wl.law == "normal":
        x = rng.standard_normal(wl.shape, dtype=np.float32)
    elif wl.law == "relu_normal":
        sigma = np.float32(wl.law_args.get("sigma", 1.0))
        x = rng.standard_normal(wl.shape, dtype=np.float32)
        if sigma != 1.0:
            x *= sigma
        np.maximum(x, 0.0, out=x)
        zero_planes = wl.law_args.get("zero_plane_fraction", 0.0)
        if zero_planes > 0.0:
            # whole (sample, channel) planes set to zero, so that groups whose
            # range is exactly zero really occur (dead channels after a ReLU)
            dead = rng.random((N, C)) < zero_planes
            x[dead] = 0.0
    elif wl.law == "laplace_channel_scale":
        lo, hi = wl.law_args.get("scale_range", (0.01, 10.0))
        s = np.exp(rng.uniform(np.log(lo), np.log(hi), size=C)).astype(np.float32)
        x = rng.laplace(0.0, 1.0, size=wl.shape).astype(np.float32)
        x *= s[None, :, None, None]
    else:
        raise ValueError(f"unknown law {wl.law}")
    return np.ascontiguousarray(x.astype(wl.np_dtype, copy=False))


def tiny() -> Workload:
    """fp32 [4,64,8,8], N(0,1), two bits everywhere."""
    return Workload("tiny_f32_4x64x8x8", (4, 64, 8, 8), "f32",
                    np.full(4, 2, dtype=np.uint8), data_seed=0, philox_seed=1, law="normal")


def r50_stage1(N: int = 128) -> Workload:
    """ResNet-50 stage-1 post-ReLU activation fp32 [128,256,56,56], mixed widths, mean 2.0."""
    counts = {1: 80 * N // 128, 2: 24 * N // 128, 4: 16 * N // 128, 8: 8 * N // 128}
    assert sum(counts.values()) == N, "N must be a multiple of 16"
    return Workload(f"r50_stage1_f32_{N}x256x56x56", (N, 256, 56, 56), "f32",
                    shuffled_multiset(counts, seed=1002), data_seed=2, philox_seed=12)


def r50_stem_f16(N: int = 256) -> Workload:
    """ResNet-50 stem activation fp16 [256,64,112,112], 10 % dead planes, two bits."""
    return Workload(f"r50_stem_f16_{N}x64x112x112", (N, 64, 112, 112), "f16",
                    np.full(N, 2, dtype=np.uint8), data_seed=3, philox_seed=13,
                    law_args={"sigma": 1.5, "zero_plane_fraction": 0.10})


def fpn(variant: int = 0, N: int = 8, H: int = 200, W: int = 304) -> Workload:
    """Detection-backbone activation fp32 [8,256,200,304], Laplace with per-channel scale."""
    counts = [{1: 4, 2: 2, 4: 2}, {1: 6, 2: 1, 8: 1}][variant]
    assert N == 8
    return Workload(f"fpn_f32_{N}x256x{H}x{W}_v{variant}", (N, 256, H, W), "f32",
                    shuffled_multiset(counts, seed=1004 + variant), data_seed=4,
                    philox_seed=14, law="laplace_channel_scale")


def resnet50_conv_input_shapes() -> list:
    """(C, H, W) of the input of each of the 53 convolutions of ResNet-50 v1.5 at 224x224."""
    shapes = [(3, 224, 224)]            # 7x7 stem
    c_in, hw = 64, 56                    # after the 3x3 max-pool
    for stage, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for blk in range(blocks):
            stride = 2 if (blk == 0 and stage > 0) else 1
            shapes.append((c_in, hw, hw))            # 1x1 reduce
            shapes.append((width, hw, hw))           # 3x3 (carries the stride in v1.5)
            hw_out = hw // stride
            shapes.append((width, hw_out, hw_out))   # 1x1 expand
            if blk == 0:
                shapes.append((c_in, hw, hw))        # 1x1 projection shortcut
            c_in, hw = width * 4, hw_out
    assert len(shapes) == 53
    assert sum(c * h * w for c, h, w in shapes) == 10_662_400
    return shapes


def lognormal_sensitivities(M: int, seed: int) -> np.ndarray:
    """Per-item sensitivities ~ LogNormal(0, 1), float32."""
    rng = np.random.default_rng(seed)
    return rng.lognormal(0.0, 1.0, size=M).astype(np.float32)


def tiered_sensitivities(bits: np.ndarray, seed: int) -> np.ndarray:
    """Sensitivities spread over orders of magnitude, one decade pair per width tier.

    Items are given weight 100**k (k = 0..3 for the tiers that should end at
    1, 2, 4, 8 bits) times a jitter in [0.9, 1.1]: a synthetic stand-in for the
    several-orders-of-magnitude spread of per-sample sensitivity.
    """
    rng = np.random.default_rng(seed)
    tier = {1: 0, 2: 1, 4: 2, 8: 3}
    base = np.array([100.0 ** tier[int(b)] for b in bits], dtype=np.float64)
    return (base * rng.uniform(0.9, 1.1, size=len(bits))).astype(np.float32)
