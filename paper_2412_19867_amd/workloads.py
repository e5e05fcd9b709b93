"""Seeded synthetic layers for the group-wise quantized Winograd convolution.

This module only describes shapes and draws random tensors.  It holds none of
the method's arithmetic (no transform, no quantizer, no convolution), so both
the HIP path and the CPU checker can be fed from it without sharing any code
that computes results.

The five layer sets stand in for the paper's workloads (3x3 stride-1 pad-1
convolutions of ResNet-18 and of a latent-diffusion UNet at 512 px / 1024 px,
Section "Experiments"); the paper's own checkpoints and datasets are not used.
Every tensor is a function of (config id, layer index) only.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np


@dataclass(frozen=True)
class Layer:
    """One 3x3 stride-1 pad-1 convolution, NHWC activations, OIHW weights."""

    cfg: int
    index: int
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    m: int            # Winograd output tile edge: F(m,3)
    group_size: int   # channels per quantization group along Cin
    x_dist: str       # "normal_outlier20" | "half_normal" | "student_t3_outlier30"
    w_dist: str       # "kaiming_gain" | "kaiming" | "normal002"
    row_scales: bool = False  # draw per-row scales u_B,u_G ~ U(0.5,2) (Eq. 11-13 inputs)
    repeat: int = 1   # how many times the conv is chained in a stack (config 5)

    @property
    def seed(self) -> int:
        return 1000 * self.cfg + self.index

    @property
    def n(self) -> int:
        return self.m + 2

    @property
    def tiles(self) -> int:
        return self.N * (-(-self.H // self.m)) * (-(-self.W // self.m))

    @property
    def direct_ops(self) -> int:
        """Multiply-adds x2 of the direct convolution this layer replaces."""
        return 2 * self.N * self.H * self.W * self.Cin * self.Cout * 9

    @property
    def name(self) -> str:
        return (f"cfg{self.cfg}.{self.index}:{self.N}x{self.H}x{self.W}:"
                f"{self.Cin}->{self.Cout}:F{self.m}g{self.group_size}")


def _layers() -> Dict[int, List[Layer]]:
    out: Dict[int, List[Layer]] = {}
    out[1] = [Layer(1, 0, 1, 32, 32, 64, 64, 4, 32, "normal_outlier20", "kaiming_gain")]
    out[2] = [Layer(2, i, 32, s, s, c, c, 6, 32, "half_normal", "kaiming")
              for i, (s, c) in enumerate([(56, 64), (28, 128), (14, 256), (7, 512)])]
    unet = [(64, 320, 320), (32, 640, 640), (16, 1280, 1280), (8, 1280, 1280)]
    out[3] = [Layer(3, i, 2, s, s, ci, co, 4, 64, "student_t3_outlier30", "normal002")
              for i, (s, ci, co) in enumerate(unet)]
    unet4 = unet + [(16, 2560, 1280), (64, 960, 320)]
    out[4] = [Layer(4, i, 2, s, s, ci, co, 6, 32, "student_t3_outlier30", "normal002",
                    row_scales=True)
              for i, (s, ci, co) in enumerate(unet4)]
    sdxl = [(128, 320), (64, 640), (32, 1280)]
    out[5] = [Layer(5, i, 2, s, s, c, c, 4, 64, "student_t3_outlier30", "normal002", repeat=4)
              for i, (s, c) in enumerate(sdxl)]
    # Not one of the five benchmark configurations: one large GEMM-shaped layer (2048 tiles,
    # 1280 -> 1280 channels) at two group sizes, to show what the contraction kernel reaches when
    # the per-tap matrices are big.  Timing only; the oracle would need minutes for it.
    out[6] = [Layer(6, i, 32, 32, 32, 1280, 1280, 4, g, "student_t3_outlier30", "normal002")
              for i, g in enumerate([64, 256])]
    return out


CONFIGS: Dict[int, List[Layer]] = _layers()


@dataclass
class LayerData:
    layer: Layer
    x: np.ndarray                 # [N,H,W,Cin] float32
    w: np.ndarray                 # [Cout,Cin,3,3] float32
    bias: np.ndarray              # [Cout] float32
    u_B: Optional[np.ndarray] = None   # [n] float64 row scales for B^T, or None
    u_G: Optional[np.ndarray] = None   # [n] float64 row scales for G, or None
    extra: dict = field(default_factory=dict)


def make_layer_data(layer: Layer, N: Optional[int] = None) -> LayerData:
    """Draw x, w, bias (and row scales) for a layer.  `N` overrides the batch
    (used to time a bounded sample of a layer on the host)."""
    rng = np.random.default_rng(layer.seed)
    nb = layer.N if N is None else N
    shape = (nb, layer.H, layer.W, layer.Cin)
    if layer.x_dist == "normal_outlier20":
        x = rng.standard_normal(shape, dtype=np.float32)
        ch = rng.choice(layer.Cin, size=2, replace=False)
        x[..., ch] *= np.float32(20.0)
    elif layer.x_dist == "half_normal":
        x = np.abs(rng.standard_normal(shape, dtype=np.float32))
    elif layer.x_dist == "student_t3_outlier30":
        x = (2.0 * rng.standard_t(3.0, size=shape)).astype(np.float32)
        k = max(1, int(round(0.01 * layer.Cin)))
        ch = rng.choice(layer.Cin, size=k, replace=False)
        x[..., ch] *= np.float32(30.0)
    else:
        raise ValueError(layer.x_dist)

    wshape = (layer.Cout, layer.Cin, 3, 3)
    if layer.w_dist in ("kaiming", "kaiming_gain"):
        std = np.float32(np.sqrt(2.0 / (9.0 * layer.Cin)))
        w = rng.standard_normal(wshape, dtype=np.float32) * std
        if layer.w_dist == "kaiming_gain":
            gain = rng.uniform(0.5, 2.0, size=(layer.Cout, 1, 1, 1)).astype(np.float32)
            w = w * gain
    elif layer.w_dist == "normal002":
        w = rng.standard_normal(wshape, dtype=np.float32) * np.float32(0.02)
    else:
        raise ValueError(layer.w_dist)
    bias = (rng.standard_normal(layer.Cout, dtype=np.float32) * np.float32(0.1))

    u_B = u_G = None
    if layer.row_scales:
        u_B = rng.uniform(0.5, 2.0, size=layer.n)
        u_G = rng.uniform(0.5, 2.0, size=layer.n)
    return LayerData(layer, np.ascontiguousarray(x, dtype=np.float32),
                     np.ascontiguousarray(w, dtype=np.float32),
                     np.ascontiguousarray(bias, dtype=np.float32), u_B, u_G)


def small_layer(seed: int, N: int, H: int, W: int, Cin: int, Cout: int, m: int,
                group_size: int, x_dist: str = "normal_outlier20",
                w_dist: str = "kaiming_gain", row_scales: bool = False) -> LayerData:
    """An ad-hoc layer for parity tests (ragged sizes, several tiles)."""
    lay = Layer(cfg=0, index=seed, N=N, H=H, W=W, Cin=Cin, Cout=Cout, m=m,
                group_size=group_size, x_dist=x_dist, w_dist=w_dist,
                row_scales=row_scales)
    return make_layer_data(lay)
