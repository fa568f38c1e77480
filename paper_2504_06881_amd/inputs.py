"""Seeded synthetic inputs for the tropical-convolution hot path.

This module only draws random tensors of the shapes and value distributions of
the benchmark layer configurations; it contains none of the operator's
arithmetic and imports neither the HIP binding nor the CPU oracle, so both
sides of a parity test can consume exactly the same host buffers.

The tensors stand in for the image-classification and segmentation feature maps
of the paper's experiments (CIFAR-sized 32x32 maps, ImageNet-style ResNet-18
stage shapes, segmentation-encoder maps; paper Sec. 5): activations ~ N(0, 1),
kernels uniform in a small symmetric range, upstream gradients ~ N(0, 1).
Draw order is fixed: x, W1, [W2 for parallel], gy, [alpha, beta].
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class LayerCfg:
    name: str
    N: int
    C_in: int
    H: int
    W: int
    C_out: int
    KH: int = 3
    KW: int = 3
    stride: int = 1
    pad: int = 1
    dil: int = 1
    mode: str = "max"          # max | min | compound | parallel | minplus_max | maxplus_min
    dtype: str = "f32"         # f32 | bf16 (storage of x, w, y)
    seed: int = 0
    w_range: float = 1.0       # kernels ~ U(-w_range, w_range)
    pad_mode: str = "identity"  # identity (padding never wins) | zero (padding holds zeros)
    stride_w: Optional[int] = None  # width parameters where they differ from the height's (None: the same)
    pad_w: Optional[int] = None
    dil_w: Optional[int] = None

    @property
    def stride_hw(self):
        return self.stride, self.stride if self.stride_w is None else self.stride_w

    @property
    def pad_hw(self):
        return self.pad, self.pad if self.pad_w is None else self.pad_w

    @property
    def dil_hw(self):
        return self.dil, self.dil if self.dil_w is None else self.dil_w

    @property
    def K(self) -> int:
        return self.C_in * self.KH * self.KW

    @property
    def out_hw(self):
        (sh, sw), (ph, pw), (dh, dw) = self.stride_hw, self.pad_hw, self.dil_hw
        ho = (self.H + 2 * ph - dh * (self.KH - 1) - 1) // sh + 1
        wo = (self.W + 2 * pw - dw * (self.KW - 1) - 1) // sw + 1
        return ho, wo

    @property
    def branches(self) -> int:
        return 2 if self.mode in ("compound", "parallel") else 1

    @property
    def candidates(self) -> int:
        ho, wo = self.out_hw
        return self.N * self.C_out * ho * wo * self.K

    @property
    def pairs(self) -> int:
        """add+compare pairs, dense count (padded taps included), one per candidate per branch."""
        return self.candidates * self.branches

    def with_(self, **kw) -> "LayerCfg":
        return replace(self, **kw)


# The benchmark layer configurations (single tropical conv layers).
CONFIGS: Dict[str, LayerCfg] = {c.name: c for c in [
    LayerCfg("cfg1", 2, 3, 16, 16, 8, mode="max", seed=0, w_range=1.0),
    LayerCfg("cfg2_main", 128, 64, 32, 32, 64, mode="compound", seed=1, w_range=0.1),
    LayerCfg("cfg2_stem", 128, 3, 32, 32, 16, mode="compound", seed=1, w_range=0.1),
    LayerCfg("cfg3a", 64, 64, 56, 56, 64, mode="parallel", seed=2, w_range=0.05),
    LayerCfg("cfg3b", 64, 128, 28, 28, 256, stride=2, mode="parallel", seed=2, w_range=0.05),
    LayerCfg("cfg3c", 64, 256, 14, 14, 256, mode="parallel", seed=2, w_range=0.05),
    LayerCfg("cfg4a", 8, 128, 128, 128, 128, mode="compound", seed=3, w_range=0.1),
    LayerCfg("cfg4b", 8, 256, 64, 64, 256, pad=2, dil=2, mode="compound", seed=3, w_range=0.1),
]}


def resnet20_layers(batch: int = 256, seed: int = 4):
    """The 19 tropical conv layers of a ResNet-20-style net on [batch, 3, 32, 32], all parallel mode."""
    layers = [LayerCfg("r20_stem", batch, 3, 32, 32, 16, mode="parallel", seed=seed, w_range=0.1)]
    spec = [(16, 32, 6), (32, 16, 6), (64, 8, 6)]
    c_prev, hw_prev = 16, 32
    li = 0
    for c, hw, n in spec:
        for b in range(n):
            first = (b == 0 and c != c_prev)
            layers.append(LayerCfg(f"r20_conv{li}", batch, c_prev if first else c,
                                   hw_prev if first else hw, hw_prev if first else hw, c,
                                   stride=2 if first else 1, mode="parallel", seed=seed + 1 + li,
                                   w_range=0.1))
            li += 1
        c_prev, hw_prev = c, hw
    return layers


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable fp32 (ties to even)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _no_neg_zero(a: np.ndarray) -> np.ndarray:
    return (a + np.float32(0.0)).astype(np.float32)


def make_inputs(cfg: LayerCfg, alpha_beta: Optional[str] = None, integer: bool = False,
                seed: Optional[int] = None) -> Dict[str, Optional[np.ndarray]]:
    """Draw x, w_min, w_max, gy, alpha, beta (numpy, host) for one layer configuration.

    alpha_beta: None -> alpha = beta = None (all ones); "random" -> U(-1, 1) per output
    channel; "half" -> 0.5 each; "contrast" -> (1, -1).
    integer: integer-valued x and w in [-4, 4] (every add exact, massive ties).
    Weight tensors: max and maxplus_min mode fill w_max, min and minplus_max mode w_min, compound one tensor returned
    as both, parallel two independent tensors (W1 -> w_min, W2 -> w_max).
    """
    rng = np.random.Generator(np.random.PCG64(cfg.seed if seed is None else seed))
    ho, wo = cfg.out_hw
    xs = (cfg.N, cfg.C_in, cfg.H, cfg.W)
    ws = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)

    def draw_x():
        if integer:
            return rng.integers(-4, 5, size=xs).astype(np.float32)
        return rng.standard_normal(size=xs, dtype=np.float32)

    def draw_w():
        if integer:
            return rng.integers(-4, 5, size=ws).astype(np.float32)
        return ((rng.random(size=ws, dtype=np.float32) * 2 - 1) * np.float32(cfg.w_range)).astype(np.float32)

    x = draw_x()
    w1 = draw_w()
    w2 = draw_w() if cfg.mode == "parallel" else None
    gy = rng.standard_normal(size=(cfg.N, cfg.C_out, ho, wo), dtype=np.float32)
    alpha = beta = None
    if alpha_beta == "random":
        alpha = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
        beta = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
    elif alpha_beta == "half":
        alpha = np.full(cfg.C_out, 0.5, np.float32)
        beta = np.full(cfg.C_out, 0.5, np.float32)
    elif alpha_beta == "contrast":
        alpha = np.full(cfg.C_out, 1.0, np.float32)
        beta = np.full(cfg.C_out, -1.0, np.float32)
    elif alpha_beta is not None:
        raise ValueError(alpha_beta)
    if cfg.dtype == "bf16":
        x, w1 = to_bf16_grid(x), to_bf16_grid(w1)
        w2 = to_bf16_grid(w2) if w2 is not None else None
    x, w1 = _no_neg_zero(x), _no_neg_zero(w1)
    w2 = _no_neg_zero(w2) if w2 is not None else None
    if cfg.mode in ("max", "maxplus_min"):
        w_min, w_max = None, w1
    elif cfg.mode in ("min", "minplus_max"):
        w_min, w_max = w1, None
    elif cfg.mode == "compound":
        w_min = w_max = w1
    else:
        w_min, w_max = w1, w2
    return dict(x=x, w_min=w_min, w_max=w_max, gy=gy, alpha=alpha, beta=beta)


# Depthwise layers: the 3x3 depthwise layers of a MobileNetV2 on 32x32 inputs (expansion 6, stride-1
# "custom" configuration of the paper's CIFAR runs) have 96 - 960 channels on 32x32 ... 4x4 maps.
DW_CONFIGS: Dict[str, LayerCfg] = {c.name: c for c in [
    LayerCfg("dw_small", 2, 6, 16, 16, 6, mode="compound", seed=60, w_range=1.0),
    LayerCfg("dw_main", 128, 192, 32, 32, 192, mode="compound", seed=61, w_range=0.1),
    LayerCfg("dw_s2", 128, 192, 32, 32, 192, stride=2, mode="compound", seed=62, w_range=0.1),
    LayerCfg("dw_16", 128, 384, 16, 16, 384, mode="compound", seed=63, w_range=0.1),
    LayerCfg("dw_8", 128, 576, 8, 8, 576, mode="compound", seed=64, w_range=0.1),
]}


def make_depthwise_inputs(cfg: LayerCfg, coef: Optional[str] = "random", integer: bool = False):
    """x [N, C_in, H, W], w_min / w_max [C_out, 1, KH, KW] (as make_inputs assigns them to the modes), gy,
    alpha / beta [C_out] (coef: None -> NULL, "random" -> U(-1, 1), "integer" -> small integers) for a
    depthwise layer with C_out = mult * C_in."""
    assert cfg.C_out % cfg.C_in == 0
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    ho, wo = cfg.out_hw
    xs, ws = (cfg.N, cfg.C_in, cfg.H, cfg.W), (cfg.C_out, 1, cfg.KH, cfg.KW)
    if integer:
        draw_x = lambda: rng.integers(-4, 5, size=xs).astype(np.float32)
        draw_w = lambda: rng.integers(-4, 5, size=ws).astype(np.float32)
    else:
        draw_x = lambda: rng.standard_normal(size=xs, dtype=np.float32)
        draw_w = lambda: ((rng.random(size=ws, dtype=np.float32) * 2 - 1) * np.float32(cfg.w_range)).astype(np.float32)
    x, w1 = _no_neg_zero(draw_x()), _no_neg_zero(draw_w())
    w2 = _no_neg_zero(draw_w()) if cfg.mode == "parallel" else None
    gy = rng.standard_normal(size=(cfg.N, cfg.C_out, ho, wo), dtype=np.float32)
    alpha = beta = None
    if coef is not None and cfg.mode in ("compound", "parallel"):
        if coef == "integer":
            alpha = rng.integers(-2, 3, cfg.C_out).astype(np.float32)
            beta = rng.integers(-2, 3, cfg.C_out).astype(np.float32)
        else:
            alpha = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
            beta = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
    if cfg.mode == "max":
        w_min, w_max = None, w1
    elif cfg.mode == "min":
        w_min, w_max = w1, None
    elif cfg.mode == "compound":
        w_min = w_max = w1
    else:
        w_min, w_max = w1, w2
    return dict(x=x, w_min=w_min, w_max=w_max, gy=gy, alpha=alpha, beta=beta)


# One-dimensional layers: shapes of 1-D LeNet-style audio classifiers (raw waveform in, a long first kernel
# with stride 4, then short kernels on a few thousand positions).
@dataclass(frozen=True)
class Layer1dCfg:
    name: str
    N: int
    C_in: int
    L: int
    C_out: int
    K: int = 3
    stride: int = 1
    pad: int = 1
    dil: int = 1
    mode: str = "max"
    dtype: str = "f32"
    seed: int = 0
    w_range: float = 1.0

    @property
    def L_out(self) -> int:
        return (self.L + 2 * self.pad - self.dil * (self.K - 1) - 1) // self.stride + 1

    @property
    def pairs(self) -> int:
        return self.N * self.C_out * self.L_out * self.C_in * self.K * (2 if self.mode in ("compound", "parallel") else 1)

    def with_(self, **kw) -> "Layer1dCfg":
        return replace(self, **kw)


CONFIGS_1D: Dict[str, Layer1dCfg] = {c.name: c for c in [
    Layer1dCfg("c1d_small", 2, 6, 100, 8, mode="compound", seed=90),
    Layer1dCfg("c1d_main", 64, 96, 8000, 96, mode="compound", seed=91, w_range=0.1),
    Layer1dCfg("c1d_stem", 64, 1, 32000, 64, K=80, stride=4, pad=38, mode="compound", seed=92, w_range=0.1),
]}


def make_1d_inputs(cfg: Layer1dCfg, alpha_beta: Optional[str] = None, integer: bool = False):
    """x [N, C_in, L], kernels [C_out, C_in, K] (assigned to the modes as make_inputs does), gy, alpha / beta."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    xs, ws = (cfg.N, cfg.C_in, cfg.L), (cfg.C_out, cfg.C_in, cfg.K)
    if integer:
        draw_x = lambda: rng.integers(-4, 5, size=xs).astype(np.float32)
        draw_w = lambda: rng.integers(-4, 5, size=ws).astype(np.float32)
    else:
        draw_x = lambda: rng.standard_normal(size=xs, dtype=np.float32)
        draw_w = lambda: ((rng.random(size=ws, dtype=np.float32) * 2 - 1) * np.float32(cfg.w_range)).astype(np.float32)
    x, w1 = draw_x(), draw_w()
    w2 = draw_w() if cfg.mode == "parallel" else None
    gy = rng.standard_normal(size=(cfg.N, cfg.C_out, cfg.L_out), dtype=np.float32)
    alpha = beta = None
    if alpha_beta == "random" and cfg.mode in ("compound", "parallel"):
        alpha = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
        beta = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
    if cfg.dtype == "bf16":
        x, w1 = to_bf16_grid(x), to_bf16_grid(w1)
        w2 = to_bf16_grid(w2) if w2 is not None else None
    x, w1 = _no_neg_zero(x), _no_neg_zero(w1)
    w2 = _no_neg_zero(w2) if w2 is not None else None
    if cfg.mode in ("max", "maxplus_min"):
        w_min, w_max = None, w1
    elif cfg.mode in ("min", "minplus_max"):
        w_min, w_max = w1, None
    elif cfg.mode == "compound":
        w_min = w_max = w1
    else:
        w_min, w_max = w1, w2
    return dict(x=x, w_min=w_min, w_max=w_max, gy=gy, alpha=alpha, beta=beta)


# Three-dimensional layers: shapes of small volumetric classifiers (voxel grids of a few tens per side).
@dataclass(frozen=True)
class Layer3dCfg:
    name: str
    N: int
    C_in: int
    D: int
    H: int
    W: int
    C_out: int
    k: tuple = (3, 3, 3)
    stride: tuple = (1, 1, 1)
    pad: tuple = (1, 1, 1)
    dil: tuple = (1, 1, 1)
    mode: str = "max"
    seed: int = 0
    w_range: float = 1.0

    @property
    def out(self):
        return tuple((n + 2 * p - d * (kk - 1) - 1) // s + 1
                     for n, kk, s, p, d in zip((self.D, self.H, self.W), self.k, self.stride, self.pad, self.dil))

    @property
    def pairs(self) -> int:
        do, ho, wo = self.out
        return (self.N * self.C_out * do * ho * wo * self.C_in * self.k[0] * self.k[1] * self.k[2]
                * (2 if self.mode in ("compound", "parallel") else 1))

    def with_(self, **kw) -> "Layer3dCfg":
        return replace(self, **kw)


CONFIGS_3D: Dict[str, Layer3dCfg] = {c.name: c for c in [
    Layer3dCfg("c3d_small", 2, 3, 6, 7, 8, 4, mode="compound", seed=120),
    Layer3dCfg("c3d_main", 32, 16, 28, 28, 28, 32, mode="compound", seed=121, w_range=0.1),
]}


def make_3d_inputs(cfg: Layer3dCfg, alpha_beta: Optional[str] = None, integer: bool = False):
    """x [N, C_in, D, H, W], kernels [C_out, C_in, KD, KH, KW] (assigned to the modes as make_inputs does), gy,
    alpha / beta."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    xs, ws = (cfg.N, cfg.C_in, cfg.D, cfg.H, cfg.W), (cfg.C_out, cfg.C_in) + tuple(cfg.k)
    if integer:
        draw_x = lambda: rng.integers(-4, 5, size=xs).astype(np.float32)
        draw_w = lambda: rng.integers(-4, 5, size=ws).astype(np.float32)
    else:
        draw_x = lambda: rng.standard_normal(size=xs, dtype=np.float32)
        draw_w = lambda: ((rng.random(size=ws, dtype=np.float32) * 2 - 1) * np.float32(cfg.w_range)).astype(np.float32)
    x, w1 = _no_neg_zero(draw_x()), _no_neg_zero(draw_w())
    w2 = _no_neg_zero(draw_w()) if cfg.mode == "parallel" else None
    gy = rng.standard_normal(size=(cfg.N, cfg.C_out) + cfg.out, dtype=np.float32)
    alpha = beta = None
    if alpha_beta == "random" and cfg.mode in ("compound", "parallel"):
        alpha = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
        beta = (rng.random(cfg.C_out, dtype=np.float32) * 2 - 1).astype(np.float32)
    if cfg.mode in ("max", "maxplus_min"):
        w_min, w_max = None, w1
    elif cfg.mode in ("min", "minplus_max"):
        w_min, w_max = w1, None
    elif cfg.mode == "compound":
        w_min = w_max = w1
    else:
        w_min, w_max = w1, w2
    return dict(x=x, w_min=w_min, w_max=w_max, gy=gy, alpha=alpha, beta=beta)
