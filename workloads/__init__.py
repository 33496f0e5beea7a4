"""Seeded synthetic inputs and layer-shape tables shared by tests, bench and smoke.

This module holds shapes and random tensors only: none of the method's
arithmetic (no norms, masks, packing, permutation search or convolution)
lives here, so both the CPU oracle's callers and the HIP path's callers can
draw identical inputs from it without sharing any computation.

The paper measured an ImageNet-trained MobileNet-v1 (Table 3, Table 4) and a
figure of "common input configurations" for single operators; neither the
weights nor the dataset are available, so tensors of the same shapes with
random values stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# MobileNet-v1 at 224x224 (the network of Table 3 / Table 4).  The paper prints
# only totals (568 M MACs, stem share 1.91 %); this is the standard 28-layer v1.
# ----------------------------------------------------------------------------


@dataclass(frozen=True)
class PwShape:
    """One pointwise (1x1) layer: input spatial size, channels in/out."""
    index: int       # 1..13
    hw: int          # input = output spatial size (square)
    c_in: int
    c_out: int


@dataclass(frozen=True)
class DwShape:
    """One depthwise 3x3 layer that precedes pointwise layer `index`."""
    index: int
    hw_in: int
    c: int
    stride: int

    @property
    def hw_out(self) -> int:
        return (self.hw_in + 2 - 3) // self.stride + 1


MOBILENET_V1_PW: Tuple[PwShape, ...] = (
    PwShape(1, 112, 32, 64),
    PwShape(2, 56, 64, 128),
    PwShape(3, 56, 128, 128),
    PwShape(4, 28, 128, 256),
    PwShape(5, 28, 256, 256),
    PwShape(6, 14, 256, 512),
    PwShape(7, 14, 512, 512),
    PwShape(8, 14, 512, 512),
    PwShape(9, 14, 512, 512),
    PwShape(10, 14, 512, 512),
    PwShape(11, 14, 512, 512),
    PwShape(12, 7, 512, 1024),
    PwShape(13, 7, 1024, 1024),
)

MOBILENET_V1_DW: Tuple[DwShape, ...] = (
    DwShape(1, 112, 32, 1),
    DwShape(2, 112, 64, 2),
    DwShape(3, 56, 128, 1),
    DwShape(4, 56, 128, 2),
    DwShape(5, 28, 256, 1),
    DwShape(6, 28, 256, 2),
    DwShape(7, 14, 512, 1),
    DwShape(8, 14, 512, 1),
    DwShape(9, 14, 512, 1),
    DwShape(10, 14, 512, 1),
    DwShape(11, 14, 512, 1),
    DwShape(12, 14, 512, 2),
    DwShape(13, 7, 1024, 1),
)

STEM = dict(hw_in=224, c_in=3, c_out=32, stride=2, hw_out=112)
FC = dict(c_in=1024, c_out=1000)

# ResNet-50-shaped 3x3 layers (stride 1, pad 1): (channels, spatial)
RESNET50_3X3: Tuple[Tuple[int, int], ...] = ((64, 56), (128, 28), (256, 14), (512, 7))


def mobilenet_v1_macs() -> dict:
    """Multiply-accumulate counts per layer family (shape bookkeeping only)."""
    stem = STEM["hw_out"] ** 2 * STEM["c_out"] * STEM["c_in"] * 9
    dw = sum(d.hw_out ** 2 * d.c * 9 for d in MOBILENET_V1_DW)
    pw = sum(p.hw ** 2 * p.c_in * p.c_out for p in MOBILENET_V1_PW)
    fc = FC["c_in"] * FC["c_out"]
    return dict(stem=stem, dw=dw, pw=pw, fc=fc, total=stem + dw + pw + fc)


# ----------------------------------------------------------------------------
# Random tensors.  numpy's PCG64 default_rng, one seed per tensor.
# ----------------------------------------------------------------------------

def uniform_activation(seed: int, shape) -> np.ndarray:
    """NHWC fp32 activations ~ U(-1, 1)."""
    rng = np.random.default_rng(seed)
    return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)


def normal_weights(seed: int, shape, std: float) -> np.ndarray:
    """OHWI fp32 weights ~ N(0, std^2)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=shape) * std).astype(np.float32)


def he_weights(seed: int, c_out: int, kh: int, kw: int, c_in: int) -> np.ndarray:
    """OHWI fp32 'random-init' weights ~ N(0, 2 / fan_in)."""
    return normal_weights(seed, (c_out, kh, kw, c_in), float(np.sqrt(2.0 / (kh * kw * c_in))))


def planted_weights(seed: int, c_out: int, c_in: int, n_profiles: int = 4, weak: float = 0.15) -> np.ndarray:
    """1x1 weights with structure for the rearrangement to find (trained networks have filters
    that attend to the same input channels; i.i.d. weights have none): filter f belongs to one of
    n_profiles profiles, drawn by a seeded shuffle so that neighbouring filters differ, and is
    He-normal on the 4-channel groups j with j % n_profiles == profile, `weak` times that
    elsewhere.  Input generator only: which grouping is best is for the search to find."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((c_out, 1, 1, c_in)) * np.sqrt(2.0 / c_in)
    profile = rng.permutation(c_out) % n_profiles
    group_of_channel = (np.arange(c_in) // 4) % n_profiles
    scale = np.where(profile[:, None] == group_of_channel[None, :], 1.0, weak)
    return (w * scale[:, None, None, :]).astype(np.float32)


def small_bias(seed: int, n: int) -> np.ndarray:
    """fp32 bias ~ N(0, 0.01^2)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=(n,)) * 0.01).astype(np.float32)


def uniform_block_mask(seed: int, rows: int, cols: int, n_removed: int) -> np.ndarray:
    """uint8 [rows][cols] mask with exactly n_removed zeros drawn without replacement."""
    rng = np.random.default_rng(seed)
    m = np.ones(rows * cols, dtype=np.uint8)
    m[rng.choice(rows * cols, size=n_removed, replace=False)] = 0
    return m.reshape(rows, cols)


def random_permutation(seed: int, n: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.permutation(n).astype(np.int32)


# ----------------------------------------------------------------------------
# The five named configurations (shapes and seeds only).
# ----------------------------------------------------------------------------

def config1():
    """Single 1x1 conv: x[1,14,14,64], W[128,1,1,64] ~ N(0,0.05^2), go=gi=4,
    256 of the 32x16 blocks removed uniformly without replacement."""
    w = normal_weights(1001, (128, 1, 1, 64), 0.05)
    mask = uniform_block_mask(1002, 128 // 4, 64 // 4, 256)
    x = uniform_activation(1003, (1, 14, 14, 64))
    return dict(x=x, w=w, mask=mask, go=4, gi=4)


def pw_layer_tensors(base_seed: int, layer: PwShape, batch: int, with_x: bool = True):
    """Weights / bias / input of one pointwise layer (configs 2-4 recipe)."""
    s = base_seed + layer.index
    w = he_weights(s, layer.c_out, 1, 1, layer.c_in)
    b = small_bias(s + 100, layer.c_out)
    x = uniform_activation(s + 200, (batch, layer.hw, layer.hw, layer.c_in)) if with_x else None
    return dict(w=w, bias=b, x=x)


def conv3x3_layer_tensors(base_seed: int, idx: int, batch: int, with_x: bool = True):
    """One ResNet-50-shaped 3x3 layer (config 5 recipe)."""
    c, hw = RESNET50_3X3[idx]
    s = base_seed + idx
    w = he_weights(s, c, 3, 3, c)
    b = small_bias(s + 100, c)
    x = uniform_activation(s + 200, (batch, hw, hw, c)) if with_x else None
    return dict(w=w, bias=b, x=x, c=c, hw=hw)


def dw_layer_tensors(base_seed: int, layer: DwShape):
    """Dense depthwise 3x3 weights [C][3][3] and bias for config 4."""
    s = base_seed + 50 + layer.index
    w = normal_weights(s, (layer.c, 3, 3), float(np.sqrt(2.0 / 9.0)))
    b = small_bias(s + 100, layer.c)
    return dict(w=w, bias=b)


def mobilenet_v1_tensors(base_seed: int = 4000):
    """Random-init parameters of the whole network (config 4 recipe): stem, 13 x (dw, pw), classifier."""
    stem = dict(w=he_weights(base_seed, STEM["c_out"], 3, 3, STEM["c_in"]), bias=small_bias(base_seed + 1, STEM["c_out"]))
    dws = [dw_layer_tensors(base_seed, d) for d in MOBILENET_V1_DW]
    pws = [pw_layer_tensors(base_seed, p, 1, with_x=False) for p in MOBILENET_V1_PW]
    fc = dict(w=he_weights(base_seed + 900, FC["c_out"], 1, 1, FC["c_in"]), bias=small_bias(base_seed + 901, FC["c_out"]))
    return dict(stem=stem, dw=dws, pw=pws, fc=fc)
