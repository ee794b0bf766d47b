"""Seeded synthetic inputs for the sparse-convolution path.

This module only draws random numbers and names layer shapes.  It holds none of
the method's arithmetic (no convolution, no encoding, no pooling), so both the
CPU oracle's tests and the HIP path's tests can take their inputs from here
without sharing any code that matters for parity.

The paper measures on real feature maps of trained networks (Section 8); those
activations are not available, so every layer here is a stand-in with the
layer's shape and the zero ratio the paper reports for such layers (Fig. 2:
above 0.7 in deep layers; Table 3: 0.83-0.95).

Recipe (all host side, numpy ``default_rng``):
    keep  = rng.random(shape) >= z              # z = zero ratio (scalar or per channel)
    x     = where(keep, magnitude, 0) as fp32   # magnitude never exactly 0
    w     = rng.normal(0, std, shape) as fp32
    seed  = 190909927 + 1000 * config_index + 7 * layer_index + batch
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 190909927


@dataclasses.dataclass(frozen=True)
class Layer:
    """One convolution (optionally followed by max pooling) in the paper's notation.

    C,H,W: input channels / height / width; K,R,S: filters / kernel height / width;
    stride = c_s, pad = symmetric zero padding, groups = G; pool = (p_h, p_w, p_s) or None.
    zero_ratio: probability that an input element is zero; ``per_channel`` draws a
    separate ratio per channel uniformly from the given (lo, hi) range instead.
    """

    name: str
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    groups: int = 1
    pool: Optional[Tuple[int, int, int]] = None
    zero_ratio: float = 0.7
    per_channel: Optional[Tuple[float, float]] = None
    magnitude: str = "halfnormal"  # "halfnormal" = |N(0,1)|, "uniform" = U(0,1)
    structure: str = "iid"         # "iid" zeros, or "clustered": dead planes + spatial clusters
    w_std: Optional[float] = None  # None = He: sqrt(2 / (C_g*R*S))

    @property
    def Cg(self) -> int:
        return self.C // self.groups

    @property
    def Kg(self) -> int:
        return self.K // self.groups

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def with_structure(self, structure: str) -> "Layer":
        return dataclasses.replace(self, structure=structure, per_channel=None,
                                   name=f"{self.name}-{structure}")

    def with_zero_ratio(self, z: float) -> "Layer":
        return dataclasses.replace(self, zero_ratio=z, per_channel=None,
                                   name=f"{self.name}-z{z:.2f}")


def _vgg_std(C: int) -> float:
    return math.sqrt(2.0 / (9.0 * C))


# Index in this list = config index of the benchmark description.
CONFIGS: List[Dict] = [
    {
        "name": "tiny",
        "batches": (1,),
        "layers": [
            Layer("tiny-16x28-k32", C=16, H=28, W=28, K=32, R=3, S=3, stride=1, pad=1,
                  zero_ratio=0.7, magnitude="uniform", w_std=0.1),
        ],
    },
    {
        "name": "vgg19",
        "batches": (1, 8),
        "layers": [
            Layer("vgg-256x56", C=256, H=56, W=56, K=256, R=3, S=3, pad=1,
                  zero_ratio=0.60, w_std=_vgg_std(256)),
            Layer("vgg-512x28", C=512, H=28, W=28, K=512, R=3, S=3, pad=1,
                  zero_ratio=0.75, w_std=_vgg_std(512)),
            Layer("vgg-512x14-pool", C=512, H=14, W=14, K=512, R=3, S=3, pad=1,
                  zero_ratio=0.85, w_std=_vgg_std(512), pool=(2, 2, 2)),
        ],
    },
    {
        "name": "resnet50",
        "batches": (1, 32),
        "layers": [
            Layer("rn-1x1-256to64x56", C=256, H=56, W=56, K=64, R=1, S=1,
                  per_channel=(0.5, 0.8)),
            Layer("rn-3x3-64x56", C=64, H=56, W=56, K=64, R=3, S=3, pad=1,
                  per_channel=(0.5, 0.8)),
            Layer("rn-3x3-128x56-s2", C=128, H=56, W=56, K=128, R=3, S=3, stride=2, pad=1,
                  per_channel=(0.5, 0.8)),
            Layer("rn-3x3-512x7", C=512, H=7, W=7, K=512, R=3, S=3, pad=1,
                  per_channel=(0.5, 0.8)),
        ],
    },
    {
        "name": "densenet121",
        "batches": (1, 16),
        "layers": [
            Layer("dn-1x1-256to128x28", C=256, H=28, W=28, K=128, R=1, S=1),
            Layer("dn-1x1-384to128x28", C=384, H=28, W=28, K=128, R=1, S=1),
            Layer("dn-1x1-512to128x28", C=512, H=28, W=28, K=128, R=1, S=1),
            Layer("dn-3x3-128to32x28", C=128, H=28, W=28, K=32, R=3, S=3, pad=1),
            Layer("dn-T-1x1-512to256x28-pool", C=512, H=28, W=28, K=256, R=1, S=1,
                  pool=(2, 2, 2)),
        ],
    },
    {
        "name": "regnetx16gf",
        "batches": (1, 32),
        "layers": [
            Layer("rx-896x14-g7", C=896, H=14, W=14, K=896, R=3, S=3, pad=1, groups=7),
            Layer("rx-2048x7-g16", C=2048, H=7, W=7, K=2048, R=3, S=3, pad=1, groups=16),
        ],
    },
    {
        # Single layers on small maps (Table 3 lists network, layer, map size and zero ratio but no
        # channel counts or kernel sizes; those are the public architectures' for the named layer,
        # with the map size as printed).
        "name": "single",
        "batches": (1, 32),
        "layers": [
            Layer("lenet-conv2-5x5-20to50x11", C=20, H=11, W=11, K=50, R=5, S=5, zero_ratio=0.95),
            Layer("alexnet-conv3-256to384x6", C=256, H=6, W=6, K=384, R=3, S=3, pad=1, zero_ratio=0.9),
            Layer("alexnet-conv4-384x5-g2", C=384, H=5, W=5, K=384, R=3, S=3, pad=1, groups=2,
                  zero_ratio=0.9),
            Layer("googlenet-4a-1x1-480to192x14", C=480, H=14, W=14, K=192, R=1, S=1, zero_ratio=0.9),
            Layer("googlenet-4a-1x1-480to96x14", C=480, H=14, W=14, K=96, R=1, S=1, zero_ratio=0.9),
            Layer("googlenet-4e-3x3-160to320x14", C=160, H=14, W=14, K=320, R=3, S=3, pad=1,
                  zero_ratio=0.9),
            Layer("googlenet-5a-1x1-832to256x7", C=832, H=7, W=7, K=256, R=1, S=1, zero_ratio=0.95),
            Layer("googlenet-5a-1x1-832to160x7", C=832, H=7, W=7, K=160, R=1, S=1, zero_ratio=0.9),
            Layer("googlenet-5b-3x3-192to384x7", C=192, H=7, W=7, K=384, R=3, S=3, pad=1,
                  zero_ratio=0.95),
            Layer("googlenet-5x5-48to128x7", C=48, H=7, W=7, K=128, R=5, S=5, pad=2, zero_ratio=0.95),
            Layer("vgg-conv15-512x14", C=512, H=14, W=14, K=512, R=3, S=3, pad=1, zero_ratio=0.83),
            Layer("resnet-conv42-256x14", C=256, H=14, W=14, K=256, R=3, S=3, pad=1, zero_ratio=0.86),
            # convolution + pooling pairs with the two other pooling windows of those networks
            Layer("lenet-conv1-5x5-1to20x28-pool2", C=1, H=28, W=28, K=20, R=5, S=5, pool=(2, 2, 2),
                  zero_ratio=0.8),
            Layer("alexnet-conv5-384to256x13-g2-pool3", C=384, H=13, W=13, K=256, R=3, S=3, pad=1, groups=2,
                  pool=(3, 3, 2), zero_ratio=0.9),
        ],
    },
]

SWEEP_ZERO_RATIOS = tuple(round(0.05 * i, 2) for i in range(20))  # 0.00 .. 0.95


def layer_seed(config_index: int, layer_index: int, batch: int) -> int:
    return BASE_SEED + 1000 * config_index + 7 * layer_index + batch


def make_feature_map(rng: np.random.Generator, N: int, layer: Layer) -> np.ndarray:
    """fp32 NCHW feature map with the layer's zero ratio; nonzeros are strictly positive."""
    shape = (N, layer.C, layer.H, layer.W)
    if layer.per_channel is not None:
        lo, hi = layer.per_channel
        z = rng.uniform(lo, hi, size=(1, layer.C, 1, 1))  # same ratios for every image
    else:
        z = layer.zero_ratio
    if layer.structure == "clustered":
        keep = _clustered_keep(rng, shape, float(layer.zero_ratio))
    else:
        keep = rng.random(shape) >= z
    if layer.magnitude == "uniform":
        mag = rng.random(shape)
    else:
        mag = np.abs(rng.standard_normal(shape))
    mag = mag.astype(np.float32)
    # a drawn magnitude that rounds to exactly 0 would silently raise the zero ratio
    mag[mag == 0] = np.float32(0.5)
    return np.where(keep, mag, np.float32(0)).astype(np.float32)


def _clustered_keep(rng: np.random.Generator, shape, z: float) -> np.ndarray:
    """Nonzero mask with the structure ReLU maps tend to have and i.i.d. zeros lack: a share
    0.3*z of the (image, channel) planes is entirely zero, and inside the other planes the zeros
    form patches (a smooth field on a 4x4-coarser grid plus a little per-element noise, cut at the
    quantile that gives the plane its share of zeros).  The overall zero ratio is z."""
    N, C, H, W = shape
    p_dead = 0.3 * z
    z_alive = (z - p_dead) / (1.0 - p_dead) if p_dead < 1.0 else 1.0
    dead = rng.random((N, C, 1, 1)) < p_dead
    coarse = rng.standard_normal((N, C, (H + 3) // 4, (W + 3) // 4)).astype(np.float32)
    field = np.repeat(np.repeat(coarse, 4, axis=2), 4, axis=3)[:, :, :H, :W]
    field = field + 0.5 * rng.standard_normal(shape).astype(np.float32)
    cut = np.quantile(field.reshape(N, C, -1), z_alive, axis=2).astype(np.float32)
    keep = field > cut[:, :, None, None]
    return keep & ~dead


def make_filters(rng: np.random.Generator, layer: Layer) -> np.ndarray:
    """fp32 filters [K][C/groups][R][S], zero-mean normal."""
    std = layer.w_std if layer.w_std is not None else math.sqrt(2.0 / (layer.Cg * layer.R * layer.S))
    w = rng.normal(0.0, std, size=(layer.K, layer.Cg, layer.R, layer.S))
    return w.astype(np.float32)


def make_layer_inputs(config_index: int, layer_index: int, N: int,
                      layer: Optional[Layer] = None) -> Tuple[Layer, np.ndarray, np.ndarray]:
    """(layer, x, w) for one layer of one config at batch N, seeded as the recipe states."""
    if layer is None:
        layer = CONFIGS[config_index]["layers"][layer_index]
    rng = np.random.default_rng(layer_seed(config_index, layer_index, N))
    x = make_feature_map(rng, N, layer)
    w = make_filters(rng, layer)
    return layer, x, w


def make_random_case(seed: int, N: int, C: int, H: int, W: int, K: int, R: int, S: int,
                     stride: int = 1, pad: int = 0, groups: int = 1,
                     pool: Optional[Tuple[int, int, int]] = None, zero_ratio: float = 0.7,
                     integer_valued: bool = False) -> Tuple[Layer, np.ndarray, np.ndarray]:
    """Arbitrary small shape for parity tests.

    integer_valued: x in {0,1,2,3} and w in {-2..2}, so every fp32 summation order is exact
    and a GPU result must equal the fp64 result bit for bit.
    """
    layer = Layer(f"case-{seed}", C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad,
                  groups=groups, pool=pool, zero_ratio=zero_ratio)
    rng = np.random.default_rng(seed)
    if integer_valued:
        keep = rng.random((N, C, H, W)) >= zero_ratio
        x = np.where(keep, rng.integers(1, 4, size=(N, C, H, W)), 0).astype(np.float32)
        w = rng.integers(-2, 3, size=(K, C // groups, R, S)).astype(np.float32)
    else:
        x = make_feature_map(rng, N, layer)
        w = make_filters(rng, layer)
    return layer, x, w


# A chain of layers in which every layer consumes the previous layer's output (the paper's
# procedure keeps the result of one layer as the next layer's input, Section 5.1): the tail of a
# VGG-19-shaped network from the 28x28 stage on.  Only the first input is drawn; every later map
# is whatever ReLU (and pooling) left, so its zeros have the structure a network produces.
# Trained filters and biases are what push real maps beyond 50 % zeros; as a stand-in the filters
# get a small negative mean, CHAIN_W_SHIFT standard deviations, which leaves 70-90 % zeros.
CHAIN_W_SHIFT = -0.03
CHAIN = [
    Layer("chain-256to512x28", C=256, H=28, W=28, K=512, R=3, S=3, pad=1, zero_ratio=0.6),
    Layer("chain-512x28-a", C=512, H=28, W=28, K=512, R=3, S=3, pad=1),
    Layer("chain-512x28-b", C=512, H=28, W=28, K=512, R=3, S=3, pad=1),
    Layer("chain-512x28-pool", C=512, H=28, W=28, K=512, R=3, S=3, pad=1, pool=(2, 2, 2)),
    Layer("chain-512x14-a", C=512, H=14, W=14, K=512, R=3, S=3, pad=1),
    Layer("chain-512x14-b", C=512, H=14, W=14, K=512, R=3, S=3, pad=1),
    Layer("chain-512x14-pool", C=512, H=14, W=14, K=512, R=3, S=3, pad=1, pool=(2, 2, 2)),
]


def make_chain_inputs(N: int, layers=None, shift: float = CHAIN_W_SHIFT):
    """(first input x, [filters per layer]) for the chain at batch N, seeded."""
    layers = CHAIN if layers is None else layers
    rng = np.random.default_rng(BASE_SEED + 9000 + N)
    x = make_feature_map(rng, N, layers[0])
    ws = []
    for layer in layers:
        w = make_filters(rng, layer)
        std = layer.w_std if layer.w_std is not None else math.sqrt(2.0 / (layer.Cg * layer.R * layer.S))
        ws.append((w + np.float32(shift * std)).astype(np.float32))
    return x, ws
