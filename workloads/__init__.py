"""Seeded synthetic inputs and layer-shape tables shared by the tests and the benchmark.

This module holds no arithmetic of the method: it only lists layer shapes and draws
weights, block masks, inputs and biases from ``numpy.random.Generator(PCG64(seed))``.
The same arrays are handed to the CPU oracle and to the HIP library, so neither side
re-implements a random generator.

The shapes are those of the networks the paper evaluates (MobileNet, ResNet-50 at
224x224 input, Section 4.1 of arXiv 2109.00170); the trained weights and masks are
not available, so kept weights are Gaussian and masks are random with the block
sparsity range the paper reports (about 70-84 % of MobileNet's parameters pruned).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional

import numpy as np

BASE_SEED = 210900170


def seed_for(config: int, layer: int) -> int:
    return BASE_SEED + 1000 * int(config) + int(layer)


def rng_for(config: int, layer: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed_for(config, layer)))


@dataclass(frozen=True)
class Layer:
    name: str
    Cin: int
    Cout: int
    H: int
    W: int
    k: int = 1
    stride: int = 1
    N: int = 1
    V: int = 4
    sparsity: float = 0.0       # fraction of blocks dropped
    repeats: int = 1            # how often the shape occurs in the network
    w_std: float = 0.1
    x_dist: str = "relu"        # "uniform" | "relu" | "relu6"
    mask_kind: str = "exact"    # "exact" | "zipf" | "none"
    tap_shared: bool = False    # 3x3: one [G,Cin] pattern copied to all taps

    @property
    def G(self) -> int:
        return (self.Cout + self.V - 1) // self.V

    @property
    def K(self) -> int:
        return self.Cin * self.k * self.k

    @property
    def Ho(self) -> int:
        return (self.H + 2 * ((self.k - 1) // 2) - self.k) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * ((self.k - 1) // 2) - self.k) // self.stride + 1

    def dense_flops(self) -> float:
        return 2.0 * self.N * self.Ho * self.Wo * self.Cout * self.K

    def x_bytes(self) -> int:
        return 4 * self.N * self.Cin * self.H * self.W

    def y_bytes(self) -> int:
        return 4 * self.N * self.Cout * self.Ho * self.Wo


# --------------------------------------------------------------------------- masks

def mask_exact(G: int, Cin: int, k: int, sparsity: float, rng: np.random.Generator,
               tap_shared: bool = False) -> np.ndarray:
    """Drop exactly round(sparsity * #blocks) blocks, chosen by a seeded permutation
    over the whole layer, so the per-group counts are unequal (as after a
    per-tensor top-N selection).  With ``tap_shared`` the pattern is drawn over
    [G, Cin] and copied to all k*k taps."""
    kk = 1 if tap_shared else k * k
    total = G * Cin * kk
    n_drop = int(round(float(sparsity) * total))
    flat = np.ones(total, dtype=np.uint8)
    flat[rng.permutation(total)[:n_drop]] = 0
    m = flat.reshape(G, Cin, kk)
    if tap_shared:
        m = np.repeat(m, k * k, axis=2)
    return np.ascontiguousarray(m.reshape(G, Cin, k, k))


def zipf_counts(G: int, K: int, mean_density: float) -> np.ndarray:
    """Kept blocks per group rank j: clip(round(c / (j+1)), 0, K), with c found by
    bisection so that the mean is mean_density * K (to rounding)."""
    target = mean_density * K
    ranks = np.arange(1, G + 1, dtype=np.float64)

    def counts(c):
        return np.clip(np.rint(c / ranks), 0, K)

    lo, hi = 0.0, float(K) * G * 4 + 1.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if counts(mid).mean() < target:
            lo = mid
        else:
            hi = mid
    return counts(hi).astype(np.int64)


def mask_zipf(G: int, Cin: int, k: int, mean_density: float, rng: np.random.Generator) -> np.ndarray:
    """Skewed sparsity: group lengths follow zipf_counts, ranks are assigned to groups
    by a seeded permutation, and each group keeps that many columns chosen uniformly
    without replacement.  Some groups end up full, some empty."""
    K = Cin * k * k
    cnt = zipf_counts(G, K, mean_density)
    owner = rng.permutation(G)
    m = np.zeros((G, K), dtype=np.uint8)
    for rank, g in enumerate(owner):
        keep = rng.permutation(K)[: int(cnt[rank])]
        m[g, keep] = 1
    return np.ascontiguousarray(m.reshape(G, Cin, k, k))


# --------------------------------------------------------------------------- tensors

@dataclass
class LayerData:
    layer: Layer
    W: np.ndarray               # [Cout,Cin,k,k] fp32 (dropped positions hold garbage on purpose)
    mask: Optional[np.ndarray]  # [G,Cin,k,k] uint8 or None
    X: np.ndarray               # [N,Cin,H,W] fp32
    bias: Optional[np.ndarray]  # [Cout] fp32 or None

    @property
    def nnzb(self) -> int:
        L = self.layer
        return L.G * L.K if self.mask is None else int(self.mask.sum())


def draw_x(shape, dist: str, rng: np.random.Generator) -> np.ndarray:
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    x = rng.standard_normal(size=shape, dtype=np.float32)
    np.maximum(x, 0.0, out=x)
    if dist == "relu6":
        np.minimum(x, 6.0, out=x)
    elif dist != "relu":
        raise ValueError(dist)
    return x


def make_layer(layer: Layer, seed: int, with_bias: bool = False, garbage: bool = True) -> LayerData:
    """Draw W, mask, X (and bias) for one layer.  Weights at dropped positions keep
    their Gaussian draw ("garbage") so that a path that ignores the mask is caught."""
    rng = np.random.Generator(np.random.PCG64(seed))
    L = layer
    if L.mask_kind == "none" or (L.mask_kind == "exact" and L.sparsity == 0.0):
        mask = None if L.mask_kind == "none" else np.ones((L.G, L.Cin, L.k, L.k), dtype=np.uint8)
    elif L.mask_kind == "exact":
        mask = mask_exact(L.G, L.Cin, L.k, L.sparsity, rng, tap_shared=L.tap_shared)
    elif L.mask_kind == "zipf":
        mask = mask_zipf(L.G, L.Cin, L.k, 1.0 - L.sparsity, rng)
    else:
        raise ValueError(L.mask_kind)
    W = (rng.standard_normal(size=(L.Cout, L.Cin, L.k, L.k), dtype=np.float32) * np.float32(L.w_std))
    if not garbage and mask is not None:
        keep = np.repeat(mask, L.V, axis=0)[: L.Cout]
        W = W * keep
    X = draw_x((L.N, L.Cin, L.H, L.W), L.x_dist, rng)
    bias = None
    if with_bias:
        bias = rng.standard_normal(size=(L.Cout,), dtype=np.float32)
    return LayerData(L, np.ascontiguousarray(W), mask, X, bias)


# --------------------------------------------------------------------------- configs

def config1() -> Layer:
    """Single 1x1 conv, batch 1, 64->64 at 56x56, V=4, half of the blocks dropped."""
    return Layer("c1_pw64", 64, 64, 56, 56, N=1, V=4, sparsity=0.5, w_std=0.1, x_dist="uniform")


_MBV1_PW = [(32, 64, 112), (64, 128, 56), (128, 128, 56), (128, 256, 28), (256, 256, 28),
            (256, 512, 14), (512, 512, 14), (512, 512, 14), (512, 512, 14), (512, 512, 14),
            (512, 512, 14), (512, 1024, 7), (1024, 1024, 7)]


def mobilenet_v1_pointwise(N: int, sparsity: Optional[float] = None) -> List[Layer]:
    """The 13 pointwise convs of MobileNetV1 at 224x224.  ``sparsity=None`` draws one
    value per layer from U(0.7, 0.9) (seeded by the layer's own seed); a number
    fixes it for all layers."""
    out = []
    for i, (ci, co, hw) in enumerate(_MBV1_PW):
        s = sparsity
        if s is None:
            s = float(np.random.Generator(np.random.PCG64(seed_for(2, 100 + i))).uniform(0.7, 0.9))
        out.append(Layer("pw%d" % (i + 1), ci, co, hw, hw, N=N, V=4, sparsity=s, w_std=0.1,
                         x_dist="relu"))
    return out


_MBV1_DW_STRIDE = [1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1]


def mobilenet_v1_blocks(N: int, sparsity: Optional[float] = None):
    """The 13 depthwise-separable blocks of MobileNetV1 at 224x224: (pointwise layer, stride of the
    depthwise 3x3 layer in front of it); the depthwise layer's input is stride times larger than
    the pointwise layer's."""
    return list(zip(mobilenet_v1_pointwise(N, sparsity), _MBV1_DW_STRIDE))


def resnet50_bottlenecks(N: int, sparsity: float = 0.8, distinct: bool = True) -> List[Layer]:
    """1x1 reduce / 3x3 / 1x1 expand convs of the 16 ResNet-50 bottleneck blocks at
    224x224 (stride on the 3x3 of each stage's first block).  ``distinct`` merges
    repeated shapes and records the repeat count."""
    stages = [(3, 64, 256, 56), (4, 128, 512, 56), (6, 256, 1024, 28), (3, 512, 2048, 14)]
    layers: List[Layer] = []
    cin = 64
    for si, (nblocks, width, cout, hin) in enumerate(stages):
        h = hin
        for b in range(nblocks):
            stride = 2 if (b == 0 and si > 0) else 1
            tag = "s%db%d" % (si + 1, b + 1)
            kw = dict(N=N, V=4, sparsity=sparsity, w_std=0.05, x_dist="relu")
            layers.append(Layer(tag + "_reduce", cin, width, h, h, k=1, **kw))
            layers.append(Layer(tag + "_3x3", width, width, h, h, k=3, stride=stride,
                                tap_shared=True, **kw))
            h = h // stride
            layers.append(Layer(tag + "_expand", width, cout, h, h, k=1, **kw))
            cin = cout
    if not distinct:
        return layers
    merged: List[Layer] = []
    for L in layers:
        for i, M in enumerate(merged):
            if (M.Cin, M.Cout, M.H, M.k, M.stride) == (L.Cin, L.Cout, L.H, L.k, L.stride):
                merged[i] = replace(M, repeats=M.repeats + 1)
                break
        else:
            merged.append(L)
    return merged


SWEEP_SPARSITIES = (0.0, 0.5, 0.7, 0.8, 0.9, 0.95)


def sweep_layer(sparsity: float, N: int = 256) -> Layer:
    """Config 4: one 1x1 conv 512->512 at 14x14, batch 256, V=4."""
    return Layer("sweep_s%02d" % int(round(sparsity * 100)), 512, 512, 14, 14, N=N, V=4,
                 sparsity=sparsity, w_std=0.1, x_dist="relu")


_MBV2_EXPAND = [(16, 96, 112, 1), (24, 144, 56, 2), (32, 192, 28, 3), (64, 384, 14, 4),
                (96, 576, 14, 3), (160, 960, 7, 3)]
_MBV2_PROJECT = [(32, 16, 112, 1), (96, 24, 56, 1), (144, 24, 56, 1), (144, 32, 28, 1), (192, 32, 28, 2),
                 (192, 64, 14, 1), (384, 64, 14, 3), (384, 96, 14, 1), (576, 96, 14, 2),
                 (576, 160, 7, 1), (960, 160, 7, 2), (960, 320, 7, 1)]


def mobilenet_v2_pointwise(N: int, V: int, mean_density: float = 0.15) -> List[Layer]:
    """Expansion (t=6) and projection 1x1 convs of MobileNetV2 at 224x224 with
    Zipf-like skewed group lengths."""
    out = []
    for kind, table in (("exp", _MBV2_EXPAND), ("proj", _MBV2_PROJECT)):
        for ci, co, hw, rep in table:
            out.append(Layer("%s_%dto%d_%d" % (kind, ci, co, hw), ci, co, hw, hw, N=N, V=V,
                             sparsity=1.0 - mean_density, repeats=rep, w_std=0.1,
                             x_dist="relu6", mask_kind="zipf"))
    return out


def macs_per_image(layers: List[Layer]) -> float:
    return sum(L.repeats * L.Ho * L.Wo * L.Cout * L.K for L in layers)
