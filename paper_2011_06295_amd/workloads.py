"""Seeded synthetic workloads for direct sparse convolution.

This module only *draws inputs*: layer shapes, dense weights, pruning masks and
input feature maps.  It contains none of the method's arithmetic (no CSR
encoding, no convolution) and imports neither the CPU oracle nor the HIP
binding, so both sides can be fed from it.

The paper prunes VGG-16 / ResNet50 / DenseNet trained on CIFAR-10/100 and times
direct sparse convolution layer by layer at ~90 % sparsity with one unified
non-zero count per output channel (sections 7, 8 and 9).  Neither the datasets
nor trained weights are available here, so every tensor below is a seeded
synthetic stand-in with the shape, value distribution and sparsity structure of
those workloads.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 20110629


def seed_for(config: int, layer: int) -> int:
    """Seed of (config, layer), both 1-based; masks use this seed + 500."""
    return BASE_SEED + 1000 * int(config) + int(layer)


def nnz_per_row(L: int, sparsity_bp: int) -> int:
    """Stored entries per output channel for a sparsity given in basis points.

    Integer round-half-up of L*(1-sparsity), at least one entry per row.
    """
    return max(1, (L * (10000 - int(sparsity_bp)) + 5000) // 10000)


@dataclass
class LayerSpec:
    """One convolution layer of a synthetic workload."""

    name: str
    C: int
    K: int
    R: int
    S: int
    H: int
    W: int
    stride: int = 1
    pad: int = 0
    sparsity_bp: int = 9000
    mask_kind: str = "exact"  # "exact" | "bernoulli" | "beta22"
    w_std: Optional[float] = None  # None: sqrt(2 / nnz_row) (Kaiming on kept fan-in)
    relu_after: bool = False
    pool_after: bool = False  # 2x2 / stride-2 max-pool after (the optional ReLU)
    pool_before_relu: bool = False

    @property
    def L(self) -> int:
        return self.C * self.R * self.S

    @property
    def E(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def F(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def row_nnz(self) -> int:
        return nnz_per_row(self.L, self.sparsity_bp)


@dataclass
class Workload:
    name: str
    config: int
    N: int
    dtype: str  # "f32" | "f16"
    input_dist: str  # "uniform01" | "normal"
    layers: List[LayerSpec] = field(default_factory=list)
    chain: bool = True  # False: independent layers, each with its own input (make_layer_input)


# --------------------------------------------------------------------------
# masks
# --------------------------------------------------------------------------

def mask_bernoulli(rng: np.random.Generator, K: int, L: int, sparsity_bp: int) -> np.ndarray:
    """i.i.d. mask, P(zero) = sparsity; rows are ragged."""
    keep = rng.random((K, L)) >= (sparsity_bp / 10000.0)
    return keep.astype(np.uint8)


def mask_exact(rng: np.random.Generator, K: int, L: int, k_per_row: int) -> np.ndarray:
    """Exactly k_per_row kept positions per row, uniformly random positions."""
    m = np.zeros((K, L), dtype=np.uint8)
    for k in range(K):
        m[k, rng.choice(L, size=k_per_row, replace=False)] = 1
    return m


def ragged_row_counts(rng: np.random.Generator, K: int, L: int, sparsity_bp: int) -> np.ndarray:
    """Per-row kept counts with density 2(1-s)*Beta(2,2), total equal to the
    unified case K*nnz_per_row(L, s)."""
    dens = 1.0 - sparsity_bp / 10000.0
    b = rng.beta(2.0, 2.0, size=K)
    cnt = np.clip(np.rint(L * 2.0 * dens * b).astype(np.int64), 0, L)
    target = K * nnz_per_row(L, sparsity_bp)
    diff = int(target - cnt.sum())
    step = 1 if diff > 0 else -1
    k = 0
    guard = 0
    while diff != 0:
        if 0 <= cnt[k] + step <= L:
            cnt[k] += step
            diff -= step
        k = (k + 1) % K
        guard += 1
        if guard > 4 * K * L:
            raise RuntimeError("cannot reach target nnz")
    return cnt


def mask_ragged(rng: np.random.Generator, K: int, L: int, sparsity_bp: int) -> np.ndarray:
    cnt = ragged_row_counts(rng, K, L, sparsity_bp)
    m = np.zeros((K, L), dtype=np.uint8)
    for k in range(K):
        if cnt[k]:
            m[k, rng.choice(L, size=int(cnt[k]), replace=False)] = 1
    return m


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------

def make_mask(config: int, layer: int, spec: LayerSpec) -> np.ndarray:
    """uint8 mask [K][C][R][S], nonzero = weight survives pruning."""
    rng = np.random.Generator(np.random.PCG64(seed_for(config, layer) + 500))
    K, L = spec.K, spec.L
    if spec.mask_kind == "bernoulli":
        m = mask_bernoulli(rng, K, L, spec.sparsity_bp)
    elif spec.mask_kind == "exact":
        m = mask_exact(rng, K, L, spec.row_nnz)
    elif spec.mask_kind == "beta22":
        m = mask_ragged(rng, K, L, spec.sparsity_bp)
    else:
        raise ValueError(spec.mask_kind)
    return m.reshape(K, spec.C, spec.R, spec.S)


def make_weights(config: int, layer: int, spec: LayerSpec) -> np.ndarray:
    """Dense fp32 weights [K][C][R][S] (before masking)."""
    rng = np.random.Generator(np.random.PCG64(seed_for(config, layer)))
    std = spec.w_std if spec.w_std is not None else float(np.sqrt(2.0 / spec.row_nnz))
    w = rng.standard_normal((spec.K, spec.C, spec.R, spec.S)) * std
    return w.astype(np.float32)


def make_codebook(config: int, layer: int, spec: LayerSpec, with_zero: bool = False):
    """Stand-in for a cluster-quantised layer (the paper's 4-bit configuration: 16 centroids): centroid
    numbers uint8 [K][C][R][S] drawn uniformly and 16 sorted centroids fp32 drawn like the weights
    (with_zero: the one nearest to zero is set to zero, as a layer that is to be unified needs)."""
    rng = np.random.Generator(np.random.PCG64(seed_for(config, layer) + 700))
    std = spec.w_std if spec.w_std is not None else float(np.sqrt(2.0 / spec.row_nnz))
    centroids = np.sort(rng.standard_normal(16) * std).astype(np.float32)
    if with_zero:
        centroids[int(np.argmin(np.abs(centroids)))] = 0.0
    index = rng.integers(0, 16, (spec.K, spec.C, spec.R, spec.S)).astype(np.uint8)
    return index, centroids


def pattern_value(flat_index):
    """Input value at a flat element index for tensors too large to draw and copy: a fixed pattern of
    251 small dyadic values, exact in binary16 and fp32 (works on numpy arrays and torch tensors alike)."""
    return ((flat_index % 251) - 125) / 64.0


def make_input(wl: Workload, N: Optional[int] = None) -> np.ndarray:
    """fp32 input feature maps [N][C][H][W] of the first layer."""
    rng = np.random.Generator(np.random.PCG64(seed_for(wl.config, 900)))
    l0 = wl.layers[0]
    n = wl.N if N is None else int(N)
    shape = (n, l0.C, l0.H, l0.W)
    if wl.input_dist == "uniform01":
        x = rng.random(shape)
    elif wl.input_dist == "normal":
        x = rng.standard_normal(shape)
    else:
        raise ValueError(wl.input_dist)
    return x.astype(np.float32)


def make_layer_input(config: int, layer: int, spec: LayerSpec, N: int, dist: str = "normal") -> np.ndarray:
    """Stand-alone fp32 input for one layer (used when a layer is run outside its chain)."""
    rng = np.random.Generator(np.random.PCG64(seed_for(config, layer) + 700))
    shape = (N, spec.C, spec.H, spec.W)
    x = rng.random(shape) if dist == "uniform01" else rng.standard_normal(shape)
    return x.astype(np.float32)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config1() -> Workload:
    """Single 3x3 layer, batch 1, Bernoulli 90 % mask (ragged rows)."""
    return Workload(
        "single3x3", 1, 1, "f32", "uniform01",
        [LayerSpec("conv", C=16, K=32, R=3, S=3, H=16, W=16, stride=1, pad=1,
                   sparsity_bp=9000, mask_kind="bernoulli", w_std=0.05)],
    )


def lenet5(N: int = 64) -> Workload:
    """LeNet-5-style stack: conv1 -> maxpool -> ReLU -> conv2, 90 % unified."""
    return Workload(
        "lenet5", 2, N, "f32", "uniform01",
        [
            LayerSpec("conv1", C=1, K=20, R=5, S=5, H=28, W=28, pad=0, sparsity_bp=9000,
                      w_std=0.1, relu_after=True, pool_after=True, pool_before_relu=True),
            LayerSpec("conv2", C=20, K=50, R=5, S=5, H=12, W=12, pad=0, sparsity_bp=9000,
                      w_std=0.1),
        ],
    )


VGG_WIDTHS = [(64, 64), (128, 128), (256, 256, 256), (512, 512, 512), (512, 512, 512)]


def vgg16(N: int = 128, dtype: str = "f32", image: int = 32, config: Optional[int] = None) -> Workload:
    """VGG-16-style 13-layer stack for 32x32 images; per-layer unified sparsity
    rising linearly from 80 % (layer 1) to 95 % (layer 13)."""
    cfg = config if config is not None else (3 if dtype == "f32" else 4)
    layers: List[LayerSpec] = []
    c_in, hw, idx = 3, image, 0
    for group in VGG_WIDTHS:
        for gi, width in enumerate(group):
            idx += 1
            layers.append(LayerSpec(
                f"conv{idx}", C=c_in, K=width, R=3, S=3, H=hw, W=hw, stride=1, pad=1,
                sparsity_bp=8000 + 125 * (idx - 1), mask_kind="exact",
                relu_after=True, pool_after=(gi == len(group) - 1)))
            c_in = width
        hw //= 2
    return Workload(f"vgg16_{image}px_{dtype}", cfg, N, dtype, "normal", layers)


SWEEP_SPARSITIES_BP = [5000, 7000, 8000, 9000, 9500, 9900]


def sweep_layer(sparsity_bp: int, ragged: bool, N: int = 256) -> Workload:
    """One 256->256 3x3 layer on 14x14 maps at a given sparsity, unified or ragged rows."""
    L = 256 * 9
    spec = LayerSpec(
        f"sweep_{sparsity_bp}{'_ragged' if ragged else ''}", C=256, K=256, R=3, S=3,
        H=14, W=14, stride=1, pad=1, sparsity_bp=sparsity_bp,
        mask_kind="beta22" if ragged else "exact",
        w_std=float(np.sqrt(2.0 / nnz_per_row(L, sparsity_bp))))
    return Workload(spec.name, 5, N, "f32", "normal", [spec])


def sweep_layer_index(sparsity_bp: int, ragged: bool) -> int:
    """Layer number used for seeding a sweep point (1-based, unified then ragged)."""
    return 1 + SWEEP_SPARSITIES_BP.index(sparsity_bp) + (len(SWEEP_SPARSITIES_BP) if ragged else 0)


# --------------------------------------------------------------------------
# 1x1 and 1-D layers (the paper's ResNet / DenseNet bottlenecks and its
# CNN-non-static text model); independent layers, not a chain
# --------------------------------------------------------------------------

def resnet_1x1(N: int = 128, dtype: str = "f32") -> Workload:
    """The two ResNet-50 bottleneck 1x1 layers of the paper's result tables ("256 filters
    1x1x64" and "64 filters 1x1x256"), 90 % unified sparsity, on 56x56 maps (the
    ImageNet-sized stage those filter counts belong to)."""
    return Workload(f"resnet_1x1_{dtype}", 6, N, dtype, "normal", [
        LayerSpec("res_256f_1x1x64", C=64, K=256, R=1, S=1, H=56, W=56, pad=0, sparsity_bp=9000),
        LayerSpec("res_64f_1x1x256", C=256, K=64, R=1, S=1, H=56, W=56, pad=0, sparsity_bp=9000),
    ], chain=False)


def densenet_1x1(N: int = 128, dtype: str = "f32") -> Workload:
    """The DenseNet 1x1 bottleneck layers of the paper's table: input channels are the block
    input plus (layer - 1) * growth, output 4 * growth, at the block's map size."""
    return Workload(f"densenet_1x1_{dtype}", 7, N, dtype, "normal", [
        LayerSpec("dn121_b3_l24_87", C=256 + 23 * 32, K=128, R=1, S=1, H=14, W=14, pad=0, sparsity_bp=8750),
        LayerSpec("dn121_b3_l24_91", C=256 + 23 * 32, K=128, R=1, S=1, H=14, W=14, pad=0, sparsity_bp=9100),
        LayerSpec("dn161_b4_l16_91", C=1056 + 15 * 48, K=192, R=1, S=1, H=7, W=7, pad=0, sparsity_bp=9100),
        LayerSpec("dn161_b3_l16_93", C=384 + 15 * 48, K=192, R=1, S=1, H=14, W=14, pad=0, sparsity_bp=9300),
    ], chain=False)


def cnn_1d(N: int = 128, dtype: str = "f32") -> Workload:
    """1-D convolutions of the CNN-non-static text model: a sentence of 64 words with
    300-dimensional embeddings is read as 300 channels of length 64 (H = 1), 100 filters
    spanning 2 or 3 words, at the paper's three sparsity levels."""
    layers = []
    for ks in (2, 3):
        for s_bp in (7700, 8300, 8750):
            layers.append(LayerSpec(f"cnn1d_k{ks}_{s_bp // 100}", C=300, K=100, R=1, S=ks, H=1, W=64,
                                    pad=0, sparsity_bp=s_bp))
    return Workload(f"cnn_1d_{dtype}", 8, N, dtype, "normal", layers, chain=False)


VGG_IMAGENET_LAYERS = [(3, 224, 64), (64, 224, 64), (64, 112, 128), (128, 112, 128), (128, 56, 256),
                       (256, 56, 256), (256, 28, 512), (512, 28, 512), (512, 14, 512)]


def vgg16_imagenet(N: int = 128, dtype: str = "f32") -> Workload:
    """The nine distinct 3x3 layer shapes (C, H = W, K) of VGG-16 on 224x224 images that the
    paper's timing table lists, each at 90 % unified sparsity; independent layers."""
    return Workload(f"vgg16_224px_{dtype}", 9, N, dtype, "normal", [
        LayerSpec(f"{c}x{hw}x{hw}x{k}", C=c, K=k, R=3, S=3, H=hw, W=hw, stride=1, pad=1, sparsity_bp=9000)
        for (c, hw, k) in VGG_IMAGENET_LAYERS], chain=False)
