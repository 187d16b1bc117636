"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no quantisation, no indexing, no coding), so both the HIP
library's callers and the CPU oracle's callers may use it.

The paper evaluates on trained, pruned AlexNet and VGG-16 (Sec. V-A, Table I);
neither the weights nor ImageNet are available here, so every layer is a random
stand-in with the same shape, the same fraction of surviving weights and the same
bit widths (5-bit FC / 8-bit CONV value indices, 4-bit AlexNet / 5-bit VGG-16
relative indices).  Surviving weights are N(0, sigma); which weights survive is
an independent Bernoulli(density) draw per element, in line with the paper's
remark that the non-zeros are spread uniformly (Sec. IV-A).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 171100244


@dataclass(frozen=True)
class LayerSpec:
    name: str
    M: int                 # outputs (rows of W)
    K: int                 # inputs (columns of W)
    density: float
    sigma: float
    r: int                 # value-index bits
    k: int                 # relative-index bits
    conv: dict | None = None   # C,H,W,R,S,stride,pad,groups,OC for conv layers


def _seed(cfg: int, layer: int, extra: int = 0) -> int:
    return BASE_SEED + 1000 * cfg + layer + extra


def pruned_weights(M: int, K: int, density: float, sigma: float, seed: int) -> np.ndarray:
    """M x K fp32; pruned positions are exactly 0, survivors are never 0."""
    rng = np.random.Generator(np.random.PCG64(seed))
    W = rng.standard_normal((M, K), dtype=np.float32) * np.float32(sigma)
    keep = rng.random((M, K), dtype=np.float32) < np.float32(density)
    W[W == 0] = np.float32(sigma) * np.float32(1e-3)
    W *= keep
    W[~keep] = 0.0   # also clears -0.0
    return W


def relu_normal(shape, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.maximum(rng.standard_normal(shape, dtype=np.float32), 0).astype(np.float32)


def uniform01(shape, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.random(shape, dtype=np.float32)


def sparse_uniform01(shape, seed: int) -> np.ndarray:
    """U(0,1) with half of the entries zeroed (post-ReLU-like)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.random(shape, dtype=np.float32)
    return (x * (rng.random(shape, dtype=np.float32) < 0.5)).astype(np.float32)


def _conv(C, H, W, R, S, stride, pad, groups, OC):
    return dict(C=C, H=H, W=W, R=R, S=S, stride=stride, pad=pad, groups=groups, OC=OC)


# The five benchmark configurations (cfg numbers are 1-based as in the brief).
CONFIGS: dict[int, dict] = {
    1: dict(layers=[LayerSpec("fc1024", 1024, 1024, 0.10, 0.02, 5, 4)], batches=[1], act="sparse_uniform"),
    2: dict(layers=[LayerSpec("fc6", 4096, 9216, 0.09, 0.01, 5, 4)], batches=[1, 8], act="relu_normal"),
    3: dict(layers=[LayerSpec("fc6", 4096, 9216, 0.09, 0.01, 5, 4),
                    LayerSpec("fc7", 4096, 4096, 0.09, 0.01, 5, 4),
                    LayerSpec("fc8", 1000, 4096, 0.25, 0.01, 5, 4)],
            batches=[1, 4, 16, 64, 256], act="relu_normal"),
    4: dict(layers=[LayerSpec("conv1", 96, 363, 0.84, 0.01, 8, 8, _conv(3, 227, 227, 11, 11, 4, 0, 1, 96)),
                    LayerSpec("conv2", 256, 1200, 0.38, 0.01, 8, 8, _conv(96, 27, 27, 5, 5, 1, 2, 2, 256)),
                    LayerSpec("conv3", 384, 2304, 0.35, 0.01, 8, 8, _conv(256, 13, 13, 3, 3, 1, 1, 1, 384)),
                    LayerSpec("conv4", 384, 1728, 0.37, 0.01, 8, 8, _conv(384, 13, 13, 3, 3, 1, 1, 2, 384)),
                    LayerSpec("conv5", 256, 1728, 0.37, 0.01, 8, 8, _conv(384, 13, 13, 3, 3, 1, 1, 2, 256))],
            batches=[1, 16, 64], act="uniform"),
    5: dict(layers=[LayerSpec("vgg_fc6", 4096, 25088, 0.04, 0.01, 5, 5),
                    LayerSpec("vgg_fc7", 4096, 4096, 0.04, 0.01, 5, 5),
                    LayerSpec("vgg_fc8", 1000, 4096, 0.23, 0.01, 5, 5)],
            batches=[1, 2, 4, 8, 16, 32, 64, 128, 256], act="relu_normal"),
}


def _vgg16_conv_layers():
    """The thirteen 3 x 3 convolutions of VGG-16 on 224 x 224 inputs with the
    densities of Table I(b) (100 % minus the pruning percentage), 8-bit codebooks
    and the 5-bit relative index the paper uses for VGG-16 (Sec. VI)."""
    plan = [("conv1_1", 3, 224, 64, 0.58), ("conv1_2", 64, 224, 64, 0.22), ("conv2_1", 64, 112, 128, 0.34),
            ("conv2_2", 128, 112, 128, 0.36), ("conv3_1", 128, 56, 256, 0.53), ("conv3_2", 256, 56, 256, 0.24),
            ("conv3_3", 256, 56, 256, 0.42), ("conv4_1", 256, 28, 512, 0.32), ("conv4_2", 512, 28, 512, 0.27),
            ("conv4_3", 512, 28, 512, 0.34), ("conv5_1", 512, 14, 512, 0.35), ("conv5_2", 512, 14, 512, 0.29),
            ("conv5_3", 512, 14, 512, 0.36)]
    return [LayerSpec(n, oc, c * 9, d, 0.01, 8, 5, _conv(c, hw, hw, 3, 3, 1, 1, 1, oc)) for n, c, hw, oc, d in plan]


# beyond the five benchmark configurations: the VGG-16 convolutions (a "next" row)
CONFIGS[6] = dict(layers=_vgg16_conv_layers(), batches=[1, 8], act="uniform")


def layer_weights(cfg: int, layer_index: int, scale: float = 1.0,
                  density: float | None = None) -> tuple[LayerSpec, np.ndarray]:
    """Weights of one layer of a configuration.  scale < 1 shrinks both
    dimensions (rounded to a multiple of 8, at least 8) for quick tests; conv
    layers are not scaled.  density overrides the configuration's fraction of
    non-zeros (the uniform 70/80/90 % pruning levels of Sec. VI)."""
    spec = CONFIGS[cfg]["layers"][layer_index]
    if density is not None:
        spec = LayerSpec(spec.name, spec.M, spec.K, density, spec.sigma, spec.r, spec.k, spec.conv)
    M, K = spec.M, spec.K
    if scale != 1.0 and spec.conv is None:
        M = max(8, int(M * scale) // 8 * 8)
        K = max(8, int(K * scale) // 8 * 8)
        spec = LayerSpec(spec.name, M, K, spec.density, spec.sigma, spec.r, spec.k, None)
    return spec, pruned_weights(M, K, spec.density, spec.sigma, _seed(cfg, layer_index))


def activations(cfg: int, batch: int, K: int | None = None, layer_index: int = 0) -> np.ndarray:
    """Input of layer ``layer_index`` of a configuration: B x K (FC) or
    B x C x H x W (conv)."""
    c = CONFIGS[cfg]
    spec = c["layers"][layer_index]
    seed = _seed(cfg, layer_index, 500 + batch)
    if spec.conv is not None:
        g = spec.conv
        return uniform01((batch, g["C"], g["H"], g["W"]), seed)
    K = spec.K if K is None else K
    if c["act"] == "sparse_uniform":
        return sparse_uniform01((batch, K), seed)
    if c["act"] == "uniform":
        return uniform01((batch, K), seed)
    return relu_normal((batch, K), seed)


def poisson_arrivals(n: int, rate_per_s: float, seed: int) -> np.ndarray:
    """Arrival times (seconds, ascending) of n single-image requests."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.cumsum(rng.exponential(1.0 / rate_per_s, size=n))
