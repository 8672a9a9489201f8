"""Seeded synthetic gradients with the shapes of the paper's workloads.

This module holds NO codec arithmetic: it only draws numbers.  It is the one
piece shared by the GPU tests/bench and the CPU oracle tests, so both sides see
identical inputs.  The paper trains AlexNet on ImageNet and a CIFAR ResNet
(Sec. 4, "Training setup") and shows near-zero-peaked gradient histograms
(Sec. 3.1, Fig. 4); those gradients are not available offline, so per-tensor
Laplace / Gaussian / Student-t draws of the same tensor shapes stand in.

Every generator is `numpy.random.Generator(PCG64(SEED0 + config index))`; the
per-tensor scale is drawn first (log-uniform), then the values, tensor by tensor.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

SEED0 = 1811_08596


@dataclass
class Workload:
    name: str
    grad: np.ndarray                      # flat float32
    chunk_len: Optional[int]              # None => per-tensor (segmented) transform
    theta: float                          # KEPT fraction
    bits: int
    seg_offsets: np.ndarray               # tensor boundaries, len = tensors + 1
    thetas: List[float] = field(default_factory=list)   # sweep / schedule, if any


def _rng(idx: int, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(SEED0 + idx + 1000 * extra))


def _offsets(sizes) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))]).astype(np.int64)


def _log_uniform(rng, lo, hi):
    return float(np.exp(rng.uniform(np.log(lo), np.log(hi))))


def _fill(rng, sizes, draw, lo, hi) -> np.ndarray:
    out = np.empty(int(sum(sizes)), dtype=np.float32)
    pos = 0
    for s in sizes:
        scale = _log_uniform(rng, lo, hi)
        out[pos:pos + s] = draw(rng, scale, s).astype(np.float32)
        pos += s
    return out


# ----------------------------------------------------------------- shapes ---
def resnet20_sizes() -> List[int]:
    """CIFAR ResNet-20: 19 3x3 convs, FC 64x10 + bias, all BN scale/shift as one vector (22 tensors)."""
    sizes = [16 * 3 * 9]
    cin = 16
    bn = 16
    for cout in (16, 32, 64):
        for _ in range(3):
            sizes.append(cout * cin * 9)
            sizes.append(cout * cout * 9)
            cin = cout
            bn += 2 * cout
    sizes += [64 * 10, 10, 2 * bn]
    return sizes


def alexnet_sizes() -> List[int]:
    w = [96 * 3 * 11 * 11, 256 * 96 * 5 * 5, 384 * 256 * 9, 384 * 384 * 9, 256 * 384 * 9,
         4096 * 9216, 4096 * 4096, 1000 * 4096]
    b = [96, 256, 384, 384, 256, 4096, 4096, 1000]
    return w + b


def resnet50_sizes() -> List[int]:
    """53 convs each followed by BN scale and BN shift, then FC 2048x1000 + bias (161 tensors)."""
    sizes: List[int] = []

    def conv_bn(cout, cin, k):
        sizes.extend([cout * cin * k * k, cout, cout])

    conv_bn(64, 3, 7)
    cin = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            conv_bn(width, cin, 1)
            conv_bn(width, width, 3)
            conv_bn(4 * width, width, 1)
            if b == 0:
                conv_bn(4 * width, cin, 1)     # projection shortcut
            cin = 4 * width
    sizes += [2048 * 1000, 1000]
    return sizes


def vgg16_sizes() -> List[int]:
    cfg = [(64, 3), (64, 64), (128, 64), (128, 128), (256, 128), (256, 256), (256, 256),
           (512, 256), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
    w = [co * ci * 9 for co, ci in cfg] + [25088 * 4096, 4096 * 4096, 4096 * 1000]
    b = [co for co, _ in cfg] + [4096, 4096, 1000]
    return w + b


# ---------------------------------------------------------------- configs ---
def config1() -> Workload:
    rng = _rng(1)
    g = (rng.standard_normal(65536) * 1e-3).astype(np.float32)
    return Workload("gauss-64k", g, 1 << 16, 0.25, 8, _offsets([65536]))


def config2() -> Workload:
    rng = _rng(2)
    sizes = resnet20_sizes()
    g = _fill(rng, sizes, lambda r, b, s: r.laplace(0.0, b, s), 1e-5, 1e-2)
    return Workload("resnet20-shaped", g, 1 << 16, 0.5, 8, _offsets(sizes))


def config3(limit_elems: Optional[int] = None) -> Workload:
    rng = _rng(3)
    sizes = alexnet_sizes()
    g = _fill(rng, sizes, lambda r, b, s: r.laplace(0.0, b, s), 1e-5, 1e-2)
    if limit_elems is not None:
        g = g[:limit_elems]
    return Workload("alexnet-shaped", g, 1 << 20, 0.5, 8, _offsets(sizes), thetas=[0.1, 0.3, 0.5, 0.7, 0.9])


def config4() -> Workload:
    rng = _rng(4)
    sizes = resnet50_sizes()
    g = _fill(rng, sizes, lambda r, sd, s: r.standard_normal(s) * sd, 1e-6, 1e-2)
    return Workload("resnet50-shaped", g, None, 0.3, 6, _offsets(sizes))


def config5(iteration: int = 0) -> Workload:
    """VGG-16-shaped; a fresh draw per iteration, kept fraction falling linearly 0.9 -> 0.1 over 10 iterations."""
    rng = _rng(5, extra=iteration)
    sizes = vgg16_sizes()

    def draw(r, _scale, s):
        v = r.standard_t(3.0, s) * 1e-4
        v[r.random(s) < 1e-3] = 0.0
        return v

    g = _fill(rng, sizes, draw, 1.0, 1.0)
    thetas = [0.9 - i * (0.8 / 9.0) for i in range(10)]
    return Workload("vgg16-shaped", g, 1 << 22, thetas[iteration], 8, _offsets(sizes), thetas=thetas)


def small_mixed(n: int, seed: int = 7, zeros: float = 0.0) -> np.ndarray:
    """Small Laplace vector with a few decades of per-block scale; for unit tests."""
    rng = np.random.Generator(np.random.PCG64(SEED0 + 100 + seed))
    g = np.empty(n, dtype=np.float32)
    pos = 0
    while pos < n:
        s = int(min(n - pos, rng.integers(1, max(2, n // 3))))
        g[pos:pos + s] = rng.laplace(0.0, _log_uniform(rng, 1e-5, 1e-2), s).astype(np.float32)
        pos += s
    if zeros > 0:
        g[rng.random(n) < zeros] = 0.0
    return g
