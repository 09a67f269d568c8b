"""Seeded synthetic inputs with the shapes of the paper's workloads.

This module holds no arithmetic of the method: it only names layer shapes and
draws tensors.  It is the one module that both the HIP path's tests/bench and
the CPU oracle's tests use, so that both sides see the same bytes.  All tensors
are generated once on the host as fp32 numpy arrays (numpy's PCG64 stream,
``default_rng(seed + offset)`` with one fixed offset per tensor role).

The layer shapes are CaffeNet's convolutional layers (the paper's benchmark
network, Sec. 3.1: n in [13, 227], k in [3, 11], d in [3, 384]); ImageNet
images and trained weights are replaced by the distributions listed per
workload below.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Layer:
    """One convolutional layer problem (NCHW input, O x C/groups x K x K kernels)."""
    name: str
    N: int
    C: int
    H: int
    W: int
    O: int
    K: int
    stride: int = 1
    pad: int = 0
    groups: int = 1
    x_dist: str = "uniform"      # "uniform" = U[-1,1]; "relu_normal" = max(0, N(0,1))
    w_std: float = 0.01
    bias_std: float = 0.0        # 0 -> zero bias

    @property
    def Hout(self) -> int:
        return (self.H + 2 * self.pad - self.K) // self.stride + 1

    @property
    def Wout(self) -> int:
        return (self.W + 2 * self.pad - self.K) // self.stride + 1

    @property
    def flops(self) -> int:
        """Algorithmic flops of ONE pass (forward, backward-data or backward-weights)."""
        return 2 * self.N * self.O * self.Hout * self.Wout * (self.C // self.groups) * self.K ** 2

    def with_batch(self, N: int) -> "Layer":
        return replace(self, N=N)


def small_case() -> Layer:
    """The small forward-only configuration (batch 4, 3x32x32, 16 kernels of 5x5, pad 2)."""
    return Layer("cfg1", 4, 3, 32, 32, 16, 5, 1, 2, 1, "uniform", 0.05, 0.1)


def caffenet(N: int = 256):
    """CaffeNet conv1..conv5 at batch N."""
    return [
        Layer("conv1", N, 3, 227, 227, 96, 11, 4, 0, 1, "uniform", 0.01, 0.0),
        Layer("conv2", N, 96, 27, 27, 256, 5, 1, 2, 2, "relu_normal", 0.01, 0.0),
        Layer("conv3", N, 256, 13, 13, 384, 3, 1, 1, 1, "relu_normal", 0.01, 0.0),
        Layer("conv4", N, 384, 13, 13, 384, 3, 1, 1, 2, "relu_normal", 0.01, 0.0),
        Layer("conv5", N, 384, 13, 13, 256, 3, 1, 1, 2, "relu_normal", 0.01, 0.0),
    ]


def tradeoff_sweep(N: int = 128, HW: int = 28):
    """Lowering trade-off sweep (Appendix A): vary #input / #output channels, k in {1, 3}."""
    out = []
    for K, pad in ((1, 0), (3, 1)):
        for C, O in ((16, 512), (64, 256), (256, 256), (256, 64), (512, 16), (1024, 32)):
            out.append(Layer("sweep_k%d_c%d_o%d" % (K, C, O), N, C, HW, HW, O, K, 1, pad, 1,
                             "uniform", 0.01, 0.0))
    return out


_OFF_X, _OFF_W, _OFF_B, _OFF_DY = 0, 1, 2, 3


def make_x(L: Layer, seed: int = 0) -> np.ndarray:
    rng = np.random.default_rng(seed * 16 + _OFF_X)
    shape = (L.N, L.C, L.H, L.W)
    if L.x_dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if L.x_dist == "relu_normal":
        return np.maximum(rng.standard_normal(size=shape, dtype=np.float32), np.float32(0))
    raise ValueError(L.x_dist)


def make_w(L: Layer, seed: int = 0) -> np.ndarray:
    rng = np.random.default_rng(seed * 16 + _OFF_W)
    shape = (L.O, L.C // L.groups, L.K, L.K)
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(L.w_std))


def make_bias(L: Layer, seed: int = 0) -> np.ndarray:
    if L.bias_std == 0.0:
        return np.zeros((L.O,), np.float32)
    rng = np.random.default_rng(seed * 16 + _OFF_B)
    return rng.standard_normal(size=(L.O,), dtype=np.float32) * np.float32(L.bias_std)


def make_dy(L: Layer, seed: int = 0) -> np.ndarray:
    """Upstream gradient ~ N(0,1) with the shape of the layer's output."""
    rng = np.random.default_rng(seed * 16 + _OFF_DY)
    return rng.standard_normal(size=(L.N, L.O, L.Hout, L.Wout), dtype=np.float32)


def sample_indices(total: int, count: int, seed: int = 0) -> np.ndarray:
    """Sorted distinct linear indices into a tensor of `total` elements (always with 0 and total-1)."""
    rng = np.random.default_rng(seed * 16 + 7)
    count = min(count, total)
    idx = rng.choice(total, size=count, replace=False) if total < (1 << 24) else \
        np.unique(rng.integers(0, total, size=count))
    idx = np.unique(np.concatenate([idx, [0, total - 1]])).astype(np.int64)
    return idx
