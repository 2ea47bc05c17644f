"""Seeded synthetic inputs and layer-shape tables for tests and benchmarks.

Holds no arithmetic of the quantized backward pass: only random tensors with
the shapes, value distributions and tail behaviour of the workloads named in
the paper (Sec. 4.1: ResNet-20 on CIFAR-100 at batch 128, ResNet-18/34/50 on
ImageNet, EDSR on DIV2K at batch 16) and layer tables of those networks.  The
paper describes layer gradients as zero-centred with most mass near zero and a
very long, sparse tail (Sec. 3.3); the recipes below reproduce that with
Student-t, Laplace-plus-outliers and Gaussian-plus-spikes draws.

Every tensor is drawn in double with numpy's PCG64 seeded by
``[seed, config, layer, tensor, iteration]`` and cast once to fp32; the same
fp32 bits go to the CPU oracle and to the GPU library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

T_X, T_W, T_DY = 0, 1, 2


def rng(seed: int, cfg: int, layer: int, tensor: int, it: int = 0) -> np.random.Generator:
    return np.random.default_rng([seed, cfg, layer, tensor, it])


def normal(r, shape, std=1.0):
    return (r.standard_normal(shape) * std).astype(np.float32)


def relu_normal(r, shape):
    return np.maximum(r.standard_normal(shape), 0.0).astype(np.float32)


def kaiming_normal(r, w_shape):
    fan_in = int(np.prod(w_shape[1:]))
    return (r.standard_normal(w_shape) * np.sqrt(2.0 / fan_in)).astype(np.float32)


def student_t(r, shape, nu, scale):
    return (r.standard_t(nu, shape) * scale).astype(np.float32)


def laplace_outliers(r, shape, b=1e-4, frac=1e-3, mult=50.0):
    g = r.laplace(0.0, b, shape)
    mask = r.random(shape) < frac
    return np.where(mask, g * mult, g).astype(np.float32)


def gauss_spikes(r, shape, std=1e-4, frac=1e-4, mult=100.0):
    g = r.standard_normal(shape) * std
    mask = r.random(shape) < frac
    return np.where(mask, g * mult, g).astype(np.float32)


@dataclass(frozen=True)
class ConvLayer:
    name: str
    count: int      # occurrences of this shape in the network
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self):
        return (self.K, self.C, self.R, self.S)

    @property
    def dy_shape(self):
        return (self.N, self.K, self.P, self.Q)

    @property
    def gemm_ops(self):
        """2*M*N*K of each of the two implicit GEMMs (padding taps counted)."""
        return 2 * self.N * self.P * self.Q * self.K * self.C * self.R * self.S


@dataclass(frozen=True)
class LinearLayer:
    name: str
    count: int
    M: int
    K: int     # in features
    N: int     # out features

    @property
    def gemm_ops(self):
        return 2 * self.M * self.K * self.N


def _c(name, count, n, c, h, k, r, stride):
    return ConvLayer(name, count, n, c, h, h, k, r, r, stride, (r - 1) // 2)


def resnet50_layers(batch: int = 64):
    """Bottleneck convolutions of ResNet-50 (stride on the 3x3) plus the classifier."""
    b = batch
    return [
        _c("l1.1x1.64-64@56", 1, b, 64, 56, 64, 1, 1),
        _c("l1.3x3.64-64@56", 3, b, 64, 56, 64, 3, 1),
        _c("l1.1x1.64-256@56", 4, b, 64, 56, 256, 1, 1),
        _c("l1.1x1.256-64@56", 2, b, 256, 56, 64, 1, 1),
        _c("l2.1x1.256-128@56", 1, b, 256, 56, 128, 1, 1),
        _c("l2.3x3s2.128-128@56", 1, b, 128, 56, 128, 3, 2),
        _c("l2.1x1.128-512@28", 4, b, 128, 28, 512, 1, 1),
        _c("l2.ds1x1s2.256-512@56", 1, b, 256, 56, 512, 1, 2),
        _c("l2.1x1.512-128@28", 3, b, 512, 28, 128, 1, 1),
        _c("l2.3x3.128-128@28", 3, b, 128, 28, 128, 3, 1),
        _c("l3.1x1.512-256@28", 1, b, 512, 28, 256, 1, 1),
        _c("l3.3x3s2.256-256@28", 1, b, 256, 28, 256, 3, 2),
        _c("l3.1x1.256-1024@14", 6, b, 256, 14, 1024, 1, 1),
        _c("l3.ds1x1s2.512-1024@28", 1, b, 512, 28, 1024, 1, 2),
        _c("l3.1x1.1024-256@14", 5, b, 1024, 14, 256, 1, 1),
        _c("l3.3x3.256-256@14", 5, b, 256, 14, 256, 3, 1),
        _c("l4.1x1.1024-512@14", 1, b, 1024, 14, 512, 1, 1),
        _c("l4.3x3s2.512-512@14", 1, b, 512, 14, 512, 3, 2),
        _c("l4.1x1.512-2048@7", 3, b, 512, 7, 2048, 1, 1),
        _c("l4.ds1x1s2.1024-2048@14", 1, b, 1024, 14, 2048, 1, 2),
        _c("l4.1x1.2048-512@7", 2, b, 2048, 7, 512, 1, 1),
        _c("l4.3x3.512-512@7", 2, b, 512, 7, 512, 3, 1),
        LinearLayer("fc.2048-1000", 1, b, 2048, 1000),
    ]


def resnet18_layers(batch: int = 64):
    b = batch
    return [
        ConvLayer("stem.7x7s2.3-64@224", 1, b, 3, 224, 224, 64, 7, 7, 2, 3),
        _c("l1.3x3.64-64@56", 4, b, 64, 56, 64, 3, 1),
        _c("l2.3x3s2.64-128@56", 1, b, 64, 56, 128, 3, 2),
        _c("l2.ds1x1s2.64-128@56", 1, b, 64, 56, 128, 1, 2),
        _c("l2.3x3.128-128@28", 3, b, 128, 28, 128, 3, 1),
        _c("l3.3x3s2.128-256@28", 1, b, 128, 28, 256, 3, 2),
        _c("l3.ds1x1s2.128-256@28", 1, b, 128, 28, 256, 1, 2),
        _c("l3.3x3.256-256@14", 3, b, 256, 14, 256, 3, 1),
        _c("l4.3x3s2.256-512@14", 1, b, 256, 14, 512, 3, 2),
        _c("l4.ds1x1s2.256-512@14", 1, b, 256, 14, 512, 1, 2),
        _c("l4.3x3.512-512@7", 3, b, 512, 7, 512, 3, 1),
        LinearLayer("fc.512-1000", 1, b, 512, 1000),
    ]


def cifar_layers(batch: int = 128):
    """3x3 residual-block convolutions of a CIFAR ResNet-20."""
    return [
        _c("s1.3x3.16-16@32", 6, batch, 16, 32, 16, 3, 1),
        _c("s2.3x3.32-32@16", 5, batch, 32, 16, 32, 3, 1),
        _c("s3.3x3.64-64@8", 5, batch, 64, 8, 64, 3, 1),
    ]


def sr_layers(batch: int = 16, patch: int = 96):
    """EDSR-shaped layers: head, residual body, x4 pixel-shuffle tail conv."""
    return [
        _c("head.3x3.3-64", 1, batch, 3, patch, 64, 3, 1),
        _c("body.3x3.64-64", 64, batch, 64, patch, 64, 3, 1),
        _c("tail.3x3.64-256", 1, batch, 64, patch, 256, 3, 1),
    ]


def vit_l_layers(batch: int = 64, tokens: int = 197):
    """Linear layers of one ViT-L/16 encoder block (width 1024, MLP 4096) at batch x tokens
    rows; the network has 24 such blocks.  ViT-L is the transformer of the paper's
    supplement (Table C); the attention products themselves are not linear layers and are
    not part of the sweep."""
    m = batch * tokens
    return [
        LinearLayer("vit.qkv.1024-3072", 1, m, 1024, 3072),
        LinearLayer("vit.proj.1024-1024", 1, m, 1024, 1024),
        LinearLayer("vit.fc1.1024-4096", 1, m, 1024, 4096),
        LinearLayer("vit.fc2.4096-1024", 1, m, 4096, 1024),
    ]


def linear_case():
    return LinearLayer("linear.512-512", 1, 256, 512, 512)


# gradient recipes per workload -------------------------------------------------
def grad_cfg1(r, shape):
    return student_t(r, shape, 3.0, 1e-3)


def grad_cfg2(r, shape, scale=1e-4):
    return laplace_outliers(r, shape, scale, 1e-3, 50.0)


def grad_cfg4(r, shape):
    return student_t(r, shape, 2.5, 1e-3)


def grad_cfg5(r, shape):
    return gauss_spikes(r, shape, 1e-4, 1e-4, 100.0)


def dense_grad(r, shape, scale=1e-3):
    """Control case: uniform over the whole interval, so all 15 codes occur."""
    return (r.uniform(-1.0, 1.0, shape) * scale).astype(np.float32)
