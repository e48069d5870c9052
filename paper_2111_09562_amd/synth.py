"""Seeded synthetic activation tensors with the shapes and statistics of the
workloads the codec is measured on.

This module only *generates inputs*.  It holds none of the codec's arithmetic
and is the one piece of code that both the CPU oracle's tests and the HIP
path's tests may share.  Everything is numpy on the host; results depend only
on (seed, shape, recipe), never on thread count.

Recipe "relu_blur" (post-BatchNorm-ReLU conv activations): i.i.d. N(0,1) field
-> k x k box blur inside every (n, c) plane (zero padding, divide by k*k) ->
standardise every channel over (N, H, W) -> * scale + shift -> ReLU.  With
shift -0.2 about 58 % of the values are exact zeros; the blur gives the spatial
correlation a Lorenzo predictor feeds on.

Recipe "relu_laplace" (heavy-tailed stress): i.i.d. Laplace(0, 1) -> ReLU,
no smoothing, about 50 % zeros.
"""
from __future__ import annotations

import numpy as np


def _box_blur_planes(a: np.ndarray, k: int) -> np.ndarray:
    """k x k box blur over the last two axes, zero padded, separable."""
    if k <= 1:
        return a
    r = k // 2
    h, w = a.shape[-2], a.shape[-1]
    pad = [(0, 0)] * (a.ndim - 2) + [(0, 0), (r, r)]
    p = np.pad(a, pad)
    acc = np.zeros_like(a)
    for j in range(k):
        acc += p[..., :, j:j + w]
    pad = [(0, 0)] * (a.ndim - 2) + [(r, r), (0, 0)]
    p = np.pad(acc, pad)
    out = np.zeros_like(a)
    for j in range(k):
        out += p[..., j:j + h, :]
    out *= np.float32(1.0 / (k * k))
    return out


def relu_blur(shape, seed: int, blur: int = 3, scale: float = 1.0, shift: float = -0.2) -> np.ndarray:
    """fp32 NCHW tensor following recipe "relu_blur"."""
    n, c, h, w = (int(s) for s in shape)
    rng = np.random.Generator(np.random.Philox(seed))
    x = np.empty((n, c, h, w), np.float32)
    # one sample at a time bounds the temporaries of the blur
    for i in range(n):
        z = rng.standard_normal((c, h, w), dtype=np.float32)
        x[i] = _box_blur_planes(z, blur)
    mean = x.mean(axis=(0, 2, 3), dtype=np.float64)
    var = np.zeros(c, np.float64)
    for i in range(n):
        d = x[i].astype(np.float64) - mean[:, None, None]
        var += (d * d).sum(axis=(1, 2))
    std = np.sqrt(var / float(n * h * w))
    std[std == 0.0] = 1.0
    a = (scale / std).astype(np.float32)[None, :, None, None]
    b = (shift - scale * mean / std).astype(np.float32)[None, :, None, None]
    for i in range(n):
        xi = x[i] * a[0] + b[0]
        np.maximum(xi, np.float32(0.0), out=xi)
        x[i] = xi
    return x


def relu_laplace(shape, seed: int) -> np.ndarray:
    """fp32 NCHW tensor following recipe "relu_laplace"."""
    n, c, h, w = (int(s) for s in shape)
    rng = np.random.Generator(np.random.Philox(seed))
    x = np.empty((n, c, h, w), np.float32)
    for i in range(n):
        z = rng.laplace(0.0, 1.0, (c, h, w)).astype(np.float32)
        np.maximum(z, np.float32(0.0), out=z)
        x[i] = z
    return x


# The workloads.  Each entry: list of (shape, seed, recipe kwargs, eb, nbins).
# Per-layer error bounds of the ResNet-50-shaped set are one fixed draw from
# {1e-3, 1e-2, 5e-2} that uses every value.

def config0():
    return [dict(shape=(8, 64, 56, 56), seed=0, recipe="relu_blur", blur=3, shift=-0.2, eb=1e-2, nbins=1024)]


def config1(batch: int = 64):
    shapes = [(batch, 64, 112, 112), (batch, 256, 56, 56), (batch, 512, 28, 28), (batch, 1024, 14, 14), (batch, 2048, 7, 7)]
    ebs = [1e-2, 1e-3, 5e-2, 1e-2, 1e-3]
    return [dict(shape=s, seed=1 + i, recipe="relu_blur", blur=3, shift=-0.2, eb=e, nbins=1024)
            for i, (s, e) in enumerate(zip(shapes, ebs))]


def config2(batch: int = 32):
    shapes = [(batch, 64, 224, 224), (batch, 128, 112, 112), (batch, 256, 56, 56), (batch, 512, 28, 28), (batch, 512, 14, 14)]
    return [dict(shape=s, seed=6 + i, recipe="relu_blur", blur=5, shift=0.0, eb=1e-2, nbins=4096)
            for i, s in enumerate(shapes)]


def config3(batch: int = 64):
    ebs = [10.0 ** (-4.0 + k / 2.0) for k in range(7)]
    bins = [65536, 32768, 16384, 4096, 1024, 1024, 1024]
    return [dict(shape=(batch, 256, 56, 56), seed=11, recipe="relu_blur", blur=3, shift=0.0, eb=e, nbins=b)
            for e, b in zip(ebs, bins)]


def config4(batch: int = 128):
    return [dict(shape=(batch, 64, 224, 224), seed=12 + i, recipe="relu_laplace", eb=1e-3, nbins=65536) for i in range(2)]


def make(entry: dict) -> np.ndarray:
    if entry["recipe"] == "relu_blur":
        return relu_blur(entry["shape"], entry["seed"], entry.get("blur", 3), 1.0, entry.get("shift", -0.2))
    if entry["recipe"] == "relu_laplace":
        return relu_laplace(entry["shape"], entry["seed"])
    raise ValueError(entry["recipe"])
