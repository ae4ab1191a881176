"""Seeded synthetic layers: the five benchmark configurations and their input recipes.

This module holds shapes and random-number recipes only -- none of the method's arithmetic -- so
that the GPU path and the CPU oracle can both be fed from it without sharing any computation.
The paper times unspecified single-channel images (Sec. IV); the layer shapes below are the
CNN-layer workloads this build is measured on, with synthetic values in place of any dataset or
trained weights.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED_BASE = 20200714 * 10


@dataclass(frozen=True)
class Layer:
    """One convolution layer: I[N][C][H][W], Wt[F][C][kh][kw], stride (sh, sw), zero pad (ph, pw)."""
    name: str
    config: int          # 1-based index of the benchmark configuration it belongs to
    N: int
    C: int
    H: int
    W: int
    F: int
    kh: int
    kw: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0
    input_dist: str = "normal"     # "normal" N(0,1) | "uniform" U[-1,1] | "normal_zeros" (5 % exact +0.0)
    weight_std: float = 1.0        # weights ~ N(0, weight_std)

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.ph - self.kh) // self.sh + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pw - self.kw) // self.sw + 1

    @property
    def n_red(self) -> int:
        return self.C * self.kh * self.kw

    @property
    def binary_macs(self) -> int:
        return self.N * self.F * self.OH * self.OW * self.n_red

    def with_batch(self, n: int) -> "Layer":
        return replace(self, N=n)


def _sq(name, config, N, C, HW, F, k, stride=1, pad=None, **kw) -> Layer:
    pad = k // 2 if pad is None else pad
    return Layer(name, config, N, C, HW, HW, F, k, k, stride, stride, pad, pad, **kw)


LAYERS = {
    # config 1: small single layer the oracle finishes in seconds
    "c1": _sq("c1", 1, 1, 64, 32, 64, 3),
    # config 2: kernel-size sweep
    "c2_k3": _sq("c2_k3", 2, 16, 128, 56, 128, 3),
    "c2_k5": _sq("c2_k5", 2, 16, 128, 56, 128, 5),
    "c2_k7": _sq("c2_k7", 2, 16, 128, 56, 128, 7),
    # config 3: ResNet-18-shaped stage (+ stride-2 variant)
    "c3_s1": _sq("c3_s1", 3, 64, 256, 14, 256, 3, weight_std=0.05),
    "c3_s2": _sq("c3_s2", 3, 64, 128, 28, 256, 3, stride=2, weight_std=0.05),
    # config 4: AlexNet-shaped binary layers
    "c4_conv2": _sq("c4_conv2", 4, 128, 96, 27, 256, 5, input_dist="uniform"),
    "c4_conv3": _sq("c4_conv3", 4, 128, 256, 13, 384, 3, input_dist="uniform"),
    "c4_conv4": _sq("c4_conv4", 4, 128, 384, 13, 384, 3, input_dist="uniform"),
    "c4_conv5": _sq("c4_conv5", 4, 128, 384, 13, 256, 3, input_dist="uniform"),
    # config 5: large-channel layer (5 % exact zeros exercise sign(0) = +1)
    "c5": _sq("c5", 5, 128, 512, 28, 512, 3, input_dist="normal_zeros"),
}


def make_input(layer: Layer, n_images: int | None = None) -> np.ndarray:
    """fp32 I[N][C][H][W].  Images are generated in order from one stream, so the first
    ``n_images`` images of a layer are the same arrays whatever N is asked for."""
    n = layer.N if n_images is None else n_images
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + layer.config))
    out = np.empty((n, layer.C, layer.H, layer.W), dtype=np.float32)
    for i in range(n):
        shape = (layer.C, layer.H, layer.W)
        if layer.input_dist == "uniform":
            img = rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
        else:
            img = rng.standard_normal(size=shape, dtype=np.float32)
            if layer.input_dist == "normal_zeros":
                img[rng.random(shape) < 0.05] = 0.0
        out[i] = img
    return out


def make_weights(layer: Layer) -> np.ndarray:
    """fp32 Wt[F][C][kh][kw] ~ N(0, weight_std)."""
    # the name enters the seed so that the layers of one configuration get different filters
    salt = sum(ord(ch) for ch in layer.name)
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + layer.config + 100 + 1000 * salt))
    w = rng.standard_normal(size=(layer.F, layer.C, layer.kh, layer.kw), dtype=np.float32)
    return (w * np.float32(layer.weight_std)).astype(np.float32)


def random_layer(rng: np.random.Generator, name: str, N, C, H, W, F, kh, kw, sh=1, sw=1, ph=0, pw=0):
    """Arbitrary-shape test case with N(0,1) data and a sprinkling of +0.0 / -0.0 / denormals."""
    layer = Layer(name, 0, N, C, H, W, F, kh, kw, sh, sw, ph, pw)
    I = rng.standard_normal(size=(N, C, H, W), dtype=np.float32)
    Wt = rng.standard_normal(size=(F, C, kh, kw), dtype=np.float32)
    for arr in (I, Wt):
        flat = arr.reshape(-1)
        k = max(1, flat.size // 16)
        idx = rng.integers(0, flat.size, size=k)
        flat[idx[0::3]] = 0.0
        flat[idx[1::3]] = -0.0
        flat[idx[2::3]] = np.float32(1e-41) * np.where(rng.random(idx[2::3].size) < 0.5, -1, 1)
    return layer, I, Wt
