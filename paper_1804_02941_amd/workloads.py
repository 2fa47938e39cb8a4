"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws numbers: it holds none of the method's arithmetic (no
binarization, no estimation, no binary product) and is imported by the tests
and the benchmark, never by the library binding or by the CPU oracle.

The paper (arXiv 1804.02941, Section 5) trains on TU-Berlin and Sketchy
sketches; neither the datasets nor trained weights are available, so every
input here is a synthetic stand-in with the shapes of the paper's networks
(Sketch-A-Net, ResNet-18-style stages, wide fully-connected layers) and with
value distributions chosen to exercise the method: filters with non-zero mean
and skew give K != n/2 and alpha != -beta.

Arrays are float32; activations are NCHW, weights are [F, C, kh, kw].
Seeds: BASE + 10*config + {0: activations, 1: weights, 2: means / skews}.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 1804029410


@dataclass(frozen=True)
class Layer:
    """Shape of one binarized layer; a fully-connected layer has H=W=kh=kw=1."""
    name: str
    C: int
    H: int
    W: int
    F: int
    kh: int
    kw: int
    pad: int = 0
    stride: int = 1
    pool_after: bool = False   # 3x3 / stride-2 max-pool between this layer and the next

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def n(self):
        return self.C * self.kh * self.kw

    @property
    def is_fc(self):
        return self.H == 1 and self.W == 1 and self.kh == 1 and self.kw == 1

    def macs(self, B):
        """Effective binary multiply-accumulates of one forward pass (padded taps counted)."""
        return B * self.Ho * self.Wo * self.F * self.n


def _rng(cfg, stream):
    return np.random.default_rng(BASE_SEED + 10 * cfg + stream)


def skewed_mixture_weights(rng_w, rng_s, F, n, fan_in):
    """Rows from 0.7*N(+0.3 d, s0) + 0.3*N(-0.7 d, s0), s0 = sqrt(2/fan_in), d = 2 s0 U(-1,1)."""
    s0 = np.sqrt(2.0 / fan_in)
    d = 2.0 * s0 * rng_s.uniform(-1.0, 1.0, size=(F, 1))
    pick = rng_w.random((F, n)) < 0.7
    centre = np.where(pick, 0.3 * d, -0.7 * d)
    return (centre + s0 * rng_w.standard_normal((F, n))).astype(np.float32)


# ---------------------------------------------------------------- config 1
CFG1 = Layer("cfg1_conv3x3", C=64, H=16, W=16, F=64, kh=3, kw=3, pad=1)


def config1(batch=1):
    """Tiny single layer: half-normal activations, N(mu_f, 0.05) filters."""
    L = CFG1
    x = np.abs(_rng(1, 0).standard_normal((batch, L.C, L.H, L.W))).astype(np.float32)
    mu = _rng(1, 2).uniform(-0.02, 0.02, size=(L.F, 1))
    w = (mu + 0.05 * _rng(1, 1).standard_normal((L.F, L.n))).astype(np.float32)
    return L, x, w.reshape(L.F, L.C, L.kh, L.kw)


# ---------------------------------------------------------------- config 2
CFG2 = Layer("cfg2_sketchanet_conv2", C=64, H=35, W=35, F=128, kh=5, kw=5)


def config2(batch=128):
    """Sketch-A-Net conv2 shape: ReLU(N(0,1)) activations, Laplacian filters."""
    L = CFG2
    x = np.maximum(_rng(2, 0).standard_normal((batch, L.C, L.H, L.W)), 0).astype(np.float32)
    m = _rng(2, 2).uniform(-0.01, 0.01, size=(L.F, 1))
    w = (m + _rng(2, 1).laplace(0.0, 0.03, size=(L.F, L.n))).astype(np.float32)
    return L, x, w.reshape(L.F, L.C, L.kh, L.kw)


# ---------------------------------------------------------------- config 3
CFG3_LAYERS = (
    Layer("conv2", C=64, H=35, W=35, F=128, kh=5, kw=5, pool_after=True),
    Layer("conv3", C=128, H=15, W=15, F=256, kh=3, kw=3, pad=1),
    Layer("conv4", C=256, H=15, W=15, F=256, kh=3, kw=3, pad=1),
    Layer("conv5", C=256, H=15, W=15, F=256, kh=3, kw=3, pad=1, pool_after=True),
    Layer("conv6", C=256, H=7, W=7, F=512, kh=7, kw=7),
    Layer("fc7", C=512, H=1, W=1, F=512, kh=1, kw=1),
)


def sketch_images(batch, size=225, seed_stream=0):
    """White images with black 3-px polylines covering 5-10 % of the pixels."""
    rng = _rng(3, seed_stream)
    imgs = np.ones((batch, 1, size, size), dtype=np.float32)
    for b in range(batch):
        while True:
            ink = np.zeros((size, size), dtype=bool)
            while ink.mean() < 0.05:
                nv = int(rng.integers(3, 9))
                pts = rng.uniform(4, size - 5, size=(nv, 2))
                for (y0, x0), (y1, x1) in zip(pts[:-1], pts[1:]):
                    steps = int(2 * max(abs(y1 - y0), abs(x1 - x0))) + 2
                    t = np.linspace(0.0, 1.0, steps)
                    ys = np.rint(y0 + t * (y1 - y0)).astype(int)
                    xs = np.rint(x0 + t * (x1 - x0)).astype(int)
                    for dy in (-1, 0, 1):
                        for dx in (-1, 0, 1):
                            ink[ys + dy, xs + dx] = True
            if ink.mean() <= 0.10:
                break
        imgs[b, 0][ink] = 0.0
    return imgs


def config3_weights():
    """He-scaled Gaussian filters for conv1 (kept fp32) and the six binarized layers."""
    rng = _rng(3, 1)
    w1 = (np.sqrt(2.0 / 225.0) * rng.standard_normal((64, 1, 15, 15))).astype(np.float32)
    ws = []
    for L in CFG3_LAYERS:
        w = np.sqrt(2.0 / L.n) * rng.standard_normal((L.F, L.C, L.kh, L.kw))
        ws.append(w.astype(np.float32))
    return w1, ws


def config3_conv1_features(images, w1, device="cpu"):
    """Input of conv2: fp32 conv1 15x15 / 3, ReLU, 3x3 / 2 max-pool -> [B, 64, 35, 35].

    conv1 is not binarized in the paper's Sketch-A-Net (Section 5.1), so this is
    ordinary fp32 arithmetic and part of input preparation.
    """
    import torch
    import torch.nn.functional as Fn
    x = torch.from_numpy(np.ascontiguousarray(images)).to(device)
    w = torch.from_numpy(np.ascontiguousarray(w1)).to(device)
    out = []
    for i in range(0, x.shape[0], 32):
        y = Fn.max_pool2d(Fn.relu(Fn.conv2d(x[i:i + 32], w, stride=3)), 3, 2)
        out.append(y)
    return torch.cat(out)


# ---------------------------------------------------------------- config 4
CFG4_LAYERS = tuple(
    Layer(f"stage{i + 1}_{c}x{s}x{s}", C=c, H=s, W=s, F=c, kh=3, kw=3, pad=1)
    for i, (c, s) in enumerate(((64, 56), (128, 28), (256, 14), (512, 7)))
)


def config4(stage, batch=64):
    """ResNet-18-style 3x3 stage: N(0,1) activations, skewed two-Gaussian filters."""
    L = CFG4_LAYERS[stage]
    rng_x = np.random.default_rng(BASE_SEED + 40 + 0 + 100 * (stage + 1))
    rng_w = np.random.default_rng(BASE_SEED + 40 + 1 + 100 * (stage + 1))
    rng_s = np.random.default_rng(BASE_SEED + 40 + 2 + 100 * (stage + 1))
    x = rng_x.standard_normal((batch, L.C, L.H, L.W)).astype(np.float32)
    w = skewed_mixture_weights(rng_w, rng_s, L.F, L.n, L.n)
    return L, x, w.reshape(L.F, L.C, L.kh, L.kw)


# ---------------------------------------------------------------- config 5
CFG5_LAYERS = (
    Layer("fc_9216_4096", C=9216, H=1, W=1, F=4096, kh=1, kw=1),
    Layer("fc_4096_4096", C=4096, H=1, W=1, F=4096, kh=1, kw=1),
)


def config5(which, batch=1024, filters=None):
    """Wide fully-connected layer: N(0,1) inputs, skewed two-Gaussian rows.

    ``filters`` limits the number of rows generated (the leading rows of the
    full matrix are not reproduced; a reduced problem is its own draw).
    """
    L = CFG5_LAYERS[which]
    F = L.F if filters is None else filters
    rng_x = np.random.default_rng(BASE_SEED + 50 + 0 + 100 * (which + 1))
    rng_w = np.random.default_rng(BASE_SEED + 50 + 1 + 100 * (which + 1))
    rng_s = np.random.default_rng(BASE_SEED + 50 + 2 + 100 * (which + 1))
    x = rng_x.standard_normal((batch, L.C)).astype(np.float32)
    w = skewed_mixture_weights(rng_w, rng_s, F, L.n, L.n)
    if filters is not None:
        L = Layer(L.name + f"_F{F}", C=L.C, H=1, W=1, F=F, kh=1, kw=1)
    return L, x, w.reshape(F, L.C, 1, 1)


def nchw_to_nhwc(x):
    """Contiguous channel-last copy of an NCHW array (pure data movement)."""
    return np.ascontiguousarray(np.transpose(x, (0, 2, 3, 1)))
