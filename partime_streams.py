"""Seeded synthetic workloads: network shapes, initial weights, streams, targets.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds none of the method's arithmetic: it only draws inputs
(numpy ``Generator(PCG64(seed))``, generated in fp64, cast once to fp32) and
names the workload shapes.  The streams stand in for the paper's visual
streams (Sec. V), which are not available: what they keep is the property the
method relies on (Sec. III, remark after Eq. 8): consecutive samples differ
little.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

# integer codes used in layer records (kind / activation / loss / weight type)
DENSE, CONV3X3, GAP_DENSE = 0, 1, 2
ACT_ID, ACT_RELU, ACT_GELU = 0, 1, 2
LOSS_NONE, LOSS_MSE, LOSS_CE = 0, 1, 2
W_F32, W_BF16 = 0, 1


@dataclass
class LayerSpec:
    kind: int = DENSE
    act: int = ACT_ID
    in_dim: int = 0
    out_dim: int = 0
    c_in: int = 0
    c_out: int = 0
    h: int = 0
    w: int = 0
    skip_from: int = -1   # index of the layer whose output is added to this layer's output (-1: none)

    @property
    def w_shape(self):
        if self.kind == DENSE:
            return (self.out_dim, self.in_dim)
        if self.kind == CONV3X3:
            return (self.c_out, self.c_in, 3, 3)
        return (self.out_dim, self.c_in)

    @property
    def b_shape(self):
        return (self.c_out,) if self.kind == CONV3X3 else (self.out_dim,)

    @property
    def fan_in(self):
        return self.c_in * 9 if self.kind == CONV3X3 else (self.in_dim if self.kind == DENSE else self.c_in)

    @property
    def in_size(self):
        return self.in_dim if self.kind == DENSE else self.c_in * self.h * self.w

    @property
    def out_size(self):
        return self.c_out * self.h * self.w if self.kind == CONV3X3 else self.out_dim


@dataclass
class Workload:
    name: str
    layers: List[LayerSpec]
    n_streams: int = 1
    w_dtype: int = W_F32
    loss: int = LOSS_MSE
    lr: float = 1e-3
    ticks: int = 1000
    drift: float = 0.01
    seed: int = 0
    target_delay: Optional[int] = None   # None -> depth-1 (sample-aligned targets)
    balance: Optional[List[int]] = None  # None -> one layer per stage
    n_classes: int = 0
    replay: bool = False                 # the streams are the slots of a sliding-window replay batch over ONE stream
    adam: Optional[tuple] = None         # None -> plain SGD; (beta1, beta2, eps) -> Adam
    extra: dict = field(default_factory=dict)

    @property
    def depth(self):
        return len(self.balance) if self.balance else len(self.layers)

    @property
    def k(self):
        return self.depth - 1 if self.target_delay is None else self.target_delay

    @property
    def in_size(self):
        return self.layers[0].in_size

    @property
    def out_size(self):
        return self.layers[-1].out_size

    @property
    def n_weights(self):
        return sum(int(np.prod(l.w_shape)) for l in self.layers)


def mlp(widths, act, last_act=ACT_ID):
    ls = []
    for i in range(len(widths) - 1):
        a = act if i < len(widths) - 2 else last_act
        ls.append(LayerSpec(DENSE, a, widths[i], widths[i + 1]))
    return ls


def workload(cfg: int, ticks: Optional[int] = None) -> Workload:
    """The five benchmark workloads (index 0..4), at their full sizes; 5 = workload 1 with two layers per stage, 6 = workload 1 with Adam,
    11 = workload 1 with residual connections, 12-15 = replay batches, 16 = workload 3 with Adam, 17 = workload 4 with Adam, 18 / 19 = workload 12 in two stages / one stage, 20 = workload 12 with residual connections,
    7 / 8 / 9 / 10 = a 150-layer conv stack in 8 stages with 64 / 10 / 1 / 100 feature maps."""
    if cfg == 0:
        w = Workload("mlp4x256_f32_relu_ce", mlp([256, 256, 256, 256, 10], ACT_RELU),
                     loss=LOSS_CE, lr=1e-3, ticks=1000, drift=0.01, n_classes=10)
    elif cfg == 1:
        w = Workload("mlp8x4096_f32_relu_mse", mlp([4096] * 9, ACT_RELU),
                     loss=LOSS_MSE, lr=1e-4, ticks=2000, drift=0.005)
    elif cfg == 2:
        w = Workload("mlp16x2048_bf16_gelu_ce", mlp([2048] * 16 + [100], ACT_GELU), w_dtype=W_BF16,
                     loss=LOSS_CE, lr=1e-3, ticks=4000, drift=0.01, n_classes=100)
    elif cfg == 3:
        ls = [LayerSpec(CONV3X3, ACT_RELU, c_in=3 if i == 0 else 64, c_out=64, h=128, w=128) for i in range(8)]
        ls.append(LayerSpec(GAP_DENSE, ACT_ID, out_dim=10, c_in=64, h=128, w=128))
        w = Workload("cnn8x64_f32_relu_ce", ls, loss=LOSS_CE, lr=1e-3, ticks=500, n_classes=10)
    elif cfg == 4:
        w = Workload("mlp8x4096_bf16_s32_ce", mlp([4096] * 8 + [1000], ACT_RELU), n_streams=32,
                     w_dtype=W_BF16, loss=LOSS_CE, lr=1e-4, ticks=2000, drift=0.01, n_classes=1000)
    elif cfg == 5:
        # the 8 x 4096 network of workload 1 cut into 4 stages of two layers (exact back-propagation inside a stage)
        w = Workload("mlp8x4096_f32_relu_mse_d4", mlp([4096] * 9, ACT_RELU), loss=LOSS_MSE, lr=1e-4, ticks=2000,
                     drift=0.005, balance=[2, 2, 2, 2])
    elif cfg == 6:
        # workload 1 trained with Adam (defaults of the usual implementations): three arrays per layer move every tick
        w = Workload("mlp8x4096_f32_relu_mse_adam", mlp([4096] * 9, ACT_RELU), loss=LOSS_MSE, lr=1e-5, ticks=2000,
                     drift=0.005, adam=(0.9, 0.999, 1e-8))
    elif cfg in (7, 8, 9, 10):
        # shaped like the paper's pixel-wise prediction experiment (Sec. V-A): 150 conv layers at a fixed 256 x 256
        # resolution, cut into 7 stages, plus the pooled head as stage 8; F = 64 (7), 10 (8), 1 (9) or 100 (10) feature maps
        feat = {7: 64, 8: 10, 9: 1, 10: 100}[cfg]
        w = Workload(f"cnn150x{feat}_256_f32_relu_ce_d8", conv_net(3, 256, 256, 150, 10, feat=feat), loss=LOSS_CE,
                     lr=1e-4, ticks=30, n_classes=10, balance=[22, 22, 22, 21, 21, 21, 21, 1])
    elif cfg == 11:
        # workload 1 with residual connections around every pair of layers (each crosses two stage boundaries)
        ls = mlp([4096] * 9, ACT_RELU)
        for dst in (2, 4, 6):
            ls[dst].skip_from = dst - 2
        w = Workload("mlp8x4096_f32_relu_mse_skips", ls, loss=LOSS_MSE, lr=1e-4, ticks=2000, drift=0.005)
    elif cfg in (12, 13, 14, 15):
        # the network of workload 4 fed with a sliding-window replay batch (Sec. V-D) of 256 / 1024 / 64 samples and
        # trained with Adam (12, 13, 14), or of 1024 samples with plain SGD (15)
        B = {12: 256, 13: 1024, 14: 64, 15: 1024}[cfg]
        w = Workload(f"mlp8x4096_bf16_b{B}_ce_" + ("sgd" if cfg == 15 else "adam"), mlp([4096] * 8 + [1000], ACT_RELU),
                     n_streams=B, w_dtype=W_BF16, loss=LOSS_CE, lr=1e-5, ticks=100, drift=0.01, n_classes=1000,
                     replay=True, adam=None if cfg == 15 else (0.9, 0.999, 1e-8))
    elif cfg == 16:
        # workload 3 trained with Adam (Sec. V-D trains a conv net with it)
        w = workload(3)
        w.name, w.lr, w.adam = "cnn8x64_f32_relu_ce_adam", 1e-4, (0.9, 0.999, 1e-8)
    elif cfg == 17:
        # workload 4 trained with Adam
        w = workload(4)
        w.name, w.lr, w.adam = "mlp8x4096_bf16_s32_ce_adam", 1e-5, (0.9, 0.999, 1e-8)
    elif cfg in (18, 19):
        # workload 12 (replay batch of 256, Adam) as the two-stage pipeline of Sec. V-D (18) and as one stage, which is
        # plain sequential training (19)
        w = workload(12)
        w.balance = [4, 4] if cfg == 18 else [8]
        w.name += "_d2" if cfg == 18 else "_d1"
    elif cfg == 20:
        # workload 12 with residual connections around every pair of hidden layers
        w = workload(12)
        for dst in (2, 4, 6):
            w.layers[dst].skip_from = dst - 2
        w.name += "_skips"
    elif cfg == 21:
        # workload 4 as four stages of two layers
        w = workload(4)
        w.balance = [2, 2, 2, 2]
        w.name += "_d4"
    else:
        raise ValueError(cfg)
    if ticks is not None:
        w.ticks = ticks
    return w


def small_mlp(widths, act=ACT_RELU, loss=LOSS_MSE, **kw) -> Workload:
    """A small test network.  Its class targets are a noisy teacher: half of the labels are replaced by seeded random
    classes, so that a short, fast-learning test run cannot drive the loss (and with it every error signal) to zero."""
    kw.setdefault("extra", {"label_noise": 0.5} if loss == LOSS_CE else {})
    return Workload("mlp_" + "x".join(map(str, widths)), mlp(widths, act), loss=loss,
                    n_classes=widths[-1] if loss == LOSS_CE else 0, **kw)


# --------------------------------------------------------------------------- inputs

def _rms_normalize(v):
    return v * (np.sqrt(v.shape[-1]) / np.linalg.norm(v, axis=-1, keepdims=True))


def smooth_stream(ticks: int, d: int, drift: float, seed: int, n_streams: int = 1) -> np.ndarray:
    """x_0 = nrm(xi_0), x_t = nrm(x_{t-1} + drift*xi_t), xi ~ N(0, I); nrm scales to unit RMS.

    Stream s uses seed+s.  Returns fp32 [ticks][n_streams][d].
    """
    out = np.empty((ticks, n_streams, d), dtype=np.float32)
    for s in range(n_streams):
        rng = np.random.Generator(np.random.PCG64(seed + s))
        x = _rms_normalize(rng.standard_normal(d))
        out[0, s] = x
        for t in range(1, ticks):
            x = _rms_normalize(x + drift * rng.standard_normal(d))
            out[t, s] = x
    return out


def init_weights(layers: List[LayerSpec], seed: int):
    """U(-1/sqrt(fan_in), 1/sqrt(fan_in)) weights and biases, fp32."""
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    Ws, bs = [], []
    for l in layers:
        a = 1.0 / np.sqrt(l.fan_in)
        Ws.append(rng.uniform(-a, a, size=l.w_shape).astype(np.float32))
        bs.append(rng.uniform(-a, a, size=l.b_shape).astype(np.float32))
    return Ws, bs


def teacher_classes(x: np.ndarray, n_classes: int, seed: int) -> np.ndarray:
    """Class ids from a fixed random 2-layer ReLU teacher; x [T][S][d] -> int32 [T][S]."""
    d = x.shape[-1]
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    A1 = rng.standard_normal((d, d)) / np.sqrt(d)
    A2 = rng.standard_normal((n_classes, d)) / np.sqrt(d)
    hdn = np.maximum(x.astype(np.float64) @ A1.T, 0.0)
    return np.argmax(hdn @ A2.T, axis=-1).astype(np.int32)


def teacher_regression(x: np.ndarray, out_dim: int, seed: int, noise: float = 0.01) -> np.ndarray:
    """gamma = A x + noise*eps from a fixed random linear teacher; fp32 [T][S][out]."""
    d = x.shape[-1]
    rng = np.random.Generator(np.random.PCG64(seed + 3000))
    A = (rng.standard_normal((out_dim, d)) / np.sqrt(d)).astype(np.float32)
    y = x.astype(np.float32) @ A.T
    y = y + noise * rng.standard_normal(y.shape).astype(np.float32)
    return y.astype(np.float32)


def blob_video(ticks: int, h: int, w: int, seed: int, n_blobs: int = 8, noise: float = 0.02):
    """Synthetic video: isotropic Gaussian blobs translating at 1 px/tick in fixed random directions on a torus,
    plus pixel noise.  Returns frames fp32 [ticks][3*h*w] (planar RGB) and int32 labels [ticks]: the quadrant
    (0 TL, 1 TR, 2 BL, 3 BR) that holds the centre of the widest blob."""
    rng = np.random.Generator(np.random.PCG64(seed + 4000))
    scale = min(h, w) / 128.0
    sigma = rng.uniform(4.0, 12.0, n_blobs) * scale
    amp = rng.uniform(0.5, 1.0, (n_blobs, 3))
    pos = rng.uniform(0, 1, (n_blobs, 2)) * np.array([h, w])
    ang = rng.uniform(0, 2 * np.pi, n_blobs)
    vel = np.stack([np.sin(ang), np.cos(ang)], axis=1)
    big = int(np.argmax(sigma))
    yy, xx = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    frames = np.empty((ticks, 3, h, w), dtype=np.float32)
    labels = np.empty((ticks,), dtype=np.int32)
    for t in range(ticks):
        img = np.zeros((3, h, w))
        for k in range(n_blobs):
            dy = (yy - pos[k, 0] + h / 2) % h - h / 2      # toroidal distance
            dx = (xx - pos[k, 1] + w / 2) % w - w / 2
            g = np.exp(-(dy * dy + dx * dx) / (2 * sigma[k] ** 2))
            img += amp[k][:, None, None] * g[None]
        img += noise * rng.standard_normal(img.shape)
        frames[t] = img
        labels[t] = (2 if pos[big, 0] >= h / 2 else 0) + (1 if pos[big, 1] >= w / 2 else 0)
        pos = (pos + vel) % np.array([h, w])
    return frames.reshape(ticks, 3 * h * w), labels


def conv_net(c_in, h, w, n_conv, n_classes, act=ACT_RELU, feat=64):
    ls = [LayerSpec(CONV3X3, act, c_in=c_in if i == 0 else feat, c_out=feat, h=h, w=w) for i in range(n_conv)]
    ls.append(LayerSpec(GAP_DENSE, ACT_ID, out_dim=n_classes, c_in=feat, h=h, w=w))
    return ls


def make_inputs(w: Workload, ticks: Optional[int] = None):
    """(x [T][S][in], target) for a workload, per its recipe."""
    T = ticks if ticks is not None else w.ticks
    if w.layers[0].kind == CONV3X3:
        l0 = w.layers[0]
        x, y = blob_video(T, l0.h, l0.w, w.seed)
        if w.loss == LOSS_CE:
            return x.reshape(T, 1, -1), (y % w.n_classes).reshape(T, 1).astype(np.int32)
        onehot = np.zeros((T, 1, w.out_size), dtype=np.float32)
        onehot[np.arange(T), 0, y % w.out_size] = 1.0
        return x.reshape(T, 1, -1), onehot
    if w.replay:
        # one smooth stream; the batch of tick t holds its samples t .. t + B - 1, sample n sitting in slot n mod B:
        # every tick the newest sample replaces the oldest one and the other slots stay as they are
        Bn = w.n_streams
        base = smooth_stream(T + Bn - 1, w.in_size, w.drift, w.seed, 1)
        tb = teacher_classes(base, w.n_classes, w.seed) if w.loss == LOSS_CE else teacher_regression(base, w.out_size, w.seed)
        t_idx, slot = np.arange(T)[:, None], np.arange(Bn)[None, :]
        idx = t_idx + (slot - t_idx) % Bn
        return base[idx, 0], tb[idx, 0]
    x = smooth_stream(T, w.in_size, w.drift, w.seed, w.n_streams)
    if w.loss == LOSS_CE:
        tgt = teacher_classes(x, w.n_classes, w.seed)
        noise = w.extra.get("label_noise", 0.0)
        if noise > 0.0:
            rng = np.random.Generator(np.random.PCG64(w.seed + 6000))
            swap = rng.random(tgt.shape) < noise
            tgt = np.where(swap, rng.integers(0, w.n_classes, size=tgt.shape), tgt).astype(np.int32)
    else:
        tgt = teacher_regression(x, w.out_size, w.seed)
    return x, tgt
