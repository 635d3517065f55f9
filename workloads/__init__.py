"""Seeded synthetic inputs for the partial-distillation workloads.

This module only *draws inputs*: feature maps standing in for the output of the
student's frozen front part, Voronoi label maps standing in for the teacher's
per-pixel pseudo-labels, and He-normal initial values for the trainable head.
It holds none of the method's arithmetic (no convolution, no loss, no metric)
and is the one module that the CPU oracle's tests and the GPU path's tests both
import, so that both sides consume identical bytes.

Everything is numpy; nothing here touches a GPU.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

IGNORE_NONE = -1


@dataclass(frozen=True)
class Workload:
    """One named configuration: head shape, input recipe and optimiser settings."""

    name: str
    n: int
    c_in: int
    h: int
    w: int
    c1: int
    c2: int
    n_classes: int
    steps: int
    lr: float
    momentum: float = 0.0
    feat_dtype: str = "bf16"        # "f32" or "bf16"
    compute: str = "bf16"           # "f32" or "bf16"
    ignore_index: int = IGNORE_NONE
    ignore_fraction: float = 0.0
    n_sites: int = 40
    feat_seed: int = 0
    label_seed: int = 0
    init_seed: int = 0
    clamp_features: bool = True     # max(N(0,1), 0): features come out of a ReLU
    upscale: int = 8
    extra: dict = field(default_factory=dict)

    @property
    def H(self) -> int:
        return self.h * self.upscale

    @property
    def W(self) -> int:
        return self.w * self.upscale

    @property
    def n_params(self) -> int:
        return (self.c1 * self.c_in * 9 + self.c1 + self.c2 * self.c1 * 9 + self.c2
                + self.n_classes * self.c2 + self.n_classes)


WORKLOADS = {
    # fp32 features, fp32 compute path, tiny enough for exhaustive element-wise parity
    "tiny": Workload("tiny", 1, 64, 16, 16, 64, 64, 9, steps=4, lr=0.01,
                     feat_dtype="f32", compute="f32", n_sites=12,
                     feat_seed=1001, label_seed=2001, init_seed=3001,
                     clamp_features=False),
    # the headline configuration: one 1280x720 key frame
    "720p": Workload("720p", 1, 256, 90, 160, 128, 128, 19, steps=8, lr=0.01,
                     n_sites=40, feat_seed=1002, label_seed=2002, init_seed=3002),
    "1080p": Workload("1080p", 1, 256, 135, 240, 128, 128, 19, steps=8, lr=0.01,
                      momentum=0.9, ignore_index=255, ignore_fraction=0.05,
                      n_sites=80, feat_seed=1003, label_seed=2003, init_seed=3003),
    "batch4": Workload("batch4", 4, 320, 90, 160, 256, 256, 21, steps=16, lr=0.005,
                       n_sites=40, feat_seed=1004, label_seed=2004, init_seed=3004),
    "clip": Workload("clip", 1, 256, 90, 160, 128, 128, 19, steps=8, lr=0.01,
                     n_sites=40, feat_seed=1005, label_seed=2005, init_seed=3005,
                     extra={"frames": 32, "drift": 0.05, "shift_px": 2,
                            "threshold": 0.75}),
}


# --------------------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16 bit patterns.

    Used only to *store* drawn feature values in the dtype the workload names."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------- features
def make_features(wl: Workload, seed: int | None = None) -> np.ndarray:
    """Feature map [n, c_in, h, w], iid N(0,1) (clamped at 0 when the workload says so).

    Returns float32 for "f32" workloads and uint16 bfloat16 bit patterns for "bf16" ones."""
    rng = np.random.default_rng(wl.feat_seed if seed is None else seed)
    f = rng.standard_normal((wl.n, wl.c_in, wl.h, wl.w), dtype=np.float32)
    if wl.clamp_features:
        np.maximum(f, 0.0, out=f)
    if wl.feat_dtype == "bf16":
        return f32_to_bf16_bits(f)
    return f


def features_as_f64(wl: Workload, feats: np.ndarray) -> np.ndarray:
    """The exact real values of a feature array, as float64 (what the oracle consumes)."""
    if feats.dtype == np.uint16:
        return bf16_bits_to_f32(feats).astype(np.float64)
    return feats.astype(np.float64)


def drift_features(master_f32: np.ndarray, sigma: float, seed: int) -> np.ndarray:
    """f_t = f_{t-1} + sigma * N(0,1) on a float32 master copy (no re-clamp)."""
    rng = np.random.default_rng(seed)
    return master_f32 + np.float32(sigma) * rng.standard_normal(master_f32.shape, dtype=np.float32)


# --------------------------------------------------------------------------- labels
def voronoi_sites(n_sites: int, H: int, W: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    ys = rng.integers(0, H, size=n_sites)
    xs = rng.integers(0, W, size=n_sites)
    return np.stack([ys, xs], axis=1).astype(np.int64)


def voronoi_labels(sites: np.ndarray, H: int, W: int, n_classes: int,
                   shift_x: int = 0) -> np.ndarray:
    """Label map [H, W] int32: pixel -> class of the nearest site (integer squared distance,
    ties to the lowest site index); site i carries class i mod n_classes.  `shift_x` moves
    the whole pattern right by that many pixels on an unbounded plane."""
    out = np.empty((H, W), dtype=np.int32)
    sy = sites[:, 0][:, None, None]
    sx = (sites[:, 1] + shift_x)[:, None, None]
    xs = np.arange(W, dtype=np.int64)[None, None, :]
    cls = (np.arange(len(sites)) % n_classes).astype(np.int32)
    rows = max(1, (1 << 22) // (W * len(sites)))
    for y0 in range(0, H, rows):
        ys = np.arange(y0, min(H, y0 + rows), dtype=np.int64)[None, :, None]
        d = (ys - sy) ** 2 + (xs - sx) ** 2
        out[y0:y0 + ys.shape[1]] = cls[np.argmin(d, axis=0)]
    return out


def make_labels(wl: Workload, frame_shift: int = 0) -> np.ndarray:
    """Teacher pseudo-labels [n, H, W] int32; frame i of a batch uses seed label_seed + i.
    With `ignore_fraction` > 0 an iid Bernoulli subset of pixels is set to ignore_index."""
    H, W = wl.H, wl.W
    lab = np.empty((wl.n, H, W), dtype=np.int32)
    for i in range(wl.n):
        sites = voronoi_sites(wl.n_sites, H, W, wl.label_seed + i)
        lab[i] = voronoi_labels(sites, H, W, wl.n_classes, shift_x=frame_shift)
    if wl.ignore_fraction > 0.0:
        rng = np.random.default_rng(wl.label_seed + 100)
        mask = rng.random(lab.shape) < wl.ignore_fraction
        lab[mask] = wl.ignore_index
    return lab


def object_weight_map(labels: np.ndarray, radius: int = 4, factor: int = 5, background: int = 0) -> np.ndarray:
    """Per-pixel loss weights [n, H, W] uint8: `factor` on every pixel within `radius` pixels
    (Chebyshev distance) of a pixel whose label is a non-background class, 1 elsewhere.  The
    radius of "near" is not given in the paper: it is an input-recipe choice here."""
    obj = (labels != background) & (labels >= 0) & (labels < 255)
    near = obj.copy()
    for _ in range(radius):       # one-pixel square dilation, `radius` times
        g = near.copy()
        g[:, 1:, :] |= near[:, :-1, :]; g[:, :-1, :] |= near[:, 1:, :]
        near = g.copy()
        near[:, :, 1:] |= g[:, :, :-1]; near[:, :, :-1] |= g[:, :, 1:]
    return np.where(near, factor, 1).astype(np.uint8)


# --------------------------------------------------------------------------- head init
def param_slices(wl: Workload) -> dict:
    """Offsets of W1 (OIHW), b1, W2, b2, W3, b3 inside the flat parameter vector."""
    sizes = [("W1", wl.c1 * wl.c_in * 9), ("b1", wl.c1), ("W2", wl.c2 * wl.c1 * 9),
             ("b2", wl.c2), ("W3", wl.n_classes * wl.c2), ("b3", wl.n_classes)]
    out, off = {}, 0
    for name, sz in sizes:
        out[name] = slice(off, off + sz)
        off += sz
    return out


def make_head_params(wl: Workload, seed: int | None = None) -> np.ndarray:
    """Flat float32 parameter vector: He-normal weights (std sqrt(2 / fan_in)), zero biases."""
    rng = np.random.default_rng(wl.init_seed if seed is None else seed)
    p = np.zeros(wl.n_params, dtype=np.float32)
    sl = param_slices(wl)
    for name, fan_in in (("W1", wl.c_in * 9), ("W2", wl.c1 * 9), ("W3", wl.c2)):
        s = sl[name]
        p[s] = rng.standard_normal(s.stop - s.start, dtype=np.float32) * np.float32(
            np.sqrt(2.0 / fan_in))
    return p


# --------------------------------------------------------------------------- test variants
def make_learnable_features(wl: Workload, labels: np.ndarray, strength: float = 2.0,
                            seed: int = 7) -> np.ndarray:
    """Features that do carry the labels (noise + a fixed random code per class placed at the
    low-resolution cell's centre label).  Not a measured workload: it lets tests reach the
    early-exit branch of the training loop, which iid-noise features never do."""
    rng = np.random.default_rng(seed)
    code = rng.standard_normal((wl.n_classes + 1, wl.c_in)).astype(np.float32)
    noise = rng.standard_normal((wl.n, wl.c_in, wl.h, wl.w), dtype=np.float32)
    s = wl.upscale
    centre = labels[:, s // 2::s, s // 2::s][:, :wl.h, :wl.w]
    centre = np.where((centre >= 0) & (centre < wl.n_classes), centre, wl.n_classes)
    f = noise * np.float32(0.3) + np.float32(strength) * np.transpose(code[centre], (0, 3, 1, 2))
    if wl.clamp_features:
        np.maximum(f, 0.0, out=f)
    if wl.feat_dtype == "bf16":
        return f32_to_bf16_bits(f)
    return f.astype(np.float32)


def clip_frames(wl: Workload, learnable: bool = False, strength: float = 2.0):
    """The frames of a temporal clip: labels are the Voronoi map moved `shift_px` pixels per frame,
    features drift as f_t = f_{t-1} + drift * N(0,1) on a float32 master.  With `learnable` the
    master of every frame additionally carries that frame's labels (see make_learnable_features),
    so that a trained head scores well on the next frame; the measured clip uses plain noise.
    Yields (features, labels) with features in the workload's dtype."""
    n_frames = int(wl.extra["frames"])
    drift, shift = float(wl.extra["drift"]), int(wl.extra["shift_px"])
    rng0 = np.random.default_rng(wl.feat_seed)
    noise = rng0.standard_normal((wl.n, wl.c_in, wl.h, wl.w), dtype=np.float32)
    if not learnable and wl.clamp_features:
        np.maximum(noise, 0.0, out=noise)
    for t in range(n_frames):
        labels = make_labels(wl, frame_shift=t * shift)
        if t > 0:
            noise = drift_features(noise, drift, wl.feat_seed + 1000 + t)
        f = noise
        if learnable:
            rng = np.random.default_rng(7)
            code = rng.standard_normal((wl.n_classes + 1, wl.c_in)).astype(np.float32)
            s_ = wl.upscale
            centre = labels[:, s_ // 2::s_, s_ // 2::s_][:, :wl.h, :wl.w]
            centre = np.where((centre >= 0) & (centre < wl.n_classes), centre, wl.n_classes)
            f = noise * np.float32(0.3) + np.float32(strength) * np.transpose(code[centre], (0, 3, 1, 2))
            if wl.clamp_features:
                f = np.maximum(f, 0.0)
        yield (f32_to_bf16_bits(f) if wl.feat_dtype == "bf16" else f.astype(np.float32)), labels


def small_variant(wl: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (ragged test sizes and the like)."""
    d = {k: getattr(wl, k) for k in wl.__dataclass_fields__}
    d.update(kw)
    return Workload(**d)
