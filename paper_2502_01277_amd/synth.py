"""Seeded synthetic inputs: camera frames, per-frame object counts, planted
detector-head tensors and request arrival times.

Input generation only - nothing here is part of the inference path, and both the
CPU oracle and the HIP path are fed from these functions.  The paper measures on
private 15 fps camera streams (Sec. IV-A); these synthetic frames stand in for
them: uniform-noise background with filled rectangles, with per-frame object
counts following the distributions each workload names (the paper stresses that
per-frame object counts are bursty and drive downstream load, Sec. III-B,
Observation 1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List

import numpy as np

from .zoo import ModelSpec, round_to_dtype


# ---------------------------------------------------------------------------
# storage-format helpers (bit plumbing, no arithmetic of the method)
# ---------------------------------------------------------------------------
def to_storage(x_f32: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 -> raw array in storage type (f32: float32, f16: float16, bf16: uint16 bit patterns)."""
    x = np.ascontiguousarray(x_f32, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        r = round_to_dtype(x, "bf16")
        return (r.view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def from_storage(raw: np.ndarray, dtype: str) -> np.ndarray:
    """raw storage array -> fp32 (exact widening)."""
    if dtype == "f32":
        return np.asarray(raw, dtype=np.float32)
    if dtype == "f16":
        return np.asarray(raw).view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return (np.asarray(raw).view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    raise ValueError(dtype)


def storage_itemsize(dtype: str) -> int:
    return 4 if dtype == "f32" else 2


def e4m3_codes(rng, shape, max_field: int = 8, p_zero: float = 0.05) -> np.ndarray:
    """Random 8-bit floating-point codes (1 sign, 4 exponent, 3 mantissa bits): uniform sign and mantissa, exponent field
    uniform in 0..max_field (field 0 = the subnormals), a fraction p_zero of exact zeros.  Never a NaN code (field 15
    with mantissa 7) as long as max_field < 15.  Bits only: what the codes mean is the business of whoever reads them."""
    assert 0 <= max_field < 15
    sign = rng.integers(0, 2, shape).astype(np.uint8) << 7
    field = rng.integers(0, max_field + 1, shape).astype(np.uint8) << 3
    mant = rng.integers(0, 8, shape).astype(np.uint8)
    codes = sign | field | mant
    return np.where(rng.random(shape) < p_zero, np.uint8(0), codes).astype(np.uint8)


# ---------------------------------------------------------------------------
# object counts
# ---------------------------------------------------------------------------
def counts_poisson(rng, n, mean=8.0, cap=64):
    return np.minimum(rng.poisson(mean, size=n), cap).astype(np.int64)


def counts_negbin(rng, n, mean=6.0, var=60.0, cap=200):
    """Negative binomial as a Gamma-Poisson mixture (shape r, scale theta): mean r*theta, var mean + mean^2/r."""
    r = mean * mean / (var - mean)
    theta = mean / r
    lam = rng.gamma(shape=r, scale=theta, size=n)
    return np.minimum(rng.poisson(lam), cap).astype(np.int64)


def counts_pareto(rng, n, alpha=1.5, x_m=5.0, cap=300):
    u = 1.0 - rng.random(size=n)          # (0, 1]
    return np.minimum(np.floor(x_m * u ** (-1.0 / alpha)), cap).astype(np.int64)


# ---------------------------------------------------------------------------
# frames
# ---------------------------------------------------------------------------
@dataclass
class Scene:
    frames: np.ndarray          # uint8 [N][H][W][3], RGB
    rects: List[np.ndarray]     # per frame: float64 [K][4] (x1, y1, x2, y2) in source pixels
    classes: List[np.ndarray]   # per frame: int64 [K]


def make_scene(rng, n_frames, h, w, counts, side_lo, side_hi, log_uniform=False, n_classes=80) -> Scene:
    frames = rng.integers(0, 256, size=(n_frames, h, w, 3), dtype=np.uint8)
    rects, classes = [], []
    for f in range(n_frames):
        k = int(counts[f])
        if log_uniform:
            sw = np.exp(rng.uniform(math.log(side_lo), math.log(side_hi), size=k))
            sh = np.exp(rng.uniform(math.log(side_lo), math.log(side_hi), size=k))
        else:
            sw = rng.integers(side_lo, side_hi + 1, size=k).astype(np.float64)
            sh = rng.integers(side_lo, side_hi + 1, size=k).astype(np.float64)
        sw = np.minimum(np.floor(sw), w - 1)
        sh = np.minimum(np.floor(sh), h - 1)
        x1 = np.floor(rng.uniform(0, 1, size=k) * (w - sw))
        y1 = np.floor(rng.uniform(0, 1, size=k) * (h - sh))
        col = rng.integers(0, 256, size=(k, 3), dtype=np.uint8)
        for j in range(k):
            frames[f, int(y1[j]):int(y1[j] + sh[j]), int(x1[j]):int(x1[j] + sw[j])] = col[j]
        rects.append(np.stack([x1, y1, x1 + sw, y1 + sh], axis=1) if k else np.zeros((0, 4)))
        classes.append(rng.integers(0, n_classes, size=k))
    return Scene(frames, rects, classes)


# ---------------------------------------------------------------------------
# planted detector heads
# ---------------------------------------------------------------------------
def _logit(p):
    return math.log(p / (1.0 - p))


def planted_heads(rng, det: ModelSpec, scene: Scene, src_h, src_w, geom, max_dups=4, n_clutter=0):
    """Head tensors whose decode yields the scene's rectangles (plus near-duplicates and clutter).

    geom = (nw, nh, left, top): size and position of the resized frame inside the detector's input, as the
    pre-processing under test places it (the caller asks the implementation it feeds: this generator holds no
    letterbox arithmetic of its own).

    Returns a list (one per level) of fp32 arrays [N][G][G][A*(5+C)] holding
    values already representable in the detector's storage type.  Random-init
    weights cannot produce a prescribed object count, so these tensors replace
    the real head outputs in front of the decode step.
    """
    n = scene.frames.shape[0]
    A, C = det.n_anchors, det.n_classes
    no = 5 + C
    table = rng.standard_normal(256).astype(np.float32) * np.float32(1.5)
    heads = []
    for g in det.grids:
        idx = rng.integers(0, 256, size=(n, g, g, A, no), dtype=np.uint8)
        h = table[idx]
        h[..., 4] = -8.0
        h[..., 5:] = np.minimum(h[..., 5:], 2.0)
        heads.append(h)
    nw, nh, left, top = geom
    rx, ry = nw / src_w, nh / src_h
    used = set()

    def plant(f, lvl, a, gy, gx, cx, cy, bw, bh, obj, cls):
        g = det.grids[lvl]
        if not (0 <= gx < g and 0 <= gy < g) or (f, lvl, gy, gx, a) in used:
            return False
        s = det.strides[lvl]
        aw, ah = det.anchors[lvl, a]
        px = ((cx / s - gx) + 0.5) / 2.0
        py = ((cy / s - gy) + 0.5) / 2.0
        pw = math.sqrt(bw / aw) / 2.0
        ph = math.sqrt(bh / ah) / 2.0
        if not (0.02 < px < 0.98 and 0.02 < py < 0.98 and 0.02 < pw < 0.98 and 0.02 < ph < 0.98):
            return False
        used.add((f, lvl, gy, gx, a))
        v = heads[lvl][f, gy, gx, a]
        v[0], v[1], v[2], v[3] = _logit(px), _logit(py), _logit(pw), _logit(ph)
        v[4] = obj
        v[5:] = -6.0
        v[5 + cls] = 4.0
        return True

    def best_slot(bw, bh):
        best, arg = -1.0, (0, 0)
        for lvl in range(len(det.grids)):
            for a in range(A):
                aw, ah = det.anchors[lvl, a]
                inter = min(aw, bw) * min(ah, bh)
                iou = inter / (aw * ah + bw * bh - inter)
                if iou > best:
                    best, arg = iou, (lvl, a)
        return arg

    for f in range(n):
        for j in range(scene.rects[f].shape[0]):
            x1, y1, x2, y2 = scene.rects[f][j]
            cx, cy = (x1 + x2) / 2 * rx + left, (y1 + y2) / 2 * ry + top
            bw, bh = max((x2 - x1) * rx, 2.0), max((y2 - y1) * ry, 2.0)
            cls = int(scene.classes[f][j]) % C
            lvl, a = best_slot(bw, bh)
            s = det.strides[lvl]
            gx, gy = int(cx // s), int(cy // s)
            obj = float(rng.uniform(1.0, 4.0))
            plant(f, lvl, a, gy, gx, cx, cy, bw, bh, obj, cls)
            for _ in range(int(rng.integers(0, max_dups + 1))):
                jw, jh = bw * rng.uniform(0.9, 1.1), bh * rng.uniform(0.9, 1.1)
                o2 = obj - float(rng.uniform(0.2, 1.0))
                if rng.random() < 0.5:
                    plant(f, lvl, int((a + 1 + rng.integers(0, A - 1)) % A), gy, gx, cx, cy, jw, jh, o2, cls)
                else:
                    dx = -1 if (cx / s - gx) < 0.5 else 1
                    dy = -1 if (cy / s - gy) < 0.5 else 1
                    if rng.random() < 0.5:
                        plant(f, lvl, a, gy, gx + dx, cx, cy, jw, jh, o2, cls)
                    else:
                        plant(f, lvl, a, gy + dy, gx, cx, cy, jw, jh, o2, cls)
        # low-score clutter so that top-k really truncates: candidates crowd around a few hot spots (same class,
        # similar size, jittered centres), so NMS has dense overlaps to resolve and removes most of them again
        n_spots = 40 if n_clutter else 0
        size = det.in_w
        spots = [(rng.uniform(0.1, 0.9) * size, rng.uniform(0.25, 0.75) * size, rng.uniform(0.05, 0.18) * size,
                  rng.uniform(0.05, 0.18) * size, int(rng.integers(0, C))) for _ in range(n_spots)]
        placed, tries = 0, 0
        while placed < n_clutter and tries < 20 * n_clutter:
            tries += 1
            sx, sy, sw, sh, scls = spots[int(rng.integers(0, n_spots))]
            cx, cy = sx + rng.uniform(-0.25, 0.25) * sw, sy + rng.uniform(-0.25, 0.25) * sh
            bw, bh = sw * rng.uniform(0.85, 1.15), sh * rng.uniform(0.85, 1.15)
            lvl = int(rng.integers(0, len(det.grids)))
            s_ = det.strides[lvl]
            a = int(rng.integers(0, A))
            gx, gy = int(cx // s_) + int(rng.integers(-1, 2)) * int(rng.random() < 0.3), int(cy // s_)
            # score = sigmoid(obj) * sigmoid(4) in (0.26, 0.30)
            target = rng.uniform(0.262, 0.298) / (1.0 / (1.0 + math.exp(-4.0)))
            placed += bool(plant(f, lvl, a, gy, gx, cx, cy, bw, bh, _logit(target), scls))
    return [round_to_dtype(h.reshape(n, g, g, A * no), det.dtype) for h, g in zip(heads, det.grids)]


# ---------------------------------------------------------------------------
# arrivals (open-loop load)
# ---------------------------------------------------------------------------
def sinusoid_arrivals(rng, n_streams, duration_s, base_fps=15.0, depth=0.5, period_s=10.0, boost=None):
    """Inhomogeneous Poisson arrivals by thinning; stream i has rate base*(1+depth*sin(2 pi t/period + 2 pi i/n)).

    boost: optional list with one entry per stream, None or (t0, t1, factor): the stream's rate is multiplied by
    factor for t0 <= t < t1 (a workload surge).  Returns a list of sorted arrival-time arrays (seconds), one per stream.
    """
    out = []
    for i in range(n_streams):
        b = boost[i] if boost is not None else None
        peak = base_fps * (1.0 + depth) * (max(1.0, b[2]) if b else 1.0)
        n_prop = rng.poisson(peak * duration_s)
        t = np.sort(rng.uniform(0.0, duration_s, size=n_prop))
        lam = base_fps * (1.0 + depth * np.sin(2 * np.pi * t / period_s + 2 * np.pi * i / n_streams))
        if b:
            lam = np.where((t >= b[0]) & (t < b[1]), lam * b[2], lam)
        keep = rng.random(size=n_prop) < lam / peak
        out.append(t[keep])
    return out
