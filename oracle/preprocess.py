"""Oracle: letterbox-resize + normalise, and ROI crop-resize (test infrastructure).

The paper is silent on pre-processing (it only states the camera resolution,
Sec. IV-A); the definitions used here are the plain ones:
aspect-preserving bilinear resize with half-pixel centres and no antialias
filter, centred padding with a constant, per-channel affine normalisation,
one rounding to the storage type.  Interpolation is evaluated in fp64.
"""
from __future__ import annotations

import math

import numpy as np

from .rounding import round_storage


def letterbox_geometry(src_h: int, src_w: int, dst_h: int, dst_w: int):
    """Scale r = min(dst_w/src_w, dst_h/src_h); resized size rounded half-up; centred (floor) offsets."""
    r = min(dst_w / src_w, dst_h / src_h)
    nw = int(math.floor(src_w * r + 0.5))
    nh = int(math.floor(src_h * r + 0.5))
    left = (dst_w - nw) // 2
    top = (dst_h - nh) // 2
    return r, nw, nh, left, top


def _bilinear_sample(img: np.ndarray, sy: np.ndarray, sx: np.ndarray) -> np.ndarray:
    """img uint8 [H][W][C]; sy [Ho], sx [Wo] fp64 source coordinates -> fp64 [Ho][Wo][C].

    Taps floor(s) and floor(s)+1 clamped to the image; weights (1-f, f).
    """
    h, w, _ = img.shape
    y0 = np.floor(sy)
    x0 = np.floor(sx)
    fy = (sy - y0)[:, None, None]
    fx = (sx - x0)[None, :, None]
    y0 = y0.astype(np.int64)
    x0 = x0.astype(np.int64)
    ya, yb = np.clip(y0, 0, h - 1), np.clip(y0 + 1, 0, h - 1)
    xa, xb = np.clip(x0, 0, w - 1), np.clip(x0 + 1, 0, w - 1)
    im = img.astype(np.float64)
    p00 = im[ya][:, xa]
    p01 = im[ya][:, xb]
    p10 = im[yb][:, xa]
    p11 = im[yb][:, xb]
    return (1 - fy) * ((1 - fx) * p00 + fx * p01) + fy * ((1 - fx) * p10 + fx * p11)


def letterbox(frames: np.ndarray, dst_h: int, dst_w: int, dtype: str,
              norm_scale=(1 / 255.0,) * 3, norm_bias=(0.0,) * 3, pad_value: int = 114) -> np.ndarray:
    """uint8 [N][Hs][Ws][3] -> fp32 array [N][dst_h][dst_w][3] of storage-type values."""
    n, hs, ws, c = frames.shape
    _, nw, nh, left, top = letterbox_geometry(hs, ws, dst_h, dst_w)
    scale = np.asarray(norm_scale, np.float64)
    bias = np.asarray(norm_bias, np.float64)
    out = np.empty((n, dst_h, dst_w, c), np.float64)
    out[:] = float(pad_value)
    sy = (np.arange(nh) + 0.5) * hs / nh - 0.5
    sx = (np.arange(nw) + 0.5) * ws / nw - 0.5
    for i in range(n):
        out[i, top:top + nh, left:left + nw] = _bilinear_sample(frames[i], sy, sx)
    return round_storage(out * scale + bias, dtype)


def crop_resize(frames: np.ndarray, roi_frame: np.ndarray, roi_box: np.ndarray, out_h: int, out_w: int,
                dtype: str, norm_scale=(1 / 255.0,) * 3, norm_bias=(0.0,) * 3) -> np.ndarray:
    """Bilinear stretch of each ROI (source-pixel box x1,y1,x2,y2) to out_h x out_w.

    Output pixel (j, i) samples the source at  x1 + (i+0.5)(x2-x1)/out_w - 0.5
    (same for y), clamp-to-edge; aspect ratio is not preserved; degenerate boxes
    are not dropped (they sample a single clamped row / column).
    """
    n = len(roi_frame)
    scale = np.asarray(norm_scale, np.float64)
    bias = np.asarray(norm_bias, np.float64)
    out = np.empty((n, out_h, out_w, frames.shape[3]), np.float64)
    for k in range(n):
        x1, y1, x2, y2 = (float(v) for v in roi_box[k])
        sx = x1 + (np.arange(out_w) + 0.5) * (x2 - x1) / out_w - 0.5
        sy = y1 + (np.arange(out_h) + 0.5) * (y2 - y1) / out_h - 0.5
        out[k] = _bilinear_sample(frames[int(roi_frame[k])], sy, sx)
    return round_storage(out * scale + bias, dtype)
