"""Pins for the oracle's letterbox and crop-resize: closed forms and a library routine."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import preprocess as pre


def _img(h, w, seed=0):
    return np.random.default_rng(seed).integers(0, 256, size=(1, h, w, 3), dtype=np.uint8)


def test_identity_scale_is_divide_by_255():
    im = _img(32, 32)
    out = pre.letterbox(im, 32, 32, "f32")
    assert np.array_equal(out, (im.astype(np.float64) / 255.0).astype(np.float32))


def test_geometry_of_the_workload_shapes():
    assert pre.letterbox_geometry(1080, 1920, 640, 640)[1:] == (640, 360, 0, 140)
    assert pre.letterbox_geometry(2160, 3840, 1280, 1280)[1:] == (1280, 720, 0, 280)
    assert pre.letterbox_geometry(720, 1280, 640, 640)[1:] == (640, 360, 0, 140)
    assert pre.letterbox_geometry(320, 320, 320, 320)[1:] == (320, 320, 0, 0)
    assert pre.letterbox_geometry(100, 37, 64, 64)[1:] == (24, 64, 20, 0)     # 37*0.64 = 23.68 -> 24


def test_one_third_scale_picks_centre_pixel_and_pads_114():
    im = _img(54, 96, 1)                      # 16:9 like 1080p, r = 1/3 into 32x32
    out = pre.letterbox(im, 32, 32, "f32")
    _, nw, nh, left, top = pre.letterbox_geometry(54, 96, 32, 32)
    assert (nw, nh, left, top) == (32, 18, 0, 7)
    exp = (im[0, 1::3, 1::3].astype(np.float64) / 255.0).astype(np.float32)
    assert np.array_equal(out[0, top:top + nh], exp)
    pad = np.float32(114.0 / 255.0)
    assert np.all(out[0, :top] == pad) and np.all(out[0, top + nh:] == pad)


def test_half_scale_is_2x2_mean():
    im = _img(36, 64, 2)
    out = pre.letterbox(im, 32, 32, "f32")
    _, nw, nh, left, top = pre.letterbox_geometry(36, 64, 32, 32)
    assert (nw, nh, top) == (32, 18, 7)
    a = im[0].astype(np.float64)
    exp = (a[0::2, 0::2] + a[0::2, 1::2] + a[1::2, 0::2] + a[1::2, 1::2]) / 4.0 / 255.0
    assert np.allclose(out[0, top:top + nh], exp, atol=1e-7, rtol=0)


def test_double_scale_has_quarter_three_quarter_weights():
    im = _img(1, 4, 3)[:, :, :, :1].repeat(3, axis=3)
    im = np.repeat(im, 4, axis=1)             # 4x4, constant along y
    out = pre.letterbox(im, 8, 8, "f32")[0, 0, :, 0].astype(np.float64) * 255.0
    p = im[0, 0, :, 0].astype(np.float64)
    exp = [p[0], .75 * p[0] + .25 * p[1], .25 * p[0] + .75 * p[1], .75 * p[1] + .25 * p[2],
           .25 * p[1] + .75 * p[2], .75 * p[2] + .25 * p[3], .25 * p[2] + .75 * p[3], p[3]]
    assert np.allclose(out, exp, atol=1e-4)


def test_constant_image_stays_constant_and_normalisation_applies():
    im = np.full((2, 45, 80, 3), 200, np.uint8)
    out = pre.letterbox(im, 64, 64, "f32", norm_scale=(0.5, 1.0, 2.0), norm_bias=(1.0, 0.0, -1.0), pad_value=10)
    _, nw, nh, left, top = pre.letterbox_geometry(45, 80, 64, 64)
    inner = out[:, top:top + nh, left:left + nw]
    assert np.allclose(inner, np.array([101.0, 200.0, 399.0], np.float32))
    assert np.allclose(out[:, 0], np.array([6.0, 10.0, 19.0], np.float32))


def test_letterbox_matches_library_bilinear():
    im = _img(45, 83, 4)
    _, nw, nh, left, top = pre.letterbox_geometry(45, 83, 64, 64)
    out = pre.letterbox(im, 64, 64, "f32")
    t = torch.from_numpy(im.astype(np.float64)).permute(0, 3, 1, 2)
    ref = F.interpolate(t, size=(nh, nw), mode="bilinear", align_corners=False, antialias=False)
    ref = (ref.permute(0, 2, 3, 1).numpy() / 255.0)
    assert np.allclose(out[:, top:top + nh, left:left + nw], ref, atol=1e-6, rtol=0)
    up = pre.letterbox(im[:, :20, :30], 64, 64, "f32")          # upscale path
    _, nw, nh, left, top = pre.letterbox_geometry(20, 30, 64, 64)
    ref = F.interpolate(t[:, :, :20, :30], size=(nh, nw), mode="bilinear", align_corners=False)
    assert np.allclose(up[:, top:top + nh, left:left + nw], ref.permute(0, 2, 3, 1).numpy() / 255.0, atol=1e-6)


def test_storage_rounding_of_letterbox():
    im = _img(16, 16, 5)
    for dt, conv in (("f16", lambda v: v.astype(np.float16).astype(np.float32)),
                     ("bf16", lambda v: torch.from_numpy(v.astype(np.float32)).bfloat16().float().numpy())):
        out = pre.letterbox(im, 16, 16, dt)
        assert np.array_equal(out, conv(im.astype(np.float64) / 255.0))


def test_crop_aligned_window_is_exact_copy_and_full_frame_equals_letterbox_interior():
    im = _img(40, 50, 6)
    frames = np.concatenate([im, _img(40, 50, 7)])
    box = np.array([[7, 5, 7 + 16, 5 + 12], [0, 0, 50, 40]], np.float32)
    out = pre.crop_resize(frames, np.array([1]), box[:1], 12, 16, "f32")
    assert np.array_equal(out[0], (frames[1, 5:17, 7:23].astype(np.float64) / 255).astype(np.float32))
    _, nw, nh, left, top = pre.letterbox_geometry(40, 50, 64, 64)
    full = pre.crop_resize(frames, np.array([0]), box[1:], nh, nw, "f32")
    lb = pre.letterbox(frames[:1], 64, 64, "f32")
    assert np.array_equal(full[0], lb[0, top:top + nh, left:left + nw])


def test_crop_degenerate_and_out_of_frame_boxes_clamp():
    im = _img(20, 30, 8)
    out = pre.crop_resize(im, np.array([0, 0]), np.array([[30, 3, 30, 9], [4.0, 20, 9, 20]], np.float32), 4, 4, "f32")
    col = im[0, :, 29].astype(np.float64) / 255           # zero-width box at the right edge: one clamped column
    sy = 3 + (np.arange(4) + 0.5) * 6 / 4 - 0.5
    y0 = np.floor(sy).astype(int); fy = (sy - y0)[:, None]
    exp = (1 - fy) * col[y0] + fy * col[y0 + 1]
    assert np.allclose(out[0], exp[:, None, :].repeat(4, axis=1), atol=1e-6)
    assert np.allclose(out[1, 0], out[1, 3])               # zero-height box: all rows equal (bottom row clamped)
