"""Pins for the oracle's layer arithmetic: brute force, closed forms, linearity, library cross-checks."""
import numpy as np
import pytest
import torch

from oracle import nn
from oracle.rounding import round_storage
from paper_2502_01277_amd import zoo


@pytest.mark.parametrize("h,w,c,k,ksz,stride,pad", [
    (5, 7, 3, 4, 3, 1, 1), (5, 7, 3, 4, 3, 2, 1), (6, 5, 2, 3, 1, 1, 0), (9, 8, 3, 2, 7, 2, 3),
    (8, 8, 3, 2, 6, 2, 2), (4, 4, 5, 3, 3, 2, 0), (7, 6, 2, 2, 1, 2, 0),
])
def test_conv_equals_brute_force(h, w, c, k, ksz, stride, pad):
    rng = np.random.default_rng(h * 100 + w * 10 + ksz)
    x = rng.standard_normal((2, h, w, c))
    wt = rng.standard_normal((k, ksz, ksz, c))
    assert np.allclose(nn.conv2d(x, wt, stride, pad), nn.direct_conv(x, wt, stride, pad), atol=1e-10, rtol=0)


def test_conv_is_cross_correlation_not_flipped():
    # asymmetric kernel: a single 1 at (r, s) = (0, 2) shifts the image by (-1, +1) with zero fill
    x = np.arange(2 * 4 * 5 * 1, dtype=np.float64).reshape(2, 4, 5, 1)
    w = np.zeros((1, 3, 3, 1)); w[0, 0, 2, 0] = 1.0
    y = nn.conv2d(x, w, 1, 1)
    exp = np.zeros_like(x)
    exp[:, 1:, :-1] = x[:, :-1, 1:]       # y[p,q] = x[p-1, q+1]
    assert np.array_equal(y, exp)


def test_conv_delta_is_identity_and_ones_is_box_count():
    x = np.random.default_rng(0).standard_normal((1, 6, 7, 2))
    w = np.zeros((2, 3, 3, 2)); w[0, 1, 1, 0] = 1; w[1, 1, 1, 1] = 1
    assert np.allclose(nn.conv2d(x, w, 1, 1), x, atol=1e-12)
    ones = np.ones((1, 6, 7, 1))
    y = nn.conv2d(ones, np.ones((1, 3, 3, 1)), 1, 1)[0, :, :, 0]
    rows = np.array([2, 3, 3, 3, 3, 2]); cols = np.array([2, 3, 3, 3, 3, 3, 2])
    assert np.array_equal(y, np.outer(rows, cols).astype(float))
    # stride 2, pad 1, 5x5 input: taps rows {-1,0,1},{1,2,3},{3,4,5} -> valid counts 2,3,2
    y2 = nn.conv2d(np.ones((1, 5, 5, 1)), np.ones((1, 3, 3, 1)), 2, 1)[0, :, :, 0]
    assert np.array_equal(y2, np.outer([2, 3, 2], [2, 3, 2]).astype(float))


def test_conv_linearity_and_1x1_is_matmul():
    rng = np.random.default_rng(1)
    x, y = rng.standard_normal((2, 1, 5, 5, 3))
    w = rng.standard_normal((4, 3, 3, 3))
    lhs = nn.conv2d(2.5 * x - 1.5 * y, w, 2, 1)
    assert np.allclose(lhs, 2.5 * nn.conv2d(x, w, 2, 1) - 1.5 * nn.conv2d(y, w, 2, 1), atol=1e-10)
    w1 = rng.standard_normal((4, 1, 1, 3))
    out = nn.conv2d(x, w1, 1, 0)
    ref = np.zeros((1, 5, 5, 4))
    for p in range(5):
        for q in range(5):
            for k in range(4):
                ref[0, p, q, k] = sum(x[0, p, q, c] * w1[k, 0, 0, c] for c in range(3))
    assert np.allclose(out, ref, atol=1e-12)


def test_maxpool_brute_force_and_padding():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((1, 6, 5, 2)) - 5.0          # all negative: zero padding would be wrong
    for k, s, p in ((5, 1, 2), (3, 2, 1)):
        y = nn.maxpool(x, k, s, p)
        ho, wo = (6 + 2 * p - k) // s + 1, (5 + 2 * p - k) // s + 1
        assert y.shape == (1, ho, wo, 2)
        for a in range(ho):
            for b in range(wo):
                ys = [t for t in range(a * s - p, a * s - p + k) if 0 <= t < 6]
                xs = [t for t in range(b * s - p, b * s - p + k) if 0 <= t < 5]
                assert np.array_equal(y[0, a, b], x[0][np.ix_(ys, xs)].max(axis=(0, 1)))


def test_activations_closed_form():
    v = np.array([-2.0, 0.0, 1.0, 3.0])
    assert np.array_equal(nn.activation(v, nn.ACT_RELU), [0, 0, 1, 3])
    assert np.allclose(nn.activation(v, nn.ACT_SILU),
                       [-2 / (1 + np.e ** 2), 0.0, 1 / (1 + 1 / np.e), 3 / (1 + np.e ** -3)], atol=1e-15)
    assert np.array_equal(nn.activation(v, nn.ACT_NONE), v)


def test_round_storage_matches_library_and_avoids_double_rounding():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(20000) * 10 ** rng.uniform(-3, 3, 20000)).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(round_storage(x.astype(np.float64), "bf16"), ref)
    assert np.array_equal(zoo.round_to_dtype(x, "bf16"), ref)
    assert np.array_equal(round_storage(x.astype(np.float64), "f16"), x.astype(np.float16).astype(np.float32))
    # 1 + 2^-8 is a bf16 tie (-> 1.0, even); a hair above must go up, a hair below stays
    tie = 1.0 + 2.0 ** -8
    assert round_storage(np.array([tie]), "bf16")[0] == 1.0
    assert round_storage(np.array([tie + 2.0 ** -30]), "bf16")[0] == np.float32(1.0 + 2.0 ** -7)
    assert round_storage(np.array([tie - 2.0 ** -30]), "bf16")[0] == 1.0
    assert round_storage(np.array([-(tie + 2.0 ** -30)]), "bf16")[0] == np.float32(-(1.0 + 2.0 ** -7))
    t3 = 1.0 + 3 * 2.0 ** -8                                 # tie between 1+2^-7 (odd) and 1+2^-6 (even)
    assert round_storage(np.array([t3]), "bf16")[0] == np.float32(1.0 + 2.0 ** -6)
    assert round_storage(np.array([t3 - 2.0 ** -30]), "bf16")[0] == np.float32(1.0 + 2.0 ** -7)


def _toy_model(dtype, res_mode, act):
    rng = np.random.default_rng(4)
    m = zoo.ModelSpec("toy", dtype, 6, 6, "classifier")
    w1 = zoo.round_to_dtype(rng.standard_normal((3, 3, 3, 3)).astype(np.float32) * 0.3, dtype)
    w2 = zoo.round_to_dtype(rng.standard_normal((3, 3, 3, 3)).astype(np.float32) * 0.3, dtype)
    b1 = rng.uniform(-0.1, 0.1, 3).astype(np.float32)
    b2 = rng.uniform(-0.1, 0.1, 3).astype(np.float32)
    m.layers = [zoo.Layer("conv", [0], cout=3, kh=3, kw=3, stride=1, pad=1, act=act, weight=w1, bias=b1),
                zoo.Layer("conv", [1, 0], cout=3, kh=3, kw=3, stride=1, pad=1, act=act, res_mode=res_mode,
                          weight=w2, bias=b2)]
    m.outputs = [2]
    return m, (w1, b1, w2, b2)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("res_mode", [zoo.RES_BEFORE_ACT, zoo.RES_AFTER_ACT])
def test_graph_residual_order_and_rounding_points(dtype, res_mode):
    m, (w1, b1, w2, b2) = _toy_model(dtype, res_mode, zoo.ACT_SILU)
    x = zoo.round_to_dtype(np.random.default_rng(5).uniform(0, 1, (1, 6, 6, 3)).astype(np.float32), dtype)
    ts = nn.run_model(m, x, keep_all=True)
    silu = lambda v: v / (1 + np.exp(-v))
    t1 = round_storage(silu(nn.direct_conv(x, w1, 1, 1) + b1), dtype)
    pre = nn.direct_conv(t1, w2, 1, 1) + b2
    t2 = silu(pre + x) if res_mode == zoo.RES_BEFORE_ACT else silu(pre) + x
    t2 = round_storage(t2, dtype)
    assert np.array_equal(ts[1], t1)
    assert np.array_equal(ts[2], t2)
    assert np.array_equal(zoo.round_to_dtype(ts[2], dtype), ts[2])      # stored values are representable


def test_graph_glue_ops():
    m = zoo.ModelSpec("glue", "f32", 4, 4, "classifier")
    rng = np.random.default_rng(6)
    wfc = rng.standard_normal((5, 1, 1, 6)).astype(np.float32)
    bfc = rng.standard_normal(5).astype(np.float32)
    m.layers = [zoo.Layer("maxpool", [0], kh=3, kw=3, stride=2, pad=1),      # t1: 2x2x3
                zoo.Layer("upsample2x", [1]),                                # t2: 4x4x3
                zoo.Layer("concat", [2, 0]),                                 # t3: 4x4x6
                zoo.Layer("add", [3, 3], act=zoo.ACT_RELU),                  # t4
                zoo.Layer("gap", [4]),                                       # t5: 1x1x6
                zoo.Layer("fc", [5], cout=5, weight=wfc, bias=bfc)]          # t6
    m.outputs = [6]
    x = rng.standard_normal((2, 4, 4, 3)).astype(np.float32)
    ts = nn.run_model(m, x, keep_all=True)
    assert m.tensor_shapes()[1:] == [(2, 2, 3), (4, 4, 3), (4, 4, 6), (4, 4, 6), (1, 1, 6), (1, 1, 5)]
    for y in range(4):
        for xx in range(4):
            assert np.array_equal(ts[2][:, y, xx], ts[1][:, y // 2, xx // 2])
    assert np.array_equal(ts[3][..., :3], ts[2]) and np.array_equal(ts[3][..., 3:], x)
    assert np.array_equal(ts[4], np.maximum(2 * ts[3], 0))
    gap = np.zeros((2, 6))
    for n in range(2):
        for c in range(6):
            gap[n, c] = sum(float(ts[4][n, a, b, c]) for a in range(4) for b in range(4)) / 16.0
    assert np.allclose(ts[5].reshape(2, 6), gap, atol=1e-6)
    fc = ts[5].reshape(2, 6).astype(np.float64) @ wfc.reshape(5, 6).T.astype(np.float64) + bfc
    assert np.allclose(ts[6].reshape(2, 5), fc, atol=1e-6)
    lab = nn.argmax_labels(np.array([[1.0, 3.0, 3.0], [2.0, 2.0, 1.0]], np.float32))
    assert lab.tolist() == [1, 0]                    # ties -> lowest index


def test_zoo_shapes():
    det = zoo.traffic_cascade().models[0]
    shp = det.tensor_shapes()
    assert [shp[t] for t in det.outputs] == [(80, 80, 255), (40, 40, 255), (20, 20, 255)]
    assert det.n_cand() == 25200
    assert 14e9 < det.flops_per_item() < 19e9
    r18 = zoo.traffic_cascade().models[1]
    assert r18.tensor_shapes()[-1] == (1, 1, 1000) and 3.2e9 < r18.flops_per_item() < 4.0e9
    hi = zoo.hires_cascade().models[0]
    assert [hi.tensor_shapes()[t][:2] for t in hi.outputs] == [(160, 160), (80, 80), (40, 40)]
    assert hi.n_cand() == 100800
    tiny = zoo.tiny_cascade()
    assert tiny.models[0].tensor_shapes()[-1] == (20, 20, 39) and tiny.models[0].n_cand() == 1200
    r50 = zoo.surveillance_cascade().models[1]
    assert r50.tensor_shapes()[-1] == (1, 1, 32) and 4.5e9 < r50.flops_per_item() < 6.5e9


def test_sampled_layer_evaluation_equals_the_full_layer():
    """conv_layer_at is the layer definition restricted to chosen output positions: it must reproduce run_model's
    tensor there, borders, stride and residual included."""
    from paper_2502_01277_amd import zoo
    rng = np.random.default_rng(5)
    B = zoo._Builder("t", "bf16", 11, 9, "classifier", rng)
    B.ch = [6]
    B.m.in_c = 6
    a = B.conv(0, 10, 3, 2, 1, act=zoo.ACT_SILU)
    b = B.conv(a, 10, 3, 1, 1, act=zoo.ACT_RELU, res=a, res_mode=zoo.RES_BEFORE_ACT)
    B.m.outputs = [B.fc(B.gap(b), 4)]
    x = zoo.round_to_dtype(rng.uniform(-1, 1, (2, 11, 9, 6)).astype(np.float32), "bf16")
    ts = nn.run_model(B.m, x, keep_all=True)
    pos = [(0, 0, 0), (1, 5, 4), (0, 3, 2), (1, 0, 4), (1, 5, 0)]
    got1 = nn.conv_layer_at(ts[0], B.m.layers[0], "bf16", pos)
    got2 = nn.conv_layer_at(ts[1], B.m.layers[1], "bf16", pos, res=ts[1])
    for j, (n, p, q) in enumerate(pos):
        assert np.array_equal(got1[j], ts[1][n, p, q])
        assert np.array_equal(got2[j], ts[2][n, p, q])
