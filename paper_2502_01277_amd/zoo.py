"""Model-graph tables and seeded random-init weights for the synthetic workloads.

This module is an *input generator*: it describes layer graphs (shapes, strides,
which tensor feeds which layer) and draws weights from a seed.  It holds none of
the inference arithmetic; both the CPU oracle and the HIP path consume the
`ModelSpec` objects it returns.

The paper runs trained detectors and classifiers inside a black-box engine
(Sec. III-A, step 4) and names only the model families (Sec. IV-A); the layer
tables below are this project's own, sized to the widths / grids the workloads
call for.  Weights are random (no trained weights exist here).

Graph convention: tensor 0 is the model input (NHWC, 3 channels); layer i
(0-based) produces tensor i+1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

ACT_NONE, ACT_RELU, ACT_SILU = 0, 1, 2
RES_NONE, RES_BEFORE_ACT, RES_AFTER_ACT = 0, 1, 2

OPS = ("conv", "maxpool", "upsample2x", "concat", "add", "gap", "fc")


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values once (nearest-even) to the storage type, return as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(x.shape)
    raise ValueError(dtype)


@dataclass
class Layer:
    op: str
    inputs: List[int]
    cout: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    act: int = ACT_NONE
    res_mode: int = RES_NONE          # conv only: inputs[1] is a residual tensor
    weight: Optional[np.ndarray] = None   # conv: [cout][kh][kw][cin]; fc: [cout][1][1][cin]; fp32 holding T-representable values
    bias: Optional[np.ndarray] = None     # fp32 [cout]


@dataclass
class ModelSpec:
    name: str
    dtype: str                     # 'f32' | 'f16' | 'bf16' (storage type T of activations and weights)
    in_h: int
    in_w: int
    kind: str                      # 'detector' | 'classifier'
    layers: List[Layer] = field(default_factory=list)
    outputs: List[int] = field(default_factory=list)   # detector: head tensors, largest grid first; classifier: logits tensor
    # detector post-processing
    n_classes: int = 0
    n_anchors: int = 3
    grids: List[int] = field(default_factory=list)      # per level (square grids; gh = in_h/stride, gw = in_w/stride)
    strides: List[int] = field(default_factory=list)
    anchors: Optional[np.ndarray] = None                # [levels][A][2] (w, h) in input pixels, fp32
    score_thr: float = 0.25
    iou_thr: float = 0.45
    topk: int = 1000
    max_det: int = 300
    # pre-processing
    norm_scale: tuple = (1.0 / 255.0,) * 3
    norm_bias: tuple = (0.0, 0.0, 0.0)
    pad_value: int = 114
    batch_size: int = 1
    in_c: int = 3

    def n_cand(self) -> int:
        return sum(self.n_anchors * (self.in_h // s) * (self.in_w // s) for s in self.strides)

    def tensor_shapes(self):
        """(h, w, c) of every tensor, by walking the graph (shape bookkeeping only)."""
        shp = [(self.in_h, self.in_w, self.in_c)]
        for L in self.layers:
            h, w, c = shp[L.inputs[0]]
            if L.op == "conv":
                ho = (h + 2 * L.pad - L.kh) // L.stride + 1
                wo = (w + 2 * L.pad - L.kw) // L.stride + 1
                shp.append((ho, wo, L.cout))
            elif L.op == "maxpool":
                ho = (h + 2 * L.pad - L.kh) // L.stride + 1
                wo = (w + 2 * L.pad - L.kw) // L.stride + 1
                shp.append((ho, wo, c))
            elif L.op == "upsample2x":
                shp.append((2 * h, 2 * w, c))
            elif L.op == "concat":
                shp.append((h, w, sum(shp[i][2] for i in L.inputs)))
            elif L.op == "add":
                shp.append((h, w, c))
            elif L.op == "gap":
                shp.append((1, 1, c))
            elif L.op == "fc":
                shp.append((1, 1, L.cout))
            else:
                raise ValueError(L.op)
        return shp

    def flops_per_item(self) -> float:
        """Dense multiply-add count x2 of all conv / fc layers for one input item."""
        shp = self.tensor_shapes()
        tot = 0.0
        for i, L in enumerate(self.layers):
            if L.op in ("conv", "fc"):
                ho, wo, co = shp[i + 1]
                cin = shp[L.inputs[0]][2]
                tot += 2.0 * ho * wo * co * cin * L.kh * L.kw
        return tot


@dataclass
class Edge:
    parent: int
    child: int
    class_mask: int = (1 << 128) - 1   # bit c set: ROIs of class c are routed to the child


@dataclass
class PipelineSpec:
    name: str
    models: List[ModelSpec]
    edges: List[Edge]
    slo_ms: float
    src_h: int
    src_w: int
    max_frames: int               # largest detector batch
    max_rois_per_frame: int


class _Builder:
    def __init__(self, name, dtype, in_h, in_w, kind, rng):
        self.m = ModelSpec(name=name, dtype=dtype, in_h=in_h, in_w=in_w, kind=kind)
        self.rng = rng
        self.ch = [3]

    def _push(self, layer, c):
        self.m.layers.append(layer)
        self.ch.append(c)
        return len(self.ch) - 1

    def conv(self, x, cout, k, s=1, p=None, act=ACT_SILU, res=None, res_mode=RES_NONE,
             gain=2.0, wscale=1.0, bias_fill=None):
        cin = self.ch[x]
        p = k // 2 if p is None else p
        std = np.sqrt(gain / (cin * k * k)) * wscale
        w = self.rng.standard_normal((cout, k, k, cin), dtype=np.float32) * np.float32(std)
        b = self.rng.uniform(-0.1, 0.1, size=cout).astype(np.float32)
        if bias_fill is not None:
            b = bias_fill(b)
        ins = [x] if res is None else [x, res]
        L = Layer("conv", ins, cout=cout, kh=k, kw=k, stride=s, pad=p, act=act,
                  res_mode=res_mode if res is not None else RES_NONE,
                  weight=round_to_dtype(w, self.m.dtype), bias=b)
        return self._push(L, cout)

    def maxpool(self, x, k, s, p):
        return self._push(Layer("maxpool", [x], kh=k, kw=k, stride=s, pad=p), self.ch[x])

    def up(self, x):
        return self._push(Layer("upsample2x", [x]), self.ch[x])

    def cat(self, xs):
        return self._push(Layer("concat", list(xs)), sum(self.ch[i] for i in xs))

    def add(self, a, b, act=ACT_NONE):
        return self._push(Layer("add", [a, b], act=act), self.ch[a])

    def gap(self, x):
        return self._push(Layer("gap", [x]), self.ch[x])

    def fc(self, x, cout):
        cin = self.ch[x]
        w = self.rng.standard_normal((cout, 1, 1, cin), dtype=np.float32) * np.float32(np.sqrt(1.0 / cin))
        b = self.rng.uniform(-0.1, 0.1, size=cout).astype(np.float32)
        L = Layer("fc", [x], cout=cout, weight=round_to_dtype(w, self.m.dtype), bias=b)
        return self._push(L, cout)


def _default_anchors(strides, rng):
    a = np.zeros((len(strides), 3, 2), np.float32)
    for l, s in enumerate(strides):
        for j, mul in enumerate((1.25, 2.5, 5.0)):
            asp = float(rng.uniform(0.6, 1.6))
            a[l, j, 0] = np.float32(round(s * mul * np.sqrt(asp)))
            a[l, j, 1] = np.float32(round(s * mul / np.sqrt(asp)))
    return a


def _head_bias(n_anchors, n_out, obj_bias):
    def f(b):
        b = b.copy()
        for a in range(n_anchors):
            b[a * n_out + 4] += np.float32(obj_bias)
        return b
    return f


def csp_detector(name, dtype, size, widths, depths, n_classes, seed, batch_size=8,
                 score_thr=0.25, iou_thr=0.45, topk=1000, max_det=300):
    """CSP-backbone + PAN-neck detector with three heads (strides 8/16/32).

    widths = five channel counts (stem .. deepest); depths = bottleneck repeats
    of the four backbone CSP blocks.  The shape mix (not fidelity to any trained
    network) is what the workload needs.
    """
    rng = np.random.default_rng(seed)
    B = _Builder(name, dtype, size, size, "detector", rng)
    w0, w1, w2, w3, w4 = widths

    def csp(x, cout, n, shortcut):
        ch = cout // 2
        a = B.conv(x, ch, 1)
        b = B.conv(x, ch, 1)
        for _ in range(n):
            t = B.conv(a, ch, 1)
            if shortcut:
                a = B.conv(t, ch, 3, res=a, res_mode=RES_AFTER_ACT, wscale=0.25)
            else:
                a = B.conv(t, ch, 3)
        return B.conv(B.cat([a, b]), cout, 1)

    x = B.conv(0, w0, 6, 2, 2)
    x = B.conv(x, w1, 3, 2)
    x = csp(x, w1, depths[0], True)
    x = B.conv(x, w2, 3, 2)
    p3 = csp(x, w2, depths[1], True)
    x = B.conv(p3, w3, 3, 2)
    p4 = csp(x, w3, depths[2], True)
    x = B.conv(p4, w4, 3, 2)
    x = csp(x, w4, depths[3], True)
    # spatial pyramid pooling (three chained 5x5 max-pools)
    h = B.conv(x, w4 // 2, 1)
    y1 = B.maxpool(h, 5, 1, 2)
    y2 = B.maxpool(y1, 5, 1, 2)
    y3 = B.maxpool(y2, 5, 1, 2)
    x = B.conv(B.cat([h, y1, y2, y3]), w4, 1)
    # top-down
    nd = depths[0]
    t5 = B.conv(x, w3, 1)
    x = csp(B.cat([B.up(t5), p4]), w3, nd, False)
    t4 = B.conv(x, w2, 1)
    n3 = csp(B.cat([B.up(t4), p3]), w2, nd, False)
    # bottom-up
    x = B.conv(n3, w2, 3, 2)
    n4 = csp(B.cat([x, t4]), w3, nd, False)
    x = B.conv(n4, w3, 3, 2)
    n5 = csp(B.cat([x, t5]), w4, nd, False)
    n_out = 5 + n_classes
    hb = _head_bias(3, n_out, -2.0)
    heads = [B.conv(t, 3 * n_out, 1, act=ACT_NONE, gain=1.0, bias_fill=hb) for t in (n3, n4, n5)]
    m = B.m
    m.outputs = heads
    m.n_classes = n_classes
    m.strides = [8, 16, 32]
    m.grids = [size // 8, size // 16, size // 32]
    m.anchors = _default_anchors(m.strides, rng)
    m.score_thr, m.iou_thr, m.topk, m.max_det = score_thr, iou_thr, topk, max_det
    m.batch_size = batch_size
    return m


def plain_detector(name, dtype, size, widths, n_classes, seed, act=ACT_RELU, batch_size=1,
                   score_thr=0.25, iou_thr=0.45, topk=100, max_det=100, obj_bias=0.0):
    """Stack of 3x3 stride-2 convolutions and one 1x1 head (single level)."""
    rng = np.random.default_rng(seed)
    B = _Builder(name, dtype, size, size, "detector", rng)
    x = 0
    for w in widths:
        x = B.conv(x, w, 3, 2, act=act)
    n_out = 5 + n_classes
    head = B.conv(x, 3 * n_out, 1, act=ACT_NONE, gain=1.0, bias_fill=_head_bias(3, n_out, obj_bias))
    m = B.m
    stride = 2 ** len(widths)
    m.outputs = [head]
    m.n_classes = n_classes
    m.strides = [stride]
    m.grids = [size // stride]
    m.anchors = _default_anchors([stride], rng)
    m.score_thr, m.iou_thr, m.topk, m.max_det = score_thr, iou_thr, topk, max_det
    m.batch_size = batch_size
    return m


def plain_classifier(name, dtype, in_h, in_w, widths, n_out, seed, batch_size=1):
    """3x3 stride-2 conv stack, global average pool, fully connected."""
    rng = np.random.default_rng(seed)
    B = _Builder(name, dtype, in_h, in_w, "classifier", rng)
    x = 0
    for w in widths:
        x = B.conv(x, w, 3, 2, act=ACT_RELU)
    x = B.fc(B.gap(x), n_out)
    B.m.outputs = [x]
    B.m.batch_size = batch_size
    return B.m


def residual_classifier(name, dtype, in_h, in_w, block, counts, n_out, seed, batch_size=1):
    """7x7 s2 stem, 3x3 s2 max-pool, four residual stages, GAP, FC.

    block='basic': two 3x3 convs per block; block='bottleneck': 1x1-3x3-1x1 with
    4x channel expansion.  Shortcut is a 1x1 stride-s conv where shapes change.
    Batch-norm is taken as already folded into (weight, bias).
    """
    rng = np.random.default_rng(seed)
    B = _Builder(name, dtype, in_h, in_w, "classifier", rng)
    x = B.conv(0, 64, 7, 2, 3, act=ACT_RELU)
    x = B.maxpool(x, 3, 2, 1)
    cin = 64
    for si, (w, n) in enumerate(zip((64, 128, 256, 512), counts)):
        for bi in range(n):
            s = 2 if (bi == 0 and si > 0) else 1
            cout = w if block == "basic" else 4 * w
            sc = x
            if s != 1 or cin != cout:
                sc = B.conv(x, cout, 1, s, 0, act=ACT_NONE, gain=1.0)
            if block == "basic":
                t = B.conv(x, w, 3, s, act=ACT_RELU)
                x = B.conv(t, w, 3, 1, act=ACT_RELU, res=sc, res_mode=RES_BEFORE_ACT, wscale=0.25)
            else:
                t = B.conv(x, w, 1, 1, act=ACT_RELU)
                t = B.conv(t, w, 3, s, act=ACT_RELU)
                x = B.conv(t, cout, 1, 1, act=ACT_RELU, res=sc, res_mode=RES_BEFORE_ACT, wscale=0.25)
            cin = cout
    x = B.fc(B.gap(x), n_out)
    B.m.outputs = [x]
    B.m.batch_size = batch_size
    return B.m


# ---------------------------------------------------------------------------
# The five workloads.  `index` follows the order the workloads are listed in
# (1 = tiny fp32 cascade ... 5 = high-resolution heavy-tail case).
# ---------------------------------------------------------------------------
SEED0 = 20250201
S_WIDTHS, S_DEPTHS = (32, 64, 128, 256, 512), (1, 2, 3, 1)
M_WIDTHS, M_DEPTHS = (48, 96, 192, 384, 768), (2, 4, 6, 2)


def tiny_cascade(dtype="f32", seed=SEED0 + 1) -> PipelineSpec:
    det = plain_detector("tiny_det", dtype, 320, (16, 32, 64, 128), 8, seed, batch_size=2,
                         score_thr=0.25, iou_thr=0.45, topk=100, max_det=100)
    cls = plain_classifier("tiny_cls", dtype, 64, 64, (16, 32, 64), 10, seed + 100, batch_size=200)
    return PipelineSpec("tiny", [det, cls], [Edge(0, 1)], 200.0, 320, 320, 2, 100)


def traffic_cascade(dtype="f16", seed=SEED0 + 2, det_batch=8, max_rois_per_frame=64,
                    with_plate=True, src_hw=(1080, 1920)) -> PipelineSpec:
    det = csp_detector("traffic_det", dtype, 640, S_WIDTHS, S_DEPTHS, 80, seed, batch_size=det_batch,
                       topk=1000, max_det=max_rois_per_frame)
    cls = residual_classifier("vehicle_cls", dtype, 224, 224, "basic", (2, 2, 2, 2), 1000, seed + 100,
                              batch_size=det_batch * max_rois_per_frame)
    models, edges = [det, cls], [Edge(0, 1)]
    if with_plate:
        plate = plain_detector("plate_det", dtype, 128, (16, 32, 64, 128, 256), 1, seed + 200, act=ACT_SILU,
                               batch_size=det_batch * max_rois_per_frame, topk=48, max_det=8, obj_bias=-1.0)
        models.append(plate)
        edges.append(Edge(0, 2))
    return PipelineSpec("traffic", models, edges, 200.0, src_hw[0], src_hw[1], det_batch, max_rois_per_frame)


def sweep_cascade(det_batch, dtype="bf16", seed=SEED0 + 3) -> PipelineSpec:
    p = traffic_cascade(dtype, seed, det_batch=det_batch, max_rois_per_frame=200, with_plate=False)
    p.name = "sweep_bz%d" % det_batch
    return p


def surveillance_cascade(dtype="bf16", seed=SEED0 + 40, det_batch=8, max_rois_per_frame=64) -> PipelineSpec:
    det = csp_detector("people_det", dtype, 640, S_WIDTHS, S_DEPTHS, 80, seed, batch_size=det_batch,
                       topk=1000, max_det=max_rois_per_frame)
    attr = residual_classifier("attr_cls", dtype, 256, 128, "bottleneck", (3, 4, 6, 3), 32, seed + 100,
                               batch_size=det_batch * max_rois_per_frame)
    return PipelineSpec("surveillance", [det, attr], [Edge(0, 1)], 200.0, 1080, 1920, det_batch, max_rois_per_frame)


def detector_only(dtype="bf16", seed=SEED0 + 41, det_batch=8, max_rois_per_frame=64) -> PipelineSpec:
    det = csp_detector("plain_det", dtype, 640, S_WIDTHS, S_DEPTHS, 80, seed, batch_size=det_batch,
                       topk=1000, max_det=max_rois_per_frame)
    return PipelineSpec("detonly", [det], [], 200.0, 1080, 1920, det_batch, max_rois_per_frame)


def hires_cascade(dtype="bf16", seed=SEED0 + 5, det_batch=32, max_rois_per_frame=300,
                  src_hw=(2160, 3840)) -> PipelineSpec:
    det = csp_detector("hires_det", dtype, 1280, M_WIDTHS, M_DEPTHS, 80, seed, batch_size=det_batch,
                       topk=1000, max_det=max_rois_per_frame)
    cls = residual_classifier("roi_cls", dtype, 224, 224, "basic", (2, 2, 2, 2), 1000, seed + 100,
                              batch_size=det_batch * max_rois_per_frame)
    return PipelineSpec("hires", [det, cls], [Edge(0, 1)], 200.0, src_hw[0], src_hw[1], det_batch, max_rois_per_frame)
