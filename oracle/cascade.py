"""Oracle: the whole cascade for one batch of frames (test infrastructure).

Order of steps: letterbox -> detector layers -> decode + threshold -> top-k ->
class-wise NMS -> cut to max_det -> per-edge ROI compaction -> crop-resize ->
child model -> label.  The cascade shape (a detector feeding classifier /
detector children with a variable number of objects) is the paper's pipeline
DAG (Sec. II, Fig. 2); the per-stage definitions live in the sibling modules.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from . import nn, postprocess as pp, preprocess as pre


@dataclass
class FrameDetections:
    cand_count: int
    top: pp.Candidates            # top-k list (sorted)
    keep: np.ndarray              # positions in `top`, ascending, cut to max_det
    box_src: np.ndarray           # fp32 [n_keep][4] source pixels


@dataclass
class ChildResult:
    rois: pp.RoiTable
    crops: Optional[np.ndarray] = None        # fp32 [n][Hc][Wc][3]
    logits: Optional[np.ndarray] = None       # classifier: fp32 [n][n_out]
    labels: Optional[np.ndarray] = None       # int32 [n]  (classifier: argmax; detector child: number of kept boxes)
    heads: Optional[List[np.ndarray]] = None  # detector child
    dets: Optional[List[FrameDetections]] = None


@dataclass
class CascadeResult:
    lb: np.ndarray
    heads: List[np.ndarray]
    dets: List[FrameDetections]
    children: Dict[int, ChildResult] = field(default_factory=dict)   # keyed by edge index


def postprocess_heads(heads, spec) -> List[FrameDetections]:
    """heads: per level fp32 [N][G][G][A*(5+C)].  Decode, top-k and NMS per frame (boxes in model-input pixels)."""
    out = []
    for f in range(heads[0].shape[0]):
        cand = pp.decode_frame([h[f] for h in heads], spec)
        top = pp.topk(cand, spec.topk)
        keep = pp.nms(top, spec.iou_thr, spec.max_det)
        out.append(FrameDetections(len(cand), top, keep, top.box[keep]))
    return out


def run_detector(spec, x, planted_heads=None, keep_all=False):
    ts = nn.run_model(spec, x, keep_all=keep_all)
    heads = [ts[t] for t in spec.outputs]
    used = planted_heads if planted_heads is not None else heads
    return ts, heads, postprocess_heads(used, spec)


def run_cascade(pipe, frames: np.ndarray, planted_heads=None, max_child_rois: Optional[int] = None) -> CascadeResult:
    det = pipe.models[0]
    n, hs, ws, _ = frames.shape
    lb = pre.letterbox(frames, det.in_h, det.in_w, det.dtype, det.norm_scale, det.norm_bias, det.pad_value)
    _, heads, dets = run_detector(det, lb, planted_heads)
    _, nw, nh, left, top = pre.letterbox_geometry(hs, ws, det.in_h, det.in_w)
    for d in dets:
        d.box_src = pp.to_source_box(d.top.box[d.keep], hs, ws, nw, nh, left, top)
    res = CascadeResult(lb, heads, dets)
    for e, edge in enumerate(pipe.edges):
        if edge.parent != 0:
            raise NotImplementedError("cascades deeper than two levels")
        child = pipe.models[edge.child]
        rois = pp.compact_rois([(d.top.cls[d.keep], d.box_src) for d in dets], edge.class_mask)
        cr = ChildResult(rois)
        m = len(rois) if max_child_rois is None else min(len(rois), max_child_rois)
        cr.crops = pre.crop_resize(frames, rois.frame[:m], rois.box[:m], child.in_h, child.in_w, child.dtype,
                                   child.norm_scale, child.norm_bias)
        if m > 0:
            ts = nn.run_model(child, cr.crops)
            if child.kind == "classifier":
                cr.logits = ts[child.outputs[0]].reshape(m, -1)
                cr.labels = nn.argmax_labels(cr.logits)
            else:
                cr.heads = [ts[t] for t in child.outputs]
                cr.dets = postprocess_heads(cr.heads, child)
                cr.labels = np.asarray([len(d.keep) for d in cr.dets], np.int32)
        else:
            cr.labels = np.zeros((0,), np.int32)
        res.children[e] = cr
    return res
