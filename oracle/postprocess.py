"""Oracle: detector post-processing - decode + threshold, top-k, class-wise NMS,
ROI compaction (test infrastructure).

The paper only says a detector emits bounding boxes whose count varies per frame
(Sec. III-B, Observation 1); the definitions here are the plain ones.  The
decisions (threshold, ordering, suppression) are taken in fp32 with every
operation rounded on its own, because an integer result hangs on them.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

f32 = np.float32


@dataclass
class Candidates:
    box: np.ndarray     # fp32 [n][4]  x1, y1, x2, y2 (letterbox pixels, not clamped)
    score: np.ndarray   # fp32 [n]
    cls: np.ndarray     # int32 [n]
    idx: np.ndarray     # int32 [n]  candidate index (level offset + (gy*G + gx)*A + a)

    def __len__(self):
        return len(self.score)

    def take(self, sel):
        sel = np.asarray(sel, dtype=np.int64)
        return Candidates(self.box[sel], self.score[sel], self.cls[sel], self.idx[sel])


def _sigmoid32(z: np.ndarray) -> np.ndarray:
    z = z.astype(f32)
    return (f32(1.0) / (f32(1.0) + np.exp(-z))).astype(f32)


def decode_frame(heads, spec) -> Candidates:
    """heads: per level fp32 [G][G][A*(5+C)] (one frame).  Returns candidates with score > thr, ascending idx.

    For logits t of a candidate at cell (gx, gy), anchor a, level l:
      cx = (2 s(t0) - 0.5 + gx) * stride,  cy likewise,
      w  = (2 s(t2))^2 * anchor_w,         h likewise,
      cls = argmax_c t[5+c] (lowest index on ties), score = s(t4) * s(t[5+cls]),
    with s the logistic function; kept iff score > thr (strict).
    """
    A, C = spec.n_anchors, spec.n_classes
    no = 5 + C
    boxes, scores, clss, idxs = [], [], [], []
    off = 0
    for l, h in enumerate(heads):
        gh, gw = h.shape[0], h.shape[1]
        t = np.asarray(h, f32).reshape(gh, gw, A, no)
        stride = f32(spec.strides[l])
        gy, gx = np.meshgrid(np.arange(gh, dtype=f32), np.arange(gw, dtype=f32), indexing="ij")
        s = _sigmoid32(t[..., :5])
        cx = ((f32(2.0) * s[..., 0] - f32(0.5)) + gx[..., None]) * stride
        cy = ((f32(2.0) * s[..., 1] - f32(0.5)) + gy[..., None]) * stride
        aw = spec.anchors[l, :, 0].astype(f32)[None, None, :]
        ah = spec.anchors[l, :, 1].astype(f32)[None, None, :]
        tw = f32(2.0) * s[..., 2]
        th = f32(2.0) * s[..., 3]
        w = (tw * tw) * aw
        hh = (th * th) * ah
        hw, hh2 = w * f32(0.5), hh * f32(0.5)
        cls = np.argmax(t[..., 5:], axis=-1)
        cl = np.take_along_axis(t[..., 5:], cls[..., None], axis=-1)[..., 0]
        score = (s[..., 4] * _sigmoid32(cl)).astype(f32)
        keep = score > f32(spec.score_thr)
        idx = off + (np.arange(gh * gw * A)).reshape(gh, gw, A)
        b = np.stack([cx - hw, cy - hh2, cx + hw, cy + hh2], axis=-1).astype(f32)
        boxes.append(b[keep]); scores.append(score[keep]); clss.append(cls[keep]); idxs.append(idx[keep])
        off += gh * gw * A
    return Candidates(np.concatenate(boxes).reshape(-1, 4), np.concatenate(scores),
                      np.concatenate(clss).astype(np.int32), np.concatenate(idxs).astype(np.int32))


def topk(c: Candidates, k: int) -> Candidates:
    """The k best candidates in the total order (score descending, idx ascending)."""
    order = sorted(range(len(c)), key=lambda i: (-float(c.score[i]), int(c.idx[i])))
    return c.take(order[:k])


def box_area(b: np.ndarray) -> np.ndarray:
    return ((b[..., 2] - b[..., 0]) * (b[..., 3] - b[..., 1])).astype(f32)


def suppresses(a_box, a_cls, b_box, b_cls, iou_thr) -> np.ndarray:
    """True where box a suppresses box(es) b: same class and inter > iou_thr * union (fp32, no division)."""
    a_box = np.asarray(a_box, f32)
    b_box = np.asarray(b_box, f32)
    iw = np.maximum(f32(0), np.minimum(a_box[..., 2], b_box[..., 2]) - np.maximum(a_box[..., 0], b_box[..., 0]))
    ih = np.maximum(f32(0), np.minimum(a_box[..., 3], b_box[..., 3]) - np.maximum(a_box[..., 1], b_box[..., 1]))
    inter = (iw * ih).astype(f32)
    uni = ((box_area(a_box) + box_area(b_box)).astype(f32) - inter).astype(f32)
    return (np.asarray(a_cls) == np.asarray(b_cls)) & (inter > (f32(iou_thr) * uni).astype(f32))


def nms(c: Candidates, iou_thr: float, max_det: int) -> np.ndarray:
    """Greedy class-wise NMS over candidates already in top-k order.

    Box i is kept iff no kept box j < i suppresses it; the keep-list (positions
    in c, ascending) is cut to max_det.
    """
    kept = []
    for i in range(len(c)):
        if kept:
            kk = np.asarray(kept)
            if suppresses(c.box[kk], c.cls[kk], c.box[i], c.cls[i], iou_thr).any():
                continue
        kept.append(i)
    return np.asarray(kept[:max_det], dtype=np.int32)


@dataclass
class RoiTable:
    frame: np.ndarray   # int32 [n] position of the source frame in the batch
    rank: np.ndarray    # int32 [n] position in that frame's keep-list
    cls: np.ndarray     # int32 [n]
    box: np.ndarray     # fp32 [n][4] source pixels, clamped to the frame

    def __len__(self):
        return len(self.frame)


def to_source_box(box_lb: np.ndarray, src_h, src_w, nw, nh, left, top) -> np.ndarray:
    """Undo the letterbox: X = (x - left) / (nw / Ws), Y = (y - top) / (nh / Hs); clamp to [0,Ws] x [0,Hs]; fp32."""
    b = np.asarray(box_lb, f32).reshape(-1, 4)
    rx = f32(nw) / f32(src_w)
    ry = f32(nh) / f32(src_h)
    out = np.empty_like(b)
    out[:, 0] = np.clip((b[:, 0] - f32(left)) / rx, f32(0), f32(src_w))
    out[:, 2] = np.clip((b[:, 2] - f32(left)) / rx, f32(0), f32(src_w))
    out[:, 1] = np.clip((b[:, 1] - f32(top)) / ry, f32(0), f32(src_h))
    out[:, 3] = np.clip((b[:, 3] - f32(top)) / ry, f32(0), f32(src_h))
    return out.astype(f32)


def compact_rois(kept_per_frame, class_mask: int) -> RoiTable:
    """kept_per_frame: list over frames of (cls int32 [k], box_src fp32 [k][4]) in keep-list order.

    Emits, frame by frame and rank by rank, every kept box whose class bit is set
    in class_mask; the ROI id is the running count.
    """
    fr, rk, cl, bx = [], [], [], []
    for f, (cls, box) in enumerate(kept_per_frame):
        for r in range(len(cls)):
            if (class_mask >> int(cls[r])) & 1:
                fr.append(f); rk.append(r); cl.append(int(cls[r])); bx.append(box[r])
    return RoiTable(np.asarray(fr, np.int32), np.asarray(rk, np.int32), np.asarray(cl, np.int32),
                    np.asarray(bx, f32).reshape(-1, 4))
