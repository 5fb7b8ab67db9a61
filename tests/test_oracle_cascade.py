"""Pins of the oracle's cascade composition (`oracle.cascade.run_cascade`): which detections survive, how they are
mapped back to source pixels, which of them an edge's class mask routes to the child and in what order, and what the
child sees.  The expected values are worked out by hand from the decode formula at zero box logits (centre of the
cell, anchor-sized box) and the letterbox geometry of a 48 x 64 frame inside a 32 x 32 input (scale 1/2, 4 rows of
padding above and below)."""
import numpy as np

from oracle import cascade, preprocess as pre
from paper_2502_01277_amd import zoo


def _spec(class_mask):
    det = zoo.plain_detector("d", "f32", 32, (8,), 2, seed=1, topk=10, max_det=3)          # one level, stride 2, grid 16, 3 anchors x (5 + 2)
    det.anchors = np.array([[[4, 4], [8, 6], [10, 10]]], np.float32)
    cls = zoo.plain_classifier("c", "f32", 8, 8, (4,), 3, seed=2)
    return zoo.PipelineSpec("p", [det, cls], [zoo.Edge(0, 1, class_mask)], 200.0, 48, 64, 2, 4)


def _plant(head, f, gy, gx, a, obj, cls, c_logit=9.0):
    """Box logits 0 (centre (g + 0.5) * stride, size = anchor), objectness `obj`, one class at +c_logit."""
    t = head[f, gy, gx].reshape(3, 7)
    t[a, :4] = 0.0
    t[a, 4] = obj
    t[a, 5:] = -9.0
    t[a, 5 + cls] = c_logit


def test_hand_built_two_frame_cascade():
    head = np.full((2, 16, 16, 21), -9.0, np.float32)
    head.reshape(2, 16, 16, 3, 7)[..., :4] = 0.0
    # frame 0: A (class 0, cell (4,4), anchor 1, the best), B (class 0, cell (4,5), anchor 1: overlaps A -> suppressed),
    #          C (class 1, cell (4,4), anchor 2: overlaps A but another class -> kept), D (class 0, cell (12,10), anchor 0 -> kept)
    _plant(head, 0, 4, 4, 1, 6.0, 0)
    _plant(head, 0, 4, 5, 1, 4.0, 0)
    _plant(head, 0, 4, 4, 2, 5.0, 1)
    _plant(head, 0, 12, 10, 0, 3.0, 0)
    # frame 1: E (class 1, cell (8,8), anchor 0), F (class 0, cell (2,13), anchor 2), G: objectness too low to pass 0.25
    _plant(head, 1, 8, 8, 0, 5.0, 1)
    _plant(head, 1, 2, 13, 2, 2.0, 0)
    _plant(head, 1, 9, 3, 1, -3.0, 0)
    frames = np.random.default_rng(0).integers(0, 256, (2, 48, 64, 3), dtype=np.uint8)
    spec = _spec(class_mask=0b01)                                    # only class 0 goes to the child
    res = cascade.run_cascade(spec, frames, planted_heads=[head])
    assert pre.letterbox_geometry(48, 64, 32, 32)[1:] == (32, 24, 0, 4)
    # frame 0: candidates A, B, C, D; order by score: A (6), C (5), B (4), D (3); B falls to A (IoU of 8x6 boxes 2 px apart:
    # 6*6 / (96 - 36) = 0.6 > 0.45), C overlaps A (10x10 around the same centre contains it: 48/100 > 0.45) but has class 1
    d0, d1 = res.dets
    assert d0.cand_count == 4 and d0.top.cls.tolist() == [0, 1, 0, 0] and d0.keep.tolist() == [0, 1, 3]
    assert d1.cand_count == 2 and d1.top.cls.tolist() == [1, 0] and d1.keep.tolist() == [0, 1]
    # boxes in the detector's input: centre (2 g + 1), size = anchor; in source pixels: x * 2, (y - 4) * 2, clamped to the frame
    A = [(9 - 4) * 2, (9 - 3 - 4) * 2, (9 + 4) * 2, (9 + 3 - 4) * 2]                       # [10, 4, 26, 16]
    Cb = [(9 - 5) * 2, max(0, (9 - 5 - 4) * 2), (9 + 5) * 2, (9 + 5 - 4) * 2]              # [8, 0, 28, 20]
    D = [(21 - 2) * 2, (25 - 2 - 4) * 2, (21 + 2) * 2, (25 + 2 - 4) * 2]                   # [38, 38, 46, 46]
    E = [(17 - 2) * 2, (17 - 2 - 4) * 2, (17 + 2) * 2, (17 + 2 - 4) * 2]                   # [30, 22, 38, 30]
    F = [(27 - 5) * 2, max(0, (5 - 5 - 4) * 2), min(64, (27 + 5) * 2), (5 + 5 - 4) * 2]    # [44, 0, 64, 12]
    assert np.allclose(d0.box_src, [A, Cb, D], atol=1e-4) and np.allclose(d1.box_src, [E, F], atol=1e-4)
    # the ROI table of the edge: class-0 boxes only, frame by frame in keep-list order, with their rank in the keep list
    r = res.children[0].rois
    assert r.frame.tolist() == [0, 0, 1] and r.rank.tolist() == [0, 2, 1] and r.cls.tolist() == [0, 0, 0]
    assert np.allclose(r.box, [A, D, F], atol=1e-4)
    # the child saw exactly those crops: a crop of an integer-aligned 8 x 8 source window is the window itself
    crops = res.children[0].crops
    assert crops.shape == (3, 8, 8, 3)
    assert np.allclose(crops[1], frames[0, 38:46, 38:46].astype(np.float64) / 255.0, atol=1e-6)
    assert res.children[0].logits.shape == (3, 3) and res.children[0].labels.tolist() == res.children[0].logits.argmax(1).tolist()
    # all classes routed: five ROIs in (frame, rank) order; no class routed: none, and the child is not run
    assert cascade.run_cascade(_spec(0b11), frames, planted_heads=[head]).children[0].rois.rank.tolist() == [0, 1, 2, 0, 1]
    none = cascade.run_cascade(_spec(0), frames, planted_heads=[head]).children[0]
    assert len(none.rois) == 0 and none.labels.shape == (0,) and none.logits is None
    # max_child_rois cuts what the child evaluates, not the table
    cut = cascade.run_cascade(_spec(0b11), frames, planted_heads=[head], max_child_rois=2).children[0]
    assert len(cut.rois) == 5 and cut.crops.shape[0] == 2 and cut.logits.shape == (2, 3)
