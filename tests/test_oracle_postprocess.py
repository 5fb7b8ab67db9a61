"""Pins for the oracle's decode / top-k / NMS / ROI compaction."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import postprocess as pp, preprocess as pre
from oracle.cascade import postprocess_heads
from paper_2502_01277_amd import synth, zoo

f32 = np.float32


def _det(dtype="f32", thr=0.25):
    d = zoo.plain_detector("d", dtype, 64, (8, 8, 8), 4, seed=1, score_thr=thr)   # stride 8, grid 8, A=3, C=4
    return d


def test_zero_logits_decode_to_cell_centre_anchor_size_and_quarter_score():
    d = _det(thr=0.25)
    h = np.zeros((8, 8, 3 * 9), f32)
    assert len(pp.decode_frame([h], d)) == 0                 # score is exactly 0.25: strict '>' drops it
    d.score_thr = 0.2499
    c = pp.decode_frame([h], d)
    assert len(c) == 8 * 8 * 3 and np.all(c.score == f32(0.25)) and np.all(c.cls == 0)
    assert np.array_equal(c.idx, np.arange(192))
    for i in (0, 5, 100, 191):
        a = i % 3; gx = (i // 3) % 8; gy = i // 24
        aw, ah = d.anchors[0, a]
        cx, cy = (gx + 0.5) * 8, (gy + 0.5) * 8
        assert np.allclose(c.box[i], [cx - aw / 2, cy - ah / 2, cx + aw / 2, cy + ah / 2], atol=1e-5)


def test_candidate_index_levels_and_class_argmax_ties():
    d = zoo.csp_detector("d", "f32", 64, (8, 8, 8, 8, 8), (1, 1, 1, 1), 4, seed=2)    # grids 8, 4, 2
    heads = [np.full((g, g, 3 * 9), -9.0, f32) for g in d.grids]
    heads[1][2, 3, 1 * 9 + 4] = 5.0                  # level 1, gy=2, gx=3, anchor 1: objectness
    heads[1][2, 3, 1 * 9 + 5 + 1] = 7.0              # classes 1 and 3 tie -> lowest index
    heads[1][2, 3, 1 * 9 + 5 + 3] = 7.0
    c = pp.decode_frame(heads, d)
    assert len(c) == 1 and c.cls[0] == 1
    assert c.idx[0] == 8 * 8 * 3 + (2 * 4 + 3) * 3 + 1
    s = 1 / (1 + np.exp(-5.0)) * 1 / (1 + np.exp(-7.0))
    assert abs(float(c.score[0]) - s) < 1e-6


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_planted_boxes_round_trip_through_decode(dtype):
    rng = np.random.default_rng(11)
    det = zoo.csp_detector("d", dtype, 640, zoo.S_WIDTHS, zoo.S_DEPTHS, 80, seed=3)
    counts = np.array([5, 0, 9])
    scene = synth.make_scene(rng, 3, 270, 480, counts, 12, 120, log_uniform=True)
    heads = synth.planted_heads(rng, det, scene, 270, 480, pre.letterbox_geometry(270, 480, det.in_h, det.in_w)[1:], max_dups=0)
    _, nw, nh, left, top = pre.letterbox_geometry(270, 480, 640, 640)
    tol = {"f32": 0.01, "f16": 0.5, "bf16": 4.0}[dtype]
    for f in range(3):
        c = pp.decode_frame([h[f] for h in heads], det)
        assert len(c) == counts[f]
        src = pp.to_source_box(c.box, 270, 480, nw, nh, left, top)
        for r, cl in zip(scene.rects[f], scene.classes[f]):
            d = np.abs(src - r.astype(f32)).max(axis=1)
            j = int(np.argmin(d))
            assert d[j] * (nw / 480) < tol and c.cls[j] == cl % 80
        assert np.all(np.diff(c.idx) > 0)


def _random_cands(rng, n, n_cls=3, span=100.0, quant=None):
    xy = rng.uniform(0, span, (n, 2)); wh = rng.uniform(5, 40, (n, 2))
    box = np.concatenate([xy, xy + wh], axis=1).astype(f32)
    score = rng.uniform(0.3, 1.0, n).astype(f32)
    if quant:
        score = (np.round(score * quant) / quant).astype(f32)          # force ties
    return pp.Candidates(box, score, rng.integers(0, n_cls, n).astype(np.int32),
                         rng.permutation(n * 3)[:n].astype(np.int32))


def test_topk_order_and_invariants():
    rng = np.random.default_rng(5)
    c = _random_cands(rng, 500, quant=20)
    t = pp.topk(c, 100)
    ref = np.lexsort((c.idx, -c.score.astype(np.float64)))[:100]
    assert np.array_equal(t.idx, c.idx[ref])
    assert len(t) == 100 and np.all(np.diff(t.score) <= 0)
    ties = np.diff(t.score) == 0
    assert ties.any() and np.all(np.diff(t.idx)[ties] > 0)
    rest = np.setdiff1d(c.idx, t.idx)
    worst = (float(t.score[-1]), -int(t.idx[-1]))
    sc = {int(i): float(s) for i, s in zip(c.idx, c.score)}
    assert all((sc[int(i)], -int(i)) < worst for i in rest)
    assert len(pp.topk(c.take(range(7)), 100)) == 7 and len(pp.topk(c.take([]), 5)) == 0


def _iou_exact(a, b):
    iw = max(Fraction(0), min(a[2], b[2]) - max(a[0], b[0])); ih = max(Fraction(0), min(a[3], b[3]) - max(a[1], b[1]))
    inter = iw * ih
    return inter, (a[2] - a[0]) * (a[3] - a[1]) + (b[2] - b[0]) * (b[3] - b[1]) - inter


def test_suppression_predicate_against_exact_rational_iou():
    rng = np.random.default_rng(6)
    thr = 0.45
    for _ in range(400):
        a = rng.integers(0, 40, 4); b = rng.integers(0, 40, 4)
        a[2:] += a[:2] + 1; b[2:] += b[:2] + 1
        inter, uni = _iou_exact([Fraction(int(v)) for v in a], [Fraction(int(v)) for v in b])
        exact = inter > Fraction(thr) * uni
        got = bool(pp.suppresses(a.astype(f32), 1, b.astype(f32), 1, thr))
        if abs(float(inter) - thr * float(uni)) > 1e-3:       # away from the fp32 rounding boundary
            assert got == exact
        assert not pp.suppresses(a.astype(f32), 1, b.astype(f32), 2, thr)
        assert bool(pp.suppresses(b.astype(f32), 1, a.astype(f32), 1, thr)) == got      # symmetric


def _greedy_by_enumeration(c, thr):
    """The unique subset S with: i in S <=> no j in S, j < i, suppresses i - found by trying all subsets."""
    n = len(c)
    sols = []
    for bits in itertools.product([0, 1], repeat=n):
        ok = True
        for i in range(n):
            sup = any(bits[j] and bool(pp.suppresses(c.box[j], c.cls[j], c.box[i], c.cls[i], thr)) for j in range(i))
            if bool(bits[i]) == sup:
                ok = False
                break
        if ok:
            sols.append([i for i in range(n) if bits[i]])
    assert len(sols) == 1
    return sols[0]


def test_nms_equals_enumeration_on_tiny_sets():
    rng = np.random.default_rng(7)
    for trial in range(12):
        c = pp.topk(_random_cands(rng, 8, n_cls=2, span=30.0), 8)
        assert pp.nms(c, 0.3, 100).tolist() == _greedy_by_enumeration(c, 0.3)


def test_nms_invariants_maximality_special_cases():
    rng = np.random.default_rng(8)
    c = pp.topk(_random_cands(rng, 300, n_cls=3, span=120.0), 300)
    keep = pp.nms(c, 0.45, 1000)
    ks = set(keep.tolist())
    assert np.all(np.diff(keep) > 0) and np.all(np.diff(c.score[keep]) <= 0)
    for a, b in itertools.combinations(keep.tolist(), 2):
        assert not pp.suppresses(c.box[a], c.cls[a], c.box[b], c.cls[b], 0.45)
    for i in range(len(c)):
        if i not in ks:
            assert any(j < i and pp.suppresses(c.box[j], c.cls[j], c.box[i], c.cls[i], 0.45) for j in ks)
    assert 20 < len(keep) < 300
    assert pp.nms(c, 0.45, 7).tolist() == keep[:7].tolist()
    # disjoint boxes: all kept; identical boxes same class: one kept; identical boxes distinct classes: all kept
    box = np.array([[i * 10, 0, i * 10 + 9, 9] for i in range(6)], f32)
    sc = np.linspace(0.9, 0.4, 6).astype(f32)
    z = np.zeros(6, np.int32)
    assert pp.nms(pp.Candidates(box, sc, z, np.arange(6, dtype=np.int32)), 0.45, 100).tolist() == list(range(6))
    same = np.tile(box[:1], (6, 1))
    assert pp.nms(pp.Candidates(same, sc, z, np.arange(6, dtype=np.int32)), 0.45, 100).tolist() == [0]
    assert pp.nms(pp.Candidates(same, sc, np.arange(6, dtype=np.int32), np.arange(6, dtype=np.int32)), 0.45, 100).tolist() == list(range(6))
    # chain a-b-c: b suppressed by a, so c (overlapping only b) survives
    chain = np.array([[0, 0, 10, 10], [4, 0, 14, 10], [8, 0, 18, 10]], f32)
    assert pp.nms(pp.Candidates(chain, sc[:3], z[:3], np.arange(3, dtype=np.int32)), 0.4, 100).tolist() == [0, 2]


def test_compaction_order_counts_masks_and_unletterbox_identity():
    rng = np.random.default_rng(9)
    kept = []
    for f in range(5):
        k = int(rng.integers(0, 7))
        kept.append((rng.integers(0, 4, k).astype(np.int32), rng.uniform(0, 50, (k, 4)).astype(f32)))
    allr = pp.compact_rois(kept, (1 << 128) - 1)
    assert len(allr) == sum(len(c) for c, _ in kept)
    pairs = list(zip(allr.frame.tolist(), allr.rank.tolist()))
    assert pairs == sorted(pairs) and len(set(pairs)) == len(pairs)
    only = pp.compact_rois(kept, 0b0101)
    assert len(only) == sum(int(np.isin(c, [0, 2]).sum()) for c, _ in kept)
    assert set(only.cls.tolist()) <= {0, 2}
    for j in range(len(only)):
        assert np.array_equal(only.box[j], kept[only.frame[j]][1][only.rank[j]])
    assert len(pp.compact_rois(kept, 0)) == 0
    # un-letterbox(letterbox(box)) = box
    _, nw, nh, left, top = pre.letterbox_geometry(1080, 1920, 640, 640)
    src = rng.uniform(0, 1, (50, 4)) * [1920, 1080, 1920, 1080]
    lb = src * np.array([nw / 1920, nh / 1080] * 2) + np.array([left, top] * 2)
    back = pp.to_source_box(lb.astype(f32), 1080, 1920, nw, nh, left, top)
    assert np.abs(back - src).max() < 1e-3 * 3
    out = pp.to_source_box(np.array([[-50, -50, 700, 700]], f32), 1080, 1920, nw, nh, left, top)
    assert out.tolist() == [[0, 0, 1920, 1080]]


def test_postprocess_pipeline_on_planted_heads_with_duplicates():
    rng = np.random.default_rng(12)
    det = zoo.csp_detector("d", "f16", 640, zoo.S_WIDTHS, zoo.S_DEPTHS, 80, seed=3, topk=1000, max_det=64)
    counts = synth.counts_poisson(rng, 4)
    scene = synth.make_scene(rng, 4, 1080, 1920, counts, 24, 360, log_uniform=True)
    heads = synth.planted_heads(rng, det, scene, 1080, 1920, pre.letterbox_geometry(1080, 1920, det.in_h, det.in_w)[1:], max_dups=4)
    dets = postprocess_heads(heads, det)
    for f, d in enumerate(dets):
        assert d.cand_count >= counts[f]
        assert len(d.keep) <= counts[f] + 2 and len(d.keep) >= min(counts[f], 1)   # duplicates mostly suppressed
        assert len(d.keep) < d.cand_count or d.cand_count == counts[f]
