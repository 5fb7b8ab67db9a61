"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times.

The traffic workload is small enough for the oracle to run whole.  The high-resolution workload (32 frames of
3840x2160) is not: there the integer work is compared in full (every frame's candidates, top-k, NMS, ROI table),
and the floating-point tensors on samples the oracle evaluates one by one - letterbox rows, single convolution
layers at sampled output positions computed from the layer's own input as it sits on the GPU, and the classifier
on a few ROIs from both ends of the ROI table.
"""
import numpy as np
import pytest

import bench
from oracle import cascade, nn, postprocess as pp, preprocess as pre
from helpers import TOL, rel_err

pytestmark = pytest.mark.gpu


def _dev(frames):
    import torch
    return [torch.from_numpy(f).cuda() for f in frames]


def test_traffic_workload_exactly_as_benchmarked(octo):
    spec, scene, heads, _ = bench.make_workload("traffic")
    det, cls, plate = spec.models
    n = scene.frames.shape[0]
    ref = cascade.run_cascade(spec, scene.frames, planted_heads=heads)
    P = octo.Pipeline(spec)
    d_heads = [octo.to_device(h, det.dtype) for h in heads]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    for rep in range(2):                                   # the second batch runs with tile shapes picked from the first one's ROI count
        P.submit(_dev(scene.frames))
        assert P.run() == n
        frames, boxes, st = P.collect()
        assert st == octo.OK
        for l, t in enumerate(det.outputs):
            assert rel_err(P.get_tensor(0, t, n), ref.heads[l]) <= TOL[det.dtype], (rep, l)
        for f, d in enumerate(ref.dets):
            cc, top, keep = P.get_detections(0, f)
            assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist()
        assert frames["n_boxes"].tolist() == [len(d.keep) for d in ref.dets]
        n_roi = len(ref.children[0].rois)
        assert n_roi == int(frames["n_boxes"].sum())
        for e in (0, 1):
            rois, r = P.get_rois(e), ref.children[e].rois
            assert rois["frame"].tolist() == r.frame.tolist() and rois["rank"].tolist() == r.rank.tolist()
        logits = P.get_tensor(1, cls.outputs[0], n_roi).reshape(n_roi, -1)
        assert rel_err(logits, ref.children[0].logits) <= TOL[det.dtype]
        for l, t in enumerate(plate.outputs):
            assert rel_err(P.get_tensor(2, t, n_roi), ref.children[1].heads[l]) <= TOL[det.dtype]
        srt = np.sort(ref.children[0].logits, axis=1)
        clear = (srt[:, -1] - srt[:, -2]) > 4 * TOL[det.dtype] * max(1.0, np.abs(ref.children[0].logits).max())
        lab = P.get_labels(0)
        assert np.array_equal(lab[clear], ref.children[0].labels[clear]) and np.array_equal(boxes["child_label"][:, 0], lab)
        assert np.all(frames["slo_met"] == 1)
    P.close()


def _sample_positions(rng, n, ho, wo, count):
    pos = [(0, 0, 0), (0, ho - 1, wo - 1), (n - 1, 0, wo - 1), (n - 1, ho - 1, 0), (n - 1, ho - 1, wo - 1)]
    for _ in range(count - len(pos)):
        pos.append((int(rng.integers(0, n)), int(rng.integers(0, ho)), int(rng.integers(0, wo))))
    return pos


def _ends(P, model, tid, n, k=2):
    """The first and the last k items of a tensor that was computed for n items: [2k][h][w][c]."""
    return np.concatenate([P.get_tensor(model, tid, k, 0), P.get_tensor(model, tid, k, n - k)])


def test_hires_workload_full_batch_on_samples(octo):
    spec, scene, heads, _ = bench.make_workload("hires")
    det, cls = spec.models
    n = scene.frames.shape[0]
    assert n == 32 and det.in_h == 1280
    P = octo.Pipeline(spec, keep_all_tensors=True)
    d_heads = [octo.to_device(h, det.dtype) for h in heads]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    P.submit(_dev(scene.frames))
    assert P.run() == n
    frames, boxes, st = P.collect(frame_cap=n, box_cap=n * det.max_det)
    assert st == octo.OK and len(frames) == n
    # -- integer work, every frame --
    dets = cascade.postprocess_heads(heads, det)
    assert max(d.cand_count for d in dets) > det.topk            # top-k really truncates somewhere
    for f, d in enumerate(dets):
        cc, top, keep = P.get_detections(0, f)
        assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist(), f
    assert frames["n_boxes"].tolist() == [len(d.keep) for d in dets]
    rois = P.get_rois(0)
    exp = [(f, r) for f, d in enumerate(dets) for r in range(len(d.keep))]
    assert list(zip(rois["frame"].tolist(), rois["rank"].tolist())) == exp
    _, nw, nh, left, top_ = pre.letterbox_geometry(spec.src_h, spec.src_w, det.in_h, det.in_w)
    src = np.concatenate([pp.to_source_box(d.top.box[d.keep], spec.src_h, spec.src_w, nw, nh, left, top_) for d in dets])
    assert np.abs(np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], 1) - src).max() < 2e-2
    # -- letterbox: the last frame in full --
    lb = P.get_tensor(0, 0, 1, n - 1)
    ref_lb = pre.letterbox(scene.frames[n - 1:], det.in_h, det.in_w, det.dtype, det.norm_scale, det.norm_bias, det.pad_value)
    assert np.abs(lb - ref_lb).max() <= 8e-3
    # -- convolution layers at full batch, sampled outputs from the layer's own GPU input --
    rng = np.random.default_rng(77)
    shapes = det.tensor_shapes()
    conv_ids = [i for i, L in enumerate(det.layers) if L.op == "conv"]
    by_size = sorted(conv_ids, key=lambda i: -shapes[det.layers[i].inputs[0]][0])
    picks = sorted(set(conv_ids[1::7] + [i for i in det_heads_layers(det)]))
    assert len(picks) >= 10
    for i in picks:
        L = det.layers[i]
        x = _ends(P, 0, L.inputs[0], n)
        y = _ends(P, 0, i + 1, n)
        res = _ends(P, 0, L.inputs[1], n) if len(L.inputs) > 1 else None
        pos = _sample_positions(rng, 4, y.shape[1], y.shape[2], 24)
        want = nn.conv_layer_at(x, L, det.dtype, pos, res)
        got = np.stack([y[a, b, c] for (a, b, c) in pos])
        assert rel_err(got, want) <= TOL[det.dtype], (i, L.kh, L.stride)
        del x, y, res
    # the first layer (largest tensors): the last frame only
    L0 = det.layers[by_size[0]]
    x = P.get_tensor(0, L0.inputs[0], 1, n - 1)
    y = P.get_tensor(0, by_size[0] + 1, 1, n - 1)
    pos = _sample_positions(rng, 1, y.shape[1], y.shape[2], 24)
    assert rel_err(np.stack([y[a, b, c] for (a, b, c) in pos]), nn.conv_layer_at(x, L0, det.dtype, pos)) <= TOL[det.dtype]
    # -- classifier on ROIs from both ends of the table --
    n_roi = len(rois)
    assert n_roi > 1000
    pick = [0, 1, 2, n_roi // 2, n_roi - 3, n_roi - 2, n_roi - 1]
    box = np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], 1)[pick].astype(np.float64)
    crops = pre.crop_resize(scene.frames, rois["frame"][pick], box, cls.in_h, cls.in_w, cls.dtype, cls.norm_scale, cls.norm_bias)
    ref_logits = nn.run_model(cls, crops)[cls.outputs[0]].reshape(len(pick), -1)
    logits = P.get_tensor(1, cls.outputs[0], n_roi).reshape(n_roi, -1)[pick]
    assert rel_err(logits, ref_logits) <= TOL[cls.dtype]
    P.close()


def det_heads_layers(det):
    return [t - 1 for t in det.outputs]


@pytest.mark.parametrize("bz", [8, 64])
def test_sweep_workload_at_full_batch_on_samples(octo, bz):
    """The batch-size sweep's configuration (bf16, negative-binomial object counts) exactly as bench.py builds it, at
    its largest batch and at 8: all integer work on every frame, convolution layers on sampled outputs from both ends
    of the batch, classifier logits on ROIs from both ends of the table."""
    from paper_2502_01277_amd import synth, zoo
    spec = zoo.sweep_cascade(bz)
    det, cls = spec.models
    rng = np.random.default_rng(zoo.SEED0 + 3)
    counts = synth.counts_negbin(rng, bz)
    scene = synth.make_scene(rng, bz, 1080, 1920, counts, 24, 200, log_uniform=True)
    heads = synth.planted_heads(rng, det, scene, 1080, 1920, pre.letterbox_geometry(1080, 1920, det.in_h, det.in_w)[1:])
    P = octo.Pipeline(spec, keep_all_tensors=True)
    d_heads = [octo.to_device(h, det.dtype) for h in heads]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    P.submit(_dev(scene.frames))
    assert P.run() == bz
    frames, boxes, st = P.collect(frame_cap=bz, box_cap=bz * det.max_det)
    assert st == octo.OK and len(frames) == bz
    dets = cascade.postprocess_heads(heads, det)
    for f, d in enumerate(dets):
        cc, top, keep = P.get_detections(0, f)
        assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist(), f
    assert frames["n_boxes"].tolist() == [len(d.keep) for d in dets]
    rois = P.get_rois(0)
    assert list(zip(rois["frame"].tolist(), rois["rank"].tolist())) == [(f, r) for f, d in enumerate(dets) for r in range(len(d.keep))]
    k = min(2, bz // 2)
    rng2 = np.random.default_rng(79)
    conv_ids = [i for i, L in enumerate(det.layers) if L.op == "conv"]
    for i in sorted(set(conv_ids[::9] + det_heads_layers(det))):
        L = det.layers[i]
        x = _ends(P, 0, L.inputs[0], bz, k)
        y = _ends(P, 0, i + 1, bz, k)
        res = _ends(P, 0, L.inputs[1], bz, k) if len(L.inputs) > 1 else None
        pos = _sample_positions(rng2, 2 * k, y.shape[1], y.shape[2], 16)
        assert rel_err(np.stack([y[a, b, c] for (a, b, c) in pos]), nn.conv_layer_at(x, L, det.dtype, pos, res)) <= TOL[det.dtype], (i, L.kh, L.stride)
    n_roi = len(rois)
    assert n_roi >= 8
    pick = [0, 1, n_roi // 2, n_roi - 2, n_roi - 1]
    box = np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], 1)[pick].astype(np.float64)
    crops = pre.crop_resize(scene.frames, rois["frame"][pick], box, cls.in_h, cls.in_w, cls.dtype, cls.norm_scale, cls.norm_bias)
    ref_logits = nn.run_model(cls, crops)[cls.outputs[0]].reshape(len(pick), -1)
    logits = P.get_tensor(1, cls.outputs[0], n_roi).reshape(n_roi, -1)[pick]
    assert rel_err(logits, ref_logits) <= TOL[cls.dtype]
    P.close()
