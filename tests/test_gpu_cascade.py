"""GPU parity of the whole cascade (octo_submit_frames / octo_run / octo_collect) against the oracle."""
import numpy as np
import pytest

from oracle import cascade, postprocess as pp, preprocess as pre
from paper_2502_01277_amd import synth, zoo
from helpers import TOL, cands_to_records, records_to_cands, rel_err

pytestmark = pytest.mark.gpu


def _frames_dev(frames):
    import torch
    return [torch.from_numpy(f).cuda() for f in frames]


def _check_postprocessing_from_gpu_candidates(P, spec, model, n_items, heads_gpu):
    """Given the GPU's own head tensors, its decode must agree with the oracle's (up to threshold rounding), and
    top-k / NMS must be bit-exact given the GPU's decoded list."""
    det = spec.models[model]
    for f in range(n_items):
        cc, top, keep = P.get_detections(model, f)
        ref = pp.decode_frame([h[f] for h in heads_gpu], det)
        assert abs(cc - len(ref)) <= 2
        # re-run the oracle's top-k + NMS on the GPU's sorted list: identical keep-list
        c = records_to_cands(top)
        assert np.all(np.diff(c.score) <= 0)
        assert keep.tolist() == pp.nms(c, det.iou_thr, det.max_det).tolist()
        if cc == len(ref):
            rt = pp.topk(ref, det.topk)
            if len(c) and np.array_equal(rt.idx, c.idx):
                assert np.abs(rt.box - c.box).max() < 1e-3 and np.abs(rt.score - c.score).max() < 1e-5


def test_tiny_cascade_fp32_natural(octo):
    spec = zoo.tiny_cascade()
    rng = np.random.default_rng(zoo.SEED0 + 1)
    scene = synth.make_scene(rng, 2, 320, 320, [6, 6], 16, 96, n_classes=8)
    ref = cascade.run_cascade(spec, scene.frames)
    P = octo.Pipeline(spec, keep_all_tensors=True)
    P.submit(_frames_dev(scene.frames), frame_ids=[10, 11])
    assert P.run() == 2
    frames, boxes, st = P.collect()
    assert st == octo.OK and frames["frame_id"].tolist() == [10, 11]
    det = spec.models[0]
    assert rel_err(P.get_tensor(0, 0, 2), ref.lb) <= 2e-6
    head = P.get_tensor(0, det.outputs[0], 2)
    assert rel_err(head, ref.heads[0]) <= TOL["f32"]
    _check_postprocessing_from_gpu_candidates(P, spec, 0, 2, [head])
    # the oracle run on the very same head gives the same keep-lists, ROI table and labels
    same = all(P.get_detections(0, f)[1]["idx"].tolist() == ref.dets[f].top.idx.tolist() for f in range(2))
    assert same, "top-k lists differ between GPU and oracle heads (threshold-rounding case); re-seed the test"
    rois = P.get_rois(0)
    assert rois["frame"].tolist() == ref.children[0].rois.frame.tolist()
    assert rois["rank"].tolist() == ref.children[0].rois.rank.tolist()
    gb = np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], axis=1)
    assert np.abs(gb - ref.children[0].rois.box).max() < 1e-3
    n_roi = len(rois)
    cls = spec.models[1]
    assert rel_err(P.get_tensor(1, 0, n_roi), ref.children[0].crops) <= 2e-4
    logits = P.get_tensor(1, cls.outputs[0], n_roi).reshape(n_roi, -1)
    assert rel_err(logits, ref.children[0].logits) <= TOL["f32"]
    lab = P.get_labels(0)
    margin = np.sort(ref.children[0].logits, axis=1)
    clear = (margin[:, -1] - margin[:, -2]) > 1e-3
    assert np.array_equal(lab[clear], ref.children[0].labels[clear]) and clear.mean() > 0.5
    # what octo_collect returned is the same thing
    assert frames["n_boxes"].tolist() == [len(d.keep) for d in ref.dets]
    off = 0
    for f, d in enumerate(ref.dets):
        b = boxes[off:off + len(d.keep)]
        assert np.abs(np.stack([b["x1"], b["y1"], b["x2"], b["y2"]], 1) - d.box_src).max() < 1e-3
        assert b["cls"].tolist() == d.top.cls[d.keep].tolist()
        mine = rois["frame"] == f
        assert b["child_label"][:, 0].tolist() == lab[mine].tolist() and np.all(b["child_label"][:, 1] == -1)
        off += len(d.keep)
    assert np.all(frames["latency_ms"] > 0) and np.all(frames["slo_met"] == 1)
    P.close()


@pytest.mark.parametrize("dtype,n_frames", [("f16", 3), ("bf16", 2)])
def test_traffic_cascade_planted(octo, dtype, n_frames):
    spec = zoo.traffic_cascade(dtype, det_batch=n_frames, max_rois_per_frame=24)
    det = spec.models[0]
    rng = np.random.default_rng(zoo.SEED0 + 2)
    counts = np.minimum(synth.counts_poisson(rng, n_frames, 8, 64), 12)
    scene = synth.make_scene(rng, n_frames, 1080, 1920, counts, 24, 360, log_uniform=True)
    planted = synth.planted_heads(rng, det, scene, 1080, 1920, pre.letterbox_geometry(1080, 1920, det.in_h, det.in_w)[1:])
    ref = cascade.run_cascade(spec, scene.frames, planted_heads=planted)
    P = octo.Pipeline(spec, keep_all_tensors=False)
    d_heads = [octo.to_device(h, dtype) for h in planted]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    P.submit(_frames_dev(scene.frames))
    assert P.run() == n_frames
    frames, boxes, st = P.collect()
    assert st == octo.OK
    # detector convolutions on the real frames
    for l, t in enumerate(det.outputs):
        assert rel_err(P.get_tensor(0, t, n_frames), ref.heads[l]) <= TOL[dtype], l
    # post-processing on the planted heads is exact
    for f, d in enumerate(ref.dets):
        cc, top, keep = P.get_detections(0, f)
        assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist()
    assert frames["n_boxes"].tolist() == [len(d.keep) for d in ref.dets]
    for e in (0, 1):
        rois = P.get_rois(e)
        r = ref.children[e].rois
        assert rois["frame"].tolist() == r.frame.tolist() and rois["rank"].tolist() == r.rank.tolist()
        assert np.abs(np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], 1) - r.box).max() < 1e-2
    n_roi = len(ref.children[0].rois)
    cls, plate = spec.models[1], spec.models[2]
    logits = P.get_tensor(1, cls.outputs[0], n_roi).reshape(n_roi, -1)
    assert rel_err(logits, ref.children[0].logits) <= TOL[dtype]
    for l, t in enumerate(plate.outputs):
        assert rel_err(P.get_tensor(2, t, n_roi), ref.children[1].heads[l]) <= TOL[dtype]
    gh = [P.get_tensor(2, t, n_roi) for t in plate.outputs]
    _check_postprocessing_from_gpu_candidates(P, spec, 2, n_roi, gh)
    lab0, lab1 = P.get_labels(0), P.get_labels(1)
    srt = np.sort(ref.children[0].logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 4 * TOL[dtype] * max(1.0, np.abs(ref.children[0].logits).max())
    assert np.array_equal(lab0[clear], ref.children[0].labels[clear])
    assert np.array_equal(lab1, np.array([len(P.get_detections(2, j)[2]) for j in range(n_roi)]))
    assert np.array_equal(boxes["child_label"][:, 0], lab0) and np.array_equal(boxes["child_label"][:, 1], lab1)
    P.close()


def test_queueing_batching_and_empty_frames(octo):
    spec = zoo.tiny_cascade()
    spec.models[0].batch_size = 2
    spec.max_frames = 2
    rng = np.random.default_rng(3)
    scene = synth.make_scene(rng, 5, 320, 320, [3] * 5, 16, 96, n_classes=8)
    P = octo.Pipeline(spec)
    dev = _frames_dev(scene.frames)
    # a head that decodes to nothing: zero detections everywhere
    import torch
    none = torch.full((2, 20, 20, 39), -20.0, device="cuda")
    P.set_head(0, 0, none)
    P.submit(dev, frame_ids=list(range(5)))
    launched = [P.run(), P.run(), P.run(), P.run()]
    assert launched == [2, 2, 1, 0]
    got_f, got_b = [], []
    while sum(len(f) for f in got_f) < 5:                    # a blocking collect returns at least the oldest batch
        f, b, st = P.collect()
        assert st == octo.OK and 1 <= len(f) <= 5
        got_f.append(f); got_b.append(b)
    frames, boxes = np.concatenate(got_f), np.concatenate(got_b)
    assert frames["frame_id"].tolist() == [0, 1, 2, 3, 4]
    assert frames["n_boxes"].sum() == 0 and len(boxes) == 0 and len(P.get_rois(0)) == 0
    _, _, st = P.collect(blocking=False)
    assert st == octo.ENOTREADY
    # queue overflow is refused without side effects
    with pytest.raises(octo.OctoError) as ei:
        P.submit(dev + dev)
    assert ei.value.status == octo.ECAP
    P.set_head(0, 0, None)
    P.submit(dev[:2], frame_ids=[7, 8])
    assert P.run() == 2
    frames, boxes, st = P.collect()
    assert frames["frame_id"].tolist() == [7, 8] and frames["n_boxes"].sum() > 0
    P.close()


def test_run_model_by_model_on_two_streams_matches_octo_run(octo):
    import torch
    spec = zoo.tiny_cascade()
    rng = np.random.default_rng(4)
    scene = synth.make_scene(rng, 2, 320, 320, [6, 6], 16, 96, n_classes=8)
    dev = _frames_dev(scene.frames)
    P = octo.Pipeline(spec)
    P.submit(dev)
    P.run()
    f0, b0, _ = P.collect()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    P.submit(dev)
    assert P.run_model(0, s1) == 2 and P.run_model(1, s2) == 2
    f1, b1, _ = P.collect()
    assert b0.tobytes() == b1.tobytes() and f0["n_boxes"].tolist() == f1["n_boxes"].tolist()
    P.close()


def test_hires_cascade_planted_heavy_tail(octo):
    """High-resolution workload at its real per-frame shape (one 3840x2160 frame, m-shaped detector at 1280, top-k 1000
    truncating, dense clutter for NMS), bf16; the classifier is checked on the first ROIs only (oracle time)."""
    spec = zoo.hires_cascade(det_batch=1, max_rois_per_frame=300)
    det = spec.models[0]
    rng = np.random.default_rng(zoo.SEED0 + 5)
    counts = np.array([37])
    scene = synth.make_scene(rng, 1, 2160, 3840, counts, 48, 720, log_uniform=True)
    planted = synth.planted_heads(rng, det, scene, 2160, 3840, pre.letterbox_geometry(2160, 3840, det.in_h, det.in_w)[1:], n_clutter=1100)
    ref = cascade.run_cascade(spec, scene.frames, planted_heads=planted, max_child_rois=6)
    assert ref.dets[0].cand_count > 1000 and len(ref.dets[0].top) == 1000 and 40 < len(ref.dets[0].keep) <= 300
    P = octo.Pipeline(spec, keep_all_tensors=True)          # the crops (child tensor 0) are read back below
    d_heads = [octo.to_device(h, "bf16") for h in planted]        # must stay alive while the pipeline reads them
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    P.submit(_frames_dev(scene.frames))
    assert P.run() == 1
    frames, boxes, st = P.collect()
    assert st == octo.OK
    for l, t in enumerate(det.outputs):
        assert rel_err(P.get_tensor(0, t, 1), ref.heads[l]) <= TOL["bf16"], l
    cc, top, keep = P.get_detections(0, 0)
    d = ref.dets[0]
    assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist()
    rois = P.get_rois(0)
    r = ref.children[0].rois
    assert rois["frame"].tolist() == r.frame.tolist() and rois["rank"].tolist() == r.rank.tolist()
    assert np.abs(np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], 1) - r.box).max() < 2e-2
    m = 6
    assert rel_err(P.get_tensor(1, 0, m), ref.children[0].crops) <= 8e-3
    logits = P.get_tensor(1, spec.models[1].outputs[0], m).reshape(m, -1)
    assert rel_err(logits, ref.children[0].logits) <= TOL["bf16"]
    assert frames["n_boxes"][0] == len(d.keep) and len(boxes) == len(d.keep)
    P.close()


def test_surveillance_cascade_planted_bottleneck_child(octo):
    """The people-surveillance pipeline of the co-location workload at its real shapes (bf16): three planted 1080p
    frames, s-shaped detector at 640, every ROI stretched to 256 x 128 and classified by the ResNet-50-shaped attribute
    model with 32 outputs.  Detector heads, all integer work and the ROI table against the oracle on every frame; the
    child on the first ROIs (oracle time): crops, every tensor of the network, logits, labels with a clear margin."""
    from oracle import nn
    dtype, n_frames, m = "bf16", 3, 8
    spec = zoo.surveillance_cascade(dtype, det_batch=n_frames, max_rois_per_frame=24)
    det, attr = spec.models
    assert (attr.in_h, attr.in_w) == (256, 128) and attr.layers[-1].cout == 32
    rng = np.random.default_rng(zoo.SEED0 + 4)
    counts = np.minimum(synth.counts_poisson(rng, n_frames, 8, 64), 12)
    scene = synth.make_scene(rng, n_frames, 1080, 1920, counts, 24, 360, log_uniform=True)
    planted = synth.planted_heads(rng, det, scene, 1080, 1920, pre.letterbox_geometry(1080, 1920, det.in_h, det.in_w)[1:])
    ref = cascade.run_cascade(spec, scene.frames, planted_heads=planted, max_child_rois=m)
    P = octo.Pipeline(spec, keep_all_tensors=True)
    d_heads = [octo.to_device(h, dtype) for h in planted]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    P.submit(_frames_dev(scene.frames))
    assert P.run() == n_frames
    frames, boxes, st = P.collect()
    assert st == octo.OK
    for l, t in enumerate(det.outputs):
        assert rel_err(P.get_tensor(0, t, n_frames), ref.heads[l]) <= TOL[dtype], l
    for f, d in enumerate(ref.dets):
        cc, top, keep = P.get_detections(0, f)
        assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist()
    assert frames["n_boxes"].tolist() == [len(d.keep) for d in ref.dets]
    rois, r = P.get_rois(0), ref.children[0].rois
    n_roi = len(r)
    assert n_roi >= m and rois["frame"].tolist() == r.frame.tolist() and rois["rank"].tolist() == r.rank.tolist()
    assert rois["cls"].tolist() == r.cls.tolist()
    assert np.abs(np.stack([rois["x1"], rois["y1"], rois["x2"], rois["y2"]], 1) - r.box).max() < 1e-2
    off = 0
    for f, d in enumerate(ref.dets):
        b = boxes[off:off + len(d.keep)]
        assert np.abs(np.stack([b["x1"], b["y1"], b["x2"], b["y2"]], 1) - d.box_src).max() < 1e-2
        assert b["cls"].tolist() == d.top.cls[d.keep].tolist()
        off += len(d.keep)
    # the child on the first m ROIs: every tensor
    assert rel_err(P.get_tensor(1, 0, m), ref.children[0].crops) <= 8e-3
    ts = nn.run_model(attr, ref.children[0].crops, keep_all=True)
    shapes = attr.tensor_shapes()
    assert max(s[2] for s in shapes) == 2048
    for t in range(1, len(attr.layers) + 1):
        got = P.get_tensor(1, t, m)
        assert rel_err(got.reshape(ts[t].shape), ts[t]) <= TOL[dtype], (t, attr.layers[t - 1].op, attr.layers[t - 1].cout)
    logits = P.get_tensor(1, attr.outputs[0], n_roi).reshape(n_roi, -1)
    assert logits.shape[1] == 32 and rel_err(logits[:m], ref.children[0].logits) <= TOL[dtype]
    lab = P.get_labels(0)
    srt = np.sort(ref.children[0].logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 4 * TOL[dtype] * max(1.0, np.abs(ref.children[0].logits).max())
    assert np.array_equal(lab[:m][clear], ref.children[0].labels[clear])
    assert np.array_equal(lab, logits.argmax(axis=1)) and np.array_equal(boxes["child_label"][:, 0], lab)
    P.close()


@pytest.mark.parametrize("bz", [1, 4])
def test_sweep_cascade_bursty_counts(octo, bz):
    """Batch-size sweep workload (bf16, negative-binomial object counts, cap 200): post-processing and ROI routing are
    exact for every batch size; a frame with zero objects and a very crowded frame sit in one batch."""
    spec = zoo.sweep_cascade(bz)
    det = spec.models[0]
    rng = np.random.default_rng(zoo.SEED0 + 3)
    counts = synth.counts_negbin(rng, bz)
    counts[0] = 0
    if bz > 1:
        counts[1] = 90
    scene = synth.make_scene(rng, bz, 1080, 1920, counts, 24, 200, log_uniform=True)
    planted = synth.planted_heads(rng, det, scene, 1080, 1920, pre.letterbox_geometry(1080, 1920, det.in_h, det.in_w)[1:])
    dets = cascade.postprocess_heads(planted, det)
    P = octo.Pipeline(spec)
    d_heads = [octo.to_device(h, "bf16") for h in planted]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    P.submit(_frames_dev(scene.frames))
    assert P.run() == bz
    frames, boxes, st = P.collect()
    assert st == octo.OK and frames["n_boxes"].tolist() == [len(d.keep) for d in dets]
    for f, d in enumerate(dets):
        cc, top, keep = P.get_detections(0, f)
        assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist()
    rois = P.get_rois(0)
    exp = [(f, r) for f, d in enumerate(dets) for r in range(len(d.keep))]
    assert list(zip(rois["frame"].tolist(), rois["rank"].tolist())) == exp
    assert frames["n_boxes"][0] == 0
    lab = P.get_labels(0)
    assert len(lab) == len(exp) and np.array_equal(boxes["child_label"][:, 0], lab) and np.all((lab >= 0) & (lab < 1000))
    P.close()


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_every_tensor_of_a_csp_detector_with_odd_widths(octo, dtype):
    """Every intermediate tensor of a small CSP detector against the oracle, with channel counts that fill no tile
    (12, 24, 40, 72, 80, 144: ragged channel tiles, a width that is not a multiple of 8 and so takes the element-wise
    gather, outputs written into concat slices at odd offsets); once with every tensor kept and once with buffers
    reused as soon as their last reader is done."""
    from oracle import nn
    det = zoo.csp_detector("odd_det", dtype, 128, (16, 24, 48, 80, 144), (1, 2, 1, 1), 3, zoo.SEED0 + 77, batch_size=3,
                           topk=100, max_det=20)
    spec = zoo.PipelineSpec("odd", [det], [], 200.0, 96, 160, 3, 8)
    rng = np.random.default_rng(zoo.SEED0 + 78)
    scene = synth.make_scene(rng, 3, 96, 160, [3, 2, 4], 8, 48, n_classes=3)
    ref = None
    for keep_all in (True, False):
        P = octo.Pipeline(spec, keep_all_tensors=keep_all)
        P.submit(_frames_dev(scene.frames))
        assert P.run() == 3
        _, _, st = P.collect()
        assert st == octo.OK
        if keep_all:
            x0 = P.get_tensor(0, 0, 3)
            ref = nn.run_model(det, x0, keep_all=True)
            shapes = det.tensor_shapes()
            for t in range(1, len(det.layers) + 1):
                got = P.get_tensor(0, t, 3)
                assert got.shape[1:] == tuple(shapes[t]), t
                assert rel_err(got, ref[t]) <= TOL[dtype], (t, det.layers[t - 1].op, det.layers[t - 1].cout)
        else:
            for t in det.outputs:
                assert rel_err(P.get_tensor(0, t, 3), ref[t]) <= TOL[dtype], t
        P.close()


def test_detector_batch_smaller_than_the_frame_batch(octo):
    """The detector at its own batch size (executions of 4, then 2 frames of a 6-frame batch; and one frame at a
    time) with the children still on the ROIs of the whole batch: every result equals the one-execution run and the
    oracle (planted heads: integer work exact, detector heads of the last execution and child tensors within tolerance)."""
    dtype, n = "f16", 6
    spec = zoo.traffic_cascade(dtype, det_batch=n, max_rois_per_frame=24)
    det, cls, plate = spec.models
    rng = np.random.default_rng(zoo.SEED0 + 9)
    counts = np.minimum(synth.counts_poisson(rng, n, 8, 64), 12)
    counts[2] = 0
    scene = synth.make_scene(rng, n, 1080, 1920, counts, 24, 360, log_uniform=True)
    planted = synth.planted_heads(rng, det, scene, 1080, 1920, pre.letterbox_geometry(1080, 1920, det.in_h, det.in_w)[1:])
    ref = cascade.run_cascade(spec, scene.frames, planted_heads=planted)
    P = octo.Pipeline(spec)
    d_heads = [octo.to_device(h, dtype) for h in planted]
    for l, h in enumerate(d_heads):
        P.set_head(0, l, h)
    runs = {}
    for b in (0, 4, 1):
        P.set_detector_batch(b)
        P.submit(_frames_dev(scene.frames))
        assert P.run() == n
        frames, boxes, st = P.collect()
        assert st == octo.OK
        rois = [P.get_rois(e) for e in (0, 1)]
        dets = [P.get_detections(0, f) for f in range(n)]
        n_roi = len(rois[0])
        logits = P.get_tensor(1, cls.outputs[0], n_roi).reshape(n_roi, -1)
        last = n - 1 - ((n - 1) % b) if b else 0                       # first frame of the last execution
        head_last = [P.get_tensor(0, t, n - last) for t in det.outputs]
        runs[b] = (frames, boxes, rois, dets, logits, head_last, last)
    with pytest.raises(octo.OctoError):
        P.set_detector_batch(n + 1)
    P.close()
    f0, b0, r0, d0, l0, _, _ = runs[0]
    assert f0["n_boxes"].tolist() == [len(d.keep) for d in ref.dets] and f0["n_boxes"][2] == 0
    for f, d in enumerate(ref.dets):
        cc, top, keep = d0[f]
        assert cc == d.cand_count and top["idx"].tolist() == d.top.idx.tolist() and keep.tolist() == d.keep.tolist()
    assert rel_err(l0, ref.children[0].logits) <= TOL[dtype]
    for b in (4, 1):
        fb, bb, rb, db, lb, hb, last = runs[b]
        for k in ("frame_id", "n_boxes", "flags", "box_offset", "slo_met"):
            assert fb[k].tolist() == f0[k].tolist(), (b, k)
        assert bb.tobytes() == b0.tobytes(), b
        for e in (0, 1):
            assert rb[e].tobytes() == r0[e].tobytes(), (b, e)
        for f in range(n):
            assert db[f][0] == d0[f][0] and db[f][1].tobytes() == d0[f][1].tobytes() and db[f][2].tolist() == d0[f][2].tolist(), (b, f)
        assert rel_err(lb, l0) <= 1e-6                                  # same crops, same kernels
        for l, t in enumerate(det.outputs):                           # the activation buffers hold the last execution
            assert rel_err(hb[l], ref.heads[l][last:]) <= TOL[dtype], (b, l)
