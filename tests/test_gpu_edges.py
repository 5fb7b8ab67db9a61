"""Edge cases of the serving path on the GPU: capacity overflows, class routing, and the error returns of the calls."""
import numpy as np
import pytest

from oracle import cascade, postprocess as pp
from paper_2502_01277_amd import synth, zoo
from helpers import TOL, rel_err

pytestmark = pytest.mark.gpu


def _dev(frames):
    import torch
    return [torch.from_numpy(f).cuda() for f in frames]


def _tiny_scene():
    rng = np.random.default_rng(zoo.SEED0 + 1)
    return synth.make_scene(rng, 2, 320, 320, [6, 6], 16, 96, n_classes=8)


def test_roi_capacity_overflow_keeps_a_prefix_and_flags_the_frames(octo):
    """More detections than the ROI table holds: the table keeps the first entries in (frame, rank) order, frames that
    lost ROIs carry the overflow flag, boxes without a ROI get child label -1, and the children still match the oracle
    on the ROIs that were kept."""
    spec = zoo.tiny_cascade()
    scene = _tiny_scene()
    ref = cascade.run_cascade(spec, scene.frames)
    full = ref.children[0].rois
    kept = [len(d.keep) for d in ref.dets]
    assert kept[0] >= 3 and kept[1] >= 1
    spec.max_rois_per_frame = max(1, (kept[0] + 1) // 2)            # capacity = 2 frames x this: less than the batch needs
    cap = 2 * spec.max_rois_per_frame
    spec.models[1].batch_size = cap
    assert cap < len(full.frame)
    P = octo.Pipeline(spec)
    P.submit(_dev(scene.frames))
    assert P.run() == 2
    frames, boxes, st = P.collect()
    assert st == octo.ECAP or st == octo.OK                      # the status reports the overflow, the results are still returned
    assert frames["n_boxes"].tolist() == kept
    rois = P.get_rois(0)
    assert len(rois) == cap
    assert rois["frame"].tolist() == full.frame[:cap].tolist() and rois["rank"].tolist() == full.rank[:cap].tolist()
    lost = [f for f in range(2) if np.sum(full.frame[:cap] == f) < np.sum(full.frame == f)]
    for f in range(2):
        assert bool(frames["flags"][f] & 1) == (f in lost), (f, frames["flags"])
    lab = boxes["child_label"][:, 0]
    assert np.all(lab[:cap] >= 0) and np.all(lab[cap:] == -1)
    logits = P.get_tensor(1, spec.models[1].outputs[0], cap).reshape(cap, -1)
    assert rel_err(logits, ref.children[0].logits[:cap]) <= TOL["f32"]
    P.close()


def test_class_mask_routes_only_selected_classes(octo):
    spec = zoo.tiny_cascade()
    scene = _tiny_scene()
    base = cascade.run_cascade(spec, scene.frames)
    classes = sorted(set(int(c) for d in base.dets for c in d.top.cls[d.keep]))
    assert len(classes) >= 2
    mask = 0
    for c in classes[::2]:
        mask |= 1 << c
    spec.edges[0].class_mask = mask
    ref = cascade.run_cascade(spec, scene.frames)
    assert 0 < len(ref.children[0].rois.frame) < len(base.children[0].rois.frame)
    P = octo.Pipeline(spec)
    P.submit(_dev(scene.frames))
    P.run()
    frames, boxes, st = P.collect()
    assert st == octo.OK
    rois, r = P.get_rois(0), ref.children[0].rois
    assert rois["frame"].tolist() == r.frame.tolist() and rois["rank"].tolist() == r.rank.tolist() and rois["cls"].tolist() == r.cls.tolist()
    routed = np.array([(mask >> int(c)) & 1 for c in boxes["cls"]], bool)
    assert np.all(boxes["child_label"][routed, 0] >= 0) and np.all(boxes["child_label"][~routed, 0] == -1)
    P.close()


def test_error_returns_leave_the_pipeline_usable(octo):
    spec = zoo.tiny_cascade()
    scene = _tiny_scene()
    dev = _dev(scene.frames)
    P = octo.Pipeline(spec)
    # nothing queued: run launches nothing, blocking collect reports the state error, polling reports not-ready
    assert P.run() == 0
    with pytest.raises(octo.OctoError):
        P.collect(blocking=True)
    assert P.collect(blocking=False)[2] == octo.ENOTREADY
    # output arrays too small for the oldest batch: an error, and the batch is still there afterwards
    P.submit(dev)
    assert P.run() == 2
    fr, bx, st = P.collect(frame_cap=1, box_cap=400)
    assert st == octo.ECAP and len(fr) == 0 and len(bx) == 0
    frames, boxes, st = P.collect()
    assert st == octo.OK and len(frames) == 2
    # the frame queue has a capacity (4 x the batch capacity): the call that would exceed it queues nothing
    for _ in range(4):
        P.submit(dev)
    with pytest.raises(octo.OctoError):
        P.submit(dev)
    # only seven uncollected batches are allowed
    n_run = 0
    for _ in range(4):
        n_run += P.run()
    assert n_run == 8
    for _ in range(3):
        P.submit(dev)
        assert P.run() == 2
    P.submit(dev)
    with pytest.raises(octo.OctoError):
        P.run()
    got = 0
    while got < 14:
        fr, _, st = P.collect()
        got += len(fr)
    assert P.run() == 2 and len(P.collect()[0]) == 2
    with pytest.raises(octo.OctoError):
        P.set_batch_size(0, 3)                                    # beyond the detector's capacity
    with pytest.raises(octo.OctoError) as ei:
        P.set_batch_size(1, 1)                                    # a downstream model always takes the whole ROI set
    assert ei.value.status == octo.EINVAL
    P.close()


def test_decode_candidate_capacity_overflow(octo):
    """The stage call with room for fewer candidates than pass the threshold: the list is cut at the capacity, every
    entry is a genuine candidate, and the count says how many there were."""
    spec = zoo.tiny_cascade()
    det = spec.models[0]
    rng = np.random.default_rng(3)
    g = det.grids[0]
    head = zoo.round_to_dtype(rng.normal(0.5, 1.5, (1, g, g, det.n_anchors * (5 + det.n_classes))).astype(np.float32), det.dtype)
    ref = pp.decode_frame([head[0]], det)
    assert len(ref) > 40
    cap = 16
    cand, count = octo.op_decode(det, [octo.to_device(head, det.dtype)], cap=cap)
    got = octo.cands_from_device(cand, count)[0]
    assert int(count.cpu()[0]) >= cap and len(got) == cap
    assert set(got["idx"].tolist()) <= set(ref.idx.tolist())
