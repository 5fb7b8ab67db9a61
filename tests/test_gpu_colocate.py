"""Co-located serving on CU-restricted streams: scheduler-lite + slot executor against solo runs and the oracle."""
import numpy as np
import pytest

from oracle import cascade, nn, postprocess as pp, preprocess as pre
from paper_2502_01277_amd import executor, zoo

pytestmark = pytest.mark.gpu


def test_stream_masks_must_cover_every_die(octo):
    total = octo.device_cu_count()
    assert total % 8 == 0
    s = octo.stream_create_range(0, 64)
    octo.stream_destroy(s)
    s = octo.stream_create_range(total - 8, 8)
    octo.stream_destroy(s)
    for bad in ((4, 64), (0, 4), (0, total + 8), (8, 12)):
        with pytest.raises(octo.OctoError):
            octo.stream_create_range(*bad)


def _validate(sch, specs, total):
    """What a schedule must satisfy whatever the heuristic chose (Sec. III-C): portions on one stream do not overlap,
    every portion ends inside its stream's duty cycle, a child starts no earlier than its parent ends, and streams
    that exist at the same time do not hold more compute units than the GPU has."""
    by_stream = {}
    for (pi, mi, st, a, b, d) in sch.placements:
        if st < 0:
            continue
        assert 0 <= a < b <= d + 1e-6 and d <= specs[pi].slo_ms / 2 + 1e-6
        by_stream.setdefault(st, []).append((a, b))
        parent = {e.child: e.parent for e in specs[pi].edges}.get(mi, -1)
        if parent >= 0 and sch.placement(pi, parent)[2] >= 0:
            assert a >= sch.placement(pi, parent)[4] - 1e-4
    for st, iv in by_stream.items():
        iv.sort()
        assert all(iv[k][1] <= iv[k + 1][0] + 1e-6 for k in range(len(iv) - 1))
    assert sum(n for (_, n) in sch.stream_cus.values()) <= total
    ranges = sorted(sch.stream_cus.values())
    assert all(ranges[k][0] + ranges[k][1] <= ranges[k + 1][0] for k in range(len(ranges) - 1))


def test_three_pipelines_sixteen_cameras(octo):
    dur = 1.0
    co = executor.make_colocation(dur, pool_frames=4, det_batch=16)
    pipes = [octo.Pipeline(s) for s in co.specs]
    total = octo.device_cu_count()
    profiles = [executor.profile_pipeline(P, widths=(64, 128, 256), iters=1) for P in pipes]
    for prof in profiles:
        for m in prof:
            lat = [m.latency_ms[b] for b in sorted(m.latency_ms)]
            assert all(x > 0 for x in lat) and lat[-1] > lat[0]            # a 16x larger batch is not free
    sch = executor.plan(co.specs, profiles, co.frame_rates, co.objects_per_frame, co.burstiness, n_streams=8)
    _validate(sch, co.specs, total)
    for i, spec in enumerate(co.specs):
        assert sch.placement(i, 0)[2] >= 0, "every detector gets a portion"
        assert sch.est_latency_ms[i] <= spec.slo_ms / 2 + 1e-3
        for mi, b in enumerate(sch.bz[i]):
            assert b in profiles[i][mi].latency_ms
    ex = executor.Executor(pipes, sch, co.cameras, co.head_pools, slotted=True, masked=True, keep_results=True)
    out = ex.serve(dur)
    ex.close()
    print(out, sch)
    for i, S in enumerate(ex.stats):
        assert S.submitted > 0 and S.served == S.submitted and len(S.results) == S.served
        assert sorted(S.results) == list(range(S.served))
    assert out["slo_attainment"] == 1.0
    # every served frame must carry exactly what the same frame gives when it runs alone on an unrestricted stream
    for i, P in enumerate(pipes):
        P.set_batch_size(0, 1)
        det = co.specs[i].models[0]
        solo = []
        for k in range(len(co.scenes[i].frames)):
            for l, pool in enumerate(co.head_pools[i]):
                P.set_head(0, l, pool[k:])
            P.submit([co.cameras[[c.pipeline for c in co.cameras].index(i)].pool[k]])
            assert P.run() == 1
            fr, bx, _ = P.collect()
            solo.append(bx.copy())
        for fid, (k, bx) in ex.stats[i].results.items():
            assert bx.tobytes() == solo[k].tobytes(), (i, fid, k)
        # and every solo result is the oracle's: post-processing of the planted heads of that pool frame (boxes in source
        # pixels, classes), and the child models of the oracle on the oracle's own crops (labels where its margin is clear)
        spec = co.specs[i]
        _, nw, nh, left, top = pre.letterbox_geometry(spec.src_h, spec.src_w, det.in_h, det.in_w)
        dets = cascade.postprocess_heads(co.heads_host[i], det)
        n_clear = 0
        for k, d in enumerate(dets):
            ref = pp.to_source_box(d.top.box[d.keep], spec.src_h, spec.src_w, nw, nh, left, top)
            b = solo[k]
            assert len(b) == len(d.keep) and b["cls"].tolist() == d.top.cls[d.keep].tolist(), (i, k)
            if len(b):
                assert np.abs(np.stack([b["x1"], b["y1"], b["x2"], b["y2"]], 1) - ref).max() < 1e-3, (i, k)
            for e, edge in enumerate(spec.edges):
                child = spec.models[edge.child]
                rois = pp.compact_rois([(d.top.cls[d.keep], ref)], edge.class_mask)
                assert len(rois) == len(b)                              # every class is routed to every child here
                if len(rois) == 0:
                    continue
                crops = pre.crop_resize(co.scenes[i].frames[k:k + 1], rois.frame, rois.box, child.in_h, child.in_w, child.dtype,
                                        child.norm_scale, child.norm_bias)
                ts = nn.run_model(child, crops)
                if child.kind == "classifier":
                    logits = ts[child.outputs[0]].reshape(len(rois), -1)
                    srt = np.sort(logits, axis=1)
                    clear = (srt[:, -1] - srt[:, -2]) > 8e-2 * max(1.0, np.abs(logits).max())
                    n_clear += int(clear.sum())
                    assert np.array_equal(b["child_label"][clear, e], nn.argmax_labels(logits)[clear]), (i, k, e)
                else:
                    # a child detector reports how many boxes it keeps per ROI; its head logits are natural (random
                    # weights), so a candidate can sit within rounding of the score threshold: allow one box of slack
                    cd = cascade.postprocess_heads([ts[t] for t in child.outputs], child)
                    want = np.asarray([len(x.keep) for x in cd])
                    assert np.abs(b["child_label"][:, e] - want).max() <= 1, (i, k, e)
            assert np.all(b["child_label"][:, len(spec.edges):] == -1)
        assert n_clear > 0 or not any(spec.models[e.child].kind == "classifier" for e in spec.edges)
        P.close()


def test_unslotted_unmasked_serving_gives_the_same_results(octo):
    """The ablation's configuration (no portions: every pipeline launches as soon as frames are queued, on one
    ordinary stream) serves the same frames with the same boxes."""
    dur = 0.5
    co = executor.make_colocation(dur, n_cameras=(3, 0, 2), pool_frames=3, det_batch=8)
    specs = [co.specs[0], co.specs[2]]
    cams = [executor.Camera(0 if c.pipeline == 0 else 1, c.arrivals_s, c.pool) for c in co.cameras]
    pools = [co.head_pools[0], co.head_pools[2]]
    pipes = [octo.Pipeline(s) for s in specs]
    profiles = [executor.profile_pipeline(P, widths=(256,), iters=1) for P in pipes]
    rates = [co.frame_rates[0], co.frame_rates[2]]
    sch = executor.plan(specs, profiles, rates, [co.objects_per_frame[0], co.objects_per_frame[2]],
                        [co.burstiness[0], co.burstiness[2]], n_streams=4)
    res = []
    for slotted, masked in ((True, True), (False, False)):
        ex = executor.Executor(pipes, sch, cams, pools, slotted=slotted, masked=masked, keep_results=True)
        out = ex.serve(dur)
        ex.close()
        assert all(S.served == S.submitted and S.submitted > 0 for S in ex.stats)
        res.append([{fid: (k, bx.tobytes()) for fid, (k, bx) in S.results.items()} for S in ex.stats])
    assert res[0] == res[1]
    for P in pipes:
        P.close()


def _two_pipelines(dur, n_traffic, n_detonly, surge):
    """Traffic cascade + detector-only pipeline (half of the GPU stays free for the scaler), surge on the first."""
    co = executor.make_colocation(dur, n_cameras=(n_traffic, 0, n_detonly), pool_frames=3, det_batch=16, surge=surge)
    specs = [co.specs[0], co.specs[2]]
    cams = [executor.Camera(0 if c.pipeline == 0 else 1, c.arrivals_s, c.pool) for c in co.cameras]
    pools = [co.head_pools[0], co.head_pools[2]]
    args = ([co.frame_rates[0], co.frame_rates[2]], [co.objects_per_frame[0], co.objects_per_frame[2]],
            [co.burstiness[0], co.burstiness[2]])
    return specs, cams, pools, args


def test_surge_lazy_dropping_and_a_second_instance(octo):
    """A 3x surge on one pipeline for 0.8 s (Sec. III-D, IV-A).  The slot discipline serves at most k+1 batches per duty
    cycle, so the scheduled instance alone falls behind; dropping requests that are already late keeps the rest on
    time; a stand-by copy that Algorithm 2 places into the free part of the GPU absorbs the surge altogether.  Whatever
    instance serves a frame, its boxes are the same."""
    dur, t0, t1 = 2.0, 0.5, 1.3
    specs, cams, pools, (rates, objs, burst) = _two_pipelines(dur, 24, 8, (0, t0, t1, 3.0))
    pipes = [octo.Pipeline(s) for s in specs]
    spare = octo.Pipeline(specs[0])
    profiles = [executor.profile_pipeline(P, widths=(64, 128, 256), iters=1) for P in pipes]
    sch = executor.plan(specs, profiles, rates, objs, burst, n_streams=8)
    total = octo.device_cu_count()
    assert sum(n for (_, n) in sch.stream_cus.values()) <= total // 2, "the scenario needs free compute units"
    cap = (sch.batches_per_cycle[0][0] + 1) * sch.bz[0][0]
    in_surge = sum(int(((c.arrivals_s >= t0) & (c.arrivals_s < t1)).sum()) for c in cams if c.pipeline == 0)
    assert in_surge / ((t1 - t0) * 1e3 / sch.duty_ms) > 1.3 * cap, "the surge must exceed what the slots can take"
    runs = {}
    for tag, kw in (("plain", {}), ("drop", dict(drop_late=True)), ("scaled", dict(spares=[spare, None]))):
        ex = executor.Executor(pipes, sch, cams, pools, slotted=True, masked=True, keep_results=True, **kw)
        out = ex.serve(dur)
        ex.close()
        runs[tag] = (out, ex.stats, dict(ex.stream_cus))
        print(tag, out)
    plain, drop, scaled = runs["plain"][0], runs["drop"][0], runs["scaled"][0]
    slo = specs[0].slo_ms
    # the scheduled instance alone: everything is served, much of it late
    assert plain["dropped"] == 0 and plain["per_pipeline"][0]["served"] == plain["per_pipeline"][0]["submitted"]
    assert plain["per_pipeline"][0]["slo_met"] < 0.8 * plain["per_pipeline"][0]["submitted"]
    assert plain["per_pipeline"][1]["slo_met"] == plain["per_pipeline"][1]["submitted"], "the other pipeline keeps its slots"
    # lazy dropping: nothing is lost track of, what is served is (almost) on time, and more results count
    p0 = drop["per_pipeline"][0]
    assert p0["dropped"] > 0 and p0["served"] + p0["dropped"] == p0["submitted"]
    assert p0["latency_ms_max"] <= slo + 0.5 * sch.duty_ms      # admitted at most one SLO old, then one slot of batches
    assert p0["slo_met"] > plain["per_pipeline"][0]["slo_met"]
    # the scaler: one copy added soon after the surge began, placed on compute units nothing else uses
    ev = scaled["scale_events"]
    ups = [e for e in ev if e[2] == 1]
    assert len(ups) == 1 and ups[0][1] == 0 and t0 < ups[0][0] <= t0 + 0.7, ev
    assert all(e[2] != 0 for e in ev), "there was room, so no request may have been denied"
    downs = [e for e in ev if e[2] == -1]
    assert len(downs) <= 1 and all(e[0] > t1 for e in downs), ev        # removed, if at all, only after the surge
    cus = runs["scaled"][2]
    new = [cus[s] for s in cus if s not in sch.stream_cus]
    assert new and all(f >= max(a + b for (a, b) in sch.stream_cus.values()) and f + n <= total for (f, n) in new)
    assert scaled["dropped"] == 0 and scaled["slo_attainment"] >= 0.97, scaled
    # every frame, whichever run and instance served it: the boxes depend on the pool frame only
    ref = {}
    for tag in runs:
        for i, S in enumerate(runs[tag][1]):
            for fid, (k, bx) in S.results.items():
                assert ref.setdefault((i, k), bx.tobytes()) == bx.tobytes(), (tag, i, fid, k)
    assert len(runs["scaled"][1][0].results) == scaled["per_pipeline"][0]["submitted"]
    spare.close()
    for P in pipes:
        P.close()
