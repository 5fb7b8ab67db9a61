"""Co-located serving on CU-restricted streams: scheduler-lite + slot executor against solo runs and the oracle."""
import numpy as np
import pytest

from oracle import cascade, postprocess as pp, preprocess as pre
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
        # and the solo result is the oracle's post-processing of the same planted heads (frame 0 of the pool)
        d = cascade.postprocess_heads([h[:1] for h in co.heads_host[i]], det)[0]
        _, nw, nh, left, top = pre.letterbox_geometry(co.specs[i].src_h, co.specs[i].src_w, det.in_h, det.in_w)
        ref = pp.to_source_box(d.top.box[d.keep], co.specs[i].src_h, co.specs[i].src_w, nw, nh, left, top)
        b = solo[0]
        assert len(b) == len(d.keep) and b["cls"].tolist() == d.top.cls[d.keep].tolist()
        assert np.abs(np.stack([b["x1"], b["y1"], b["x2"], b["y2"]], 1) - ref).max() < 1e-3
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
