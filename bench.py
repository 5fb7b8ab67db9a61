#!/usr/bin/env python3
"""Benchmark of the cascade hot path on one MI355X.

A step is one pass of the whole path (letterbox, detector, decode, top-k, NMS, ROI compaction, crop-resize,
classifier, result copy) over one batch of the high-resolution workload, the largest single-GPU configuration: 32
synthetic 3840x2160 frames, m-shaped detector at 1280 x 1280 in bf16, planted detector heads (Pareto object counts,
top-k truncating), every ROI through the ResNet-18-shaped classifier.  The traffic workload (8 frames of 1920x1080,
fp16, four pipeline instances on their own streams) runs in the same process and is reported under the key
"traffic".  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"f16": 2500.0, "bf16": 2500.0, "f32": 157.3}    # dense MFMA TFLOP/s (fp32: vector/matrix fp32 rate)
HBM_PEAK = 8000.0                                        # GB/s


def make_workload(name: str):
    from paper_2502_01277_amd import binding, synth, zoo
    if name == "traffic":
        spec = zoo.traffic_cascade()
        rng = np.random.default_rng(zoo.SEED0 + 2)
        counts = synth.counts_poisson(rng, 8, 8.0, 64)
        scene = synth.make_scene(rng, 8, 1080, 1920, counts, 24, 360, log_uniform=True)
        heads = synth.planted_heads(rng, spec.models[0], scene, 1080, 1920, binding.letterbox_geometry(1080, 1920, spec.models[0].in_h, spec.models[0].in_w))
        desc = "traffic cascade: 8x1920x1080 u8 frames (4 cameras x 2), CSP-s detector 640 fp16, planted heads Poisson(8), " \
               "ResNet-18-shaped classifier 224 + 6-layer plate detector 128 on every ROI"
    elif name == "hires":
        spec = zoo.hires_cascade()
        rng = np.random.default_rng(zoo.SEED0 + 5)
        counts = synth.counts_pareto(rng, 32)
        scene = synth.make_scene(rng, 32, 2160, 3840, counts, 48, 720, log_uniform=True)
        heads = synth.planted_heads(rng, spec.models[0], scene, 2160, 3840, binding.letterbox_geometry(2160, 3840, spec.models[0].in_h, spec.models[0].in_w), n_clutter=1100)
        desc = "high-resolution cascade: 32x3840x2160 frames, CSP-m detector 1280 bf16, planted heads Pareto(1.5), ResNet-18-shaped classifier"
    elif name == "tiny":
        spec = zoo.tiny_cascade()
        rng = np.random.default_rng(zoo.SEED0 + 1)
        scene = synth.make_scene(rng, 2, 320, 320, [6, 6], 16, 96, n_classes=8)
        heads = None
        desc = "tiny fp32 cascade: 2x320x320 frames, natural heads"
    else:
        raise SystemExit("unknown workload %s" % name)
    return spec, scene, heads, desc


def conv_name(kid: int, dtype: str) -> str:
    """Template instance behind a conv kernel id (digits 1 BBB PPP K M V), as rocprofv3 prints it."""
    d = kid - 1000000000
    ctype = {"f16": "_Float16", "bf16": "__bf16", "f32": "float", "f8": "octo::f8"}[dtype]
    if 700000000 <= d < 800000000:                       # wide 3x3 kernel: digits P BBB TTT (512-pixel tile, channel tile, tile width)
        bc = ((d - 700000000) // 1000) % 1000
        tc, tp, wc = (3, 4, 1) if bc == 96 else (bc // 64, 4, 2)
        return "octo::conv3x3_big_kernel<%s, %d, %d, %d, 4>" % (ctype, tc, tp, wc)
    if 800000000 <= d < 900000000:                       # 3x3 kernel with the input patch in LDS: channel slice
        return "octo::conv3x3_patch_kernel<%s, %d, %d>" % (ctype, (d - 800000000) % 1000, (d - 800000000) // 1000)
    if d >= 900000000:                                   # first-layer kernel: digits BBB KK P
        d -= 900000000                                   # F BBB KK P: F = 1 with the following max-pool fused
        return "octo::stem_conv_kernel<%s, %d, %d, %d, %s>" % (ctype, (d // 1000) % 1000, (d // 10) % 100, d % 10, "true" if d >= 1000000 else "false")
    bc, bp, kv, minb, v = d // 1000000, (d // 1000) % 1000, (d // 100) % 10, (d // 10) % 10, d % 10
    vec, dma = v & 1, v >> 1
    wc, wp = (1, 4) if (bc == 32 or bp == 256) else (2, 2)
    depth = 1 if dma else 2
    return "octo::conv_mfma_kernel<%s, %d, %d, %d, %d, %d, %d, %d, %s, %s>" % (
        ctype, bc, bp, wc, wp, kv, depth, minb, "true" if vec else "false", "true" if dma else "false")


# HBM traffic per launch of the dominant kernel, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of
# `bench.py --calib-copy-mib 256` (counters in KiB per dispatch, scaled by what the same counter reads for the
# calibration pass of known size).  Valid only for the kernel sources it was taken with: keyed by their hash.
TRAFFIC = {
    # hash of the convolution sources (conv_sources_key): {kernel name: HBM bytes per launch}
    "93d07c228e907e2c": {
        "octo::conv_mfma_kernel<__bf16, 128, 128, 2, 2, 8, 1, 2, true, true>": 624532799,
        "octo::conv3x3_patch_kernel<__bf16, 64, 64>": 4275894878,
        "octo::conv_mfma_kernel<__bf16, 64, 256, 1, 4, 4, 1, 3, true, true>": 412985885,
        "octo::conv3x3_big_kernel<__bf16, 4, 4, 2, 4>": 1153790470,
        "octo::stem_conv_kernel<__bf16, 64, 7, 4, true>": 3409215376,
        "octo::conv3x3_big_kernel<__bf16, 3, 4, 1, 4>": 526039832,
        "octo::conv3x3_big_kernel<__bf16, 3, 4, 2, 4>": 244944910,
        "octo::stem_conv_kernel<__bf16, 64, 6, 3, false>": 1753120816,
        "octo::conv_mfma_kernel<__bf16, 64, 128, 2, 2, 8, 1, 3, true, true>": 541911139,
        "octo::conv_mfma_kernel<_Float16, 128, 128, 2, 2, 8, 1, 2, true, true>": 29254610,
        "octo::conv_mfma_kernel<_Float16, 64, 128, 2, 2, 8, 1, 3, true, true>": 18779512,
        "octo::conv3x3_patch_kernel<_Float16, 64, 64>": 69226266,
        "octo::stem_conv_kernel<_Float16, 32, 6, 3, false>": 78867677,
        "octo::conv_mfma_kernel<_Float16, 64, 64, 2, 2, 8, 1, 4, true, true>": 6645295,
        "octo::stem_conv_kernel<_Float16, 64, 7, 4, true>": 55154702,
        "octo::conv_mfma_kernel<_Float16, 32, 128, 1, 4, 4, 2, 4, true, false>": 13644829,
        "octo::conv3x3_patch_kernel<_Float16, 32, 64>": 39928727,
        "octo::stem_conv_kernel<_Float16, 32, 3, 2, false>": 18000958,
    },
}


TRAFFIC_SOURCE = "profiles/*_hbm_counters.md: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs of this command, scaled by the " \
                 "same counters on a copy of known size; looked up by the hash of the convolution sources they were taken with"


def conv_sources_key() -> str:
    import hashlib
    h = hashlib.sha256()
    for f in ("conv.hip", "convbig.hip", "conv3x3.hip", "stem.hip", "mfma_common.h"):
        try:
            h.update(open(os.path.join(ROOT, "paper_2502_01277_amd", "csrc", f), "rb").read())
        except OSError:
            pass
    return h.hexdigest()[:16]


def traffic_per_launch(kernel_name: str):
    """(HBM bytes per launch from the committed counter runs, where they come from), or (None, why not): the figure is
    only valid for the kernel sources it was measured with."""
    got = TRAFFIC.get(conv_sources_key(), {}).get(kernel_name)
    if got is None:
        return None, "no counter run for the current convolution sources (key %s); see profiles/ for the last one" % conv_sources_key()
    return got, TRAFFIC_SOURCE


def cpu_baseline(spec, scene, heads, min_seconds=10.0, max_batches=8, subset=False, rois_per_frame=None):
    """The oracle, as it stands, on the same workload, bounded to tens of seconds of CPU work.

    Default: whole batches until about 10 s are done.  subset (batches that would take many minutes): the first frame
    only, twice, with 8 and with 24 of its ROIs per child; the difference gives the time per ROI, the rest the time per
    frame, and the rate is put together with the batch's mean ROI count per frame and child, as the GPU run found it
    (said so in `sample`)."""
    import torch
    from oracle import cascade
    n = scene.frames.shape[0]
    cores = int(torch.get_num_threads())
    if subset:
        h1 = [h[:1] for h in heads] if heads is not None else None
        times = []
        for m in (8, 24):
            t0 = time.time()
            ref = cascade.run_cascade(spec, scene.frames[:1], planted_heads=h1, max_child_rois=m)
            times.append(time.time() - t0)
        got = [min(len(ref.children[e].rois), 24) - min(len(ref.children[e].rois), 8) for e in ref.children]
        per_roi = (times[1] - times[0]) / max(1, sum(got)) if sum(got) > 0 else 0.0            # all children together
        n_children = max(1, len(ref.children))
        first8 = sum(min(len(ref.children[e].rois), 8) for e in ref.children)
        per_frame = max(1e-9, times[0] - per_roi * first8)
        if rois_per_frame is None:
            rois_per_frame = float(np.mean([len(r) for r in scene.rects]))
        t_frame = per_frame + per_roi * rois_per_frame * n_children
        return {"value": 1.0 / t_frame, "unit": "frames/s", "cores": cores, "kind": "oracle",
                "sample": "first frame of the batch with 8 and with 24 ROIs per child (%.1f s + %.1f s): %.2f s per frame without ROIs, "
                          "%.3f s per ROI, extrapolated to the batch's mean of %.1f ROIs per frame" %
                          (times[0], times[1], per_frame, per_roi, rois_per_frame)}, None
    t0 = time.time()
    reps = 0
    while True:
        ref = cascade.run_cascade(spec, scene.frames, planted_heads=heads)
        reps += 1
        dt = time.time() - t0
        if dt >= min_seconds or reps >= max_batches:
            break
    return {"value": reps * n / dt, "unit": "frames/s", "cores": cores, "kind": "oracle",
            "sample": "%d full batch(es) of %d frames through the whole cascade (%d ROIs per child), %.1f s" %
                      (reps, n, len(ref.children[0].rois) if ref.children else 0, dt)}, ref


def run_sweep(args):
    """Batch-size sweep (the paper's Observation 2: throughput and latency against batch size): detector + classifier,
    bf16, negative-binomial object counts, every batch size from 1 to 64 at its real shape."""
    import torch
    from paper_2502_01277_amd import binding, synth, zoo
    n_cu = binding.device_cu_count()
    ninst = max(1, args.instances)
    streams = [binding.stream_create_range(0, n_cu) for _ in range(ninst)]
    now = binding.lib().octo_now_ms
    rows = []
    for bz in (1, 2, 4, 8, 16, 32, 64):
        spec = zoo.sweep_cascade(bz)
        det = spec.models[0]
        rng = np.random.default_rng(zoo.SEED0 + 3)
        counts = synth.counts_negbin(rng, bz)
        scene = synth.make_scene(rng, bz, 1080, 1920, counts, 24, 200, log_uniform=True)
        heads = synth.planted_heads(rng, det, scene, 1080, 1920, binding.letterbox_geometry(1080, 1920, det.in_h, det.in_w))
        dev = [torch.from_numpy(f).cuda() for f in scene.frames]
        pipes, keep = [], []
        for _ in range(ninst):
            P = binding.Pipeline(spec)
            dh = [binding.to_device(h, det.dtype) for h in heads]
            for l, h in enumerate(dh):
                P.set_head(0, l, h)
            keep.append(dh); pipes.append(P)
        # batch latency alone on the GPU
        solo = []
        for k in range(10 + 30):
            pipes[0].submit(dev, arrival_ms=[now()] * bz); pipes[0].run(streams[0])
            fr, _, _ = pipes[0].collect()
            if k >= 10:
                solo.append(float(fr["latency_ms"].max()))
        # throughput with all instances busy
        steps = max(50, args.steps // 4)
        lat, met, done = [], 0, 0
        pend = [0] * ninst
        def take(j):
            nonlocal met, done
            fr, _, _ = pipes[j].collect()
            pend[j] -= len(fr) // bz; done += len(fr); met += int(fr["slo_met"].sum()); lat.extend(fr["latency_ms"].tolist())
        for k in range(10):
            pipes[k % ninst].submit(dev); pipes[k % ninst].run(streams[k % ninst]); pipes[k % ninst].collect()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            j = k % ninst
            if pend[j] >= 2:
                take(j)
            pipes[j].submit(dev, arrival_ms=[now()] * bz); pipes[j].run(streams[j]); pend[j] += 1
        for j in range(ninst):
            while pend[j] > 0:
                take(j)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        rows.append({"bz": bz, "objects_per_batch": int(counts.sum()), "batch_latency_ms_p50": float(np.percentile(solo, 50)),
                     "batch_latency_ms_p99": float(np.percentile(solo, 99)), "frames_per_s": done / dt,
                     "slo_met_frames_per_s": met / dt, "latency_ms_p99_loaded": float(np.percentile(lat, 99))})
        print("bz %2d  objects %4d  latency %.2f ms  %.0f frames/s" % (bz, counts.sum(), rows[-1]["batch_latency_ms_p50"], done / dt), file=sys.stderr)
        torch.cuda.synchronize()
        for P in pipes:
            P.close()
        del pipes, keep, dev
    best = max(rows, key=lambda r: r["slo_met_frames_per_s"])
    for st in streams:
        binding.stream_destroy(st)
    print(json.dumps({
        "metric": "pipeline frames/s within 200 ms SLO on 1 GPU", "value": best["slo_met_frames_per_s"], "unit": "frames/s",
        "n_gpus": 1, "steps": max(50, args.steps // 4), "warmup": 10, "ms_per_step": 1e3 * best["bz"] / best["frames_per_s"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "batch-size sweep: CSP-s detector 640 + ResNet-18-shaped classifier 224, bf16, 1080p frames, "
                               "planted heads NegBin(mean 6, var 60) cap 200", "best_bz": best["bz"], "instances": ninst,
                   "slo_ms": 200.0, "heads": "planted"},
        "sweep": rows}))


def run_colocate(args):
    """Three pipelines and sixteen cameras sharing the GPU (Sec. III-C): scheduler-lite + slot executor on CU-range
    streams, and for comparison the same load without portions (one ordinary stream, launch on arrival)."""
    import torch
    from paper_2502_01277_amd import binding, executor
    dur = args.duration
    scale = max(1, args.camera_scale)
    co = executor.make_colocation(dur, n_cameras=(6 * scale, 6 * scale, 4 * scale), pool_frames=8, det_batch=args.det_batch,
                                  slo_ms=args.slo_ms)
    pipes = [binding.Pipeline(s) for s in co.specs]
    profiles = [executor.profile_pipeline(P, widths=(64, 128, 256), iters=2) for P in pipes]
    sch = executor.plan(co.specs, profiles, co.frame_rates, co.objects_per_frame, co.burstiness, n_streams=8)
    # the paper's ablations (Sec. IV-C): no spatiotemporal portions (launch on arrival, one ordinary stream), and
    # static batch sizes (detector 8, downstream models 2) under the same portion scheduler
    static = executor.plan(co.specs, profiles, co.frame_rates, co.objects_per_frame, co.burstiness, n_streams=8,
                           fixed_bz=[[min(8, args.det_batch)] + [2] * (len(s.models) - 1) for s in co.specs])
    res = {}
    for tag, plan_, slotted, masked in (("portions", sch, True, True), ("no_portions", sch, False, False),
                                        ("static_batch", static, True, True)):
        ex = executor.Executor(pipes, plan_, co.cameras, co.head_pools, slotted=slotted, masked=masked)
        res[tag] = ex.serve(dur)
        ex.close()
    out = res["portions"]
    print(json.dumps({
        "metric": "pipeline frames/s within %g ms SLO on 1 GPU" % args.slo_ms, "value": out["effective_frames_per_s"], "unit": "frames/s",
        "n_gpus": 1, "steps": int(1e3 * dur / sch.duty_ms), "warmup": 1, "ms_per_step": sch.duty_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "co-location: traffic + surveillance + detector-only pipelines, %d cameras at 15 fps "
                               "(sinusoidal), %.0f s, planted heads Poisson(8); offered load %.0f frames/s" %
                               (16 * scale, dur, sum(co.frame_rates)), "slo_ms": args.slo_ms, "heads": "planted"},
        "schedule": {"duty_ms": sch.duty_ms, "bz": sch.bz, "batches_per_cycle": sch.batches_per_cycle,
                     "placements": sch.placements, "stream_cus": {str(k): v for k, v in sch.stream_cus.items()},
                     "est_latency_ms": sch.est_latency_ms, "widths": [[m.util for m in pr] for pr in profiles]},
        "portions": res["portions"], "no_portions": res["no_portions"], "static_batch": res["static_batch"],
        "static_batch_schedule": {"bz": static.bz, "batches_per_cycle": static.batches_per_cycle}}))
    for P in pipes:
        P.close()


def run_placement(args):
    """Cross-device placement (Algorithm 1, ToEdge) as a host simulation: the traffic cascade with its batch latencies
    measured on this GPU - the "edge device" is a stream of --edge-cus compute units (default 8), the "server" one of the rest - and a synthetic
    bandwidth trace; for every bandwidth the batch sizes are searched on the server (octo_cwd_search) and the models then
    moved towards the edge (octo_to_edge).  Nothing is served across devices: the line reports placements and estimates."""
    from paper_2502_01277_amd import binding, executor, zoo
    spec = zoo.traffic_cascade(dtype="bf16", det_batch=16)
    P = binding.Pipeline(spec)
    grid = [1, 2, 4, 8, 16]
    ecu = args.edge_cus
    scu = binding.device_cu_count() - ecu
    prof = executor.profile_pipeline(P, widths=(ecu, scu), iters=3, det_batches=grid, child_batches=[1, 2, 4, 8, 16, 32, 64, 128])
    P.close()
    fps, objs = 15.0 * args.camera_scale, 8.0
    h, w = spec.src_h, spec.src_w
    parent = {e.child: e.parent for e in spec.edges}
    models = []
    for mi, m in enumerate(spec.models):
        in_bytes = float(h * w * 3) if mi == 0 else float(m.in_h * m.in_w * 3)
        models.append(dict(parent=parent.get(mi, -1), rate=fps * (objs if mi else 1.0), burstiness=0.0 if mi == 0 else 1.0,
                           server_ms=dict(prof[mi].by_width[scu]), edge_ms=dict(prof[mi].by_width[ecu]), in_bytes=in_bytes,
                           result_bytes=32.0 * (objs if mi == 0 else 1.0), weight_mem=1.0, inter_mem=0.0, util=1.0))
    rows = []
    for mbit in (5, 20, 50, 100, 200, 500, 1000, 2000, 5000, 20000):
        bw = mbit * 1e6 / 8.0
        sm = [dict(parent=m["parent"], profile=m["server_ms"], rate=m["rate"], burstiness=m["burstiness"], util=1.0, bz=1) for m in models]
        bzs = binding.cwd_search(sm, spec.slo_ms)
        placed, lat, thr = binding.to_edge([dict(m, bz=b) for m, b in zip(models, bzs)], spec.slo_ms, bw, args.alpha)
        rows.append({"mbit_per_s": mbit, "server_bz": bzs, "on_edge": [int(e) for e, _ in placed], "bz": [b for _, b in placed],
                     "est_latency_ms": lat, "est_throughput_per_s": thr})
        print("%6d Mbit/s  edge %s  bz %s  latency %.1f ms  throughput %.1f /s" % (mbit, rows[-1]["on_edge"], rows[-1]["bz"], lat, thr), file=sys.stderr)
    best = max(rows, key=lambda r: r["est_throughput_per_s"])
    print(json.dumps({
        "metric": "pipeline frames/s within 200 ms SLO on 1 GPU", "value": best["est_throughput_per_s"], "unit": "frames/s (estimate, Eq. 2)",
        "n_gpus": 1, "steps": len(rows), "warmup": 0, "ms_per_step": 0.0, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "placement simulation: traffic cascade, edge = %d compute units, server = %d, %g frames/s x %g objects, "
                               "synthetic bandwidth trace, alpha %g" % (ecu, scu, fps, objs, args.alpha), "slo_ms": spec.slo_ms},
        "profiles_ms": {"edge": [p.by_width[ecu] for p in prof], "server": [p.by_width[scu] for p in prof]},
        "placement": rows}))


def run_conv8(args):
    """The 8-bit floating-point (E4M3) variant of the convolution kernel against the bf16 kernels, layer by layer: every
    convolution of the high-resolution cascade's two models whose input channels come in 16s (all but the two first
    layers), at the batch the cascade serves (32 frames, 4170 ROIs), each run alone through octo_op_conv on random
    tensors of identical shape.  bf16 takes whichever kernel the pipeline would (patch, wide or general); E4M3 has the
    general kernel only."""
    import torch
    from paper_2502_01277_amd import binding, zoo
    spec = zoo.hires_cascade()
    batches = [32, 4170]
    reps = max(3, min(args.steps, 20))
    peak8 = binding.probe_mfma("f8", 20000, 3)
    peak16 = binding.probe_mfma("bf16", 20000, 3)
    gen = torch.Generator(device="cuda"); gen.manual_seed(1234)
    rows, seen = [], {}
    for mi, m in enumerate(spec.models):
        shp = m.tensor_shapes()
        n = batches[mi]
        for li, L in enumerate(m.layers):
            if L.op != "conv":
                continue
            h, w, cin = shp[L.inputs[0]]
            if cin % 16:
                continue
            has_res = L.res_mode != 0 and len(L.inputs) > 1
            key = (n, h, w, cin, L.cout, L.kh, L.stride, L.pad, L.act, L.res_mode if has_res else 0)
            if key in seen:
                seen[key]["count"] += 1
                continue
            ho, wo = (h + 2 * L.pad - L.kh) // L.stride + 1, (w + 2 * L.pad - L.kw) // L.stride + 1
            flop = 2.0 * n * ho * wo * L.cout * cin * L.kh * L.kw
            row = {"model": m.name, "layer": li, "n": n, "h": h, "w": w, "cin": cin, "cout": L.cout, "k": L.kh, "stride": L.stride,
                   "residual": bool(has_res), "count": 1, "gflop": flop / 1e9}
            K = L.kh * L.kw * cin
            for dt in ("bf16", "f8"):
                es = 2 if dt == "bf16" else 1
                if dt == "bf16":
                    wraw = (np.random.default_rng(li).standard_normal((L.cout, L.kh, L.kw, cin)) / np.sqrt(K)).astype(np.float32)
                    layer = binding.ConvOp(binding.to_storage(wraw, "bf16"), np.zeros(L.cout, np.float32), "bf16", L.stride, L.pad, L.act)
                    x = torch.randn((n, h, w, cin), device="cuda", dtype=torch.bfloat16, generator=gen)
                    y = torch.empty((n, ho, wo, L.cout), device="cuda", dtype=torch.bfloat16)
                    res = torch.randn((n, ho, wo, L.cout), device="cuda", dtype=torch.bfloat16, generator=gen) if has_res else None
                else:
                    wr = np.random.default_rng(li)
                    wraw = (wr.integers(0, 0x40, (L.cout, L.kh, L.kw, cin)) | (wr.integers(0, 2, (L.cout, L.kh, L.kw, cin)) << 7)).astype(np.uint8)
                    layer = binding.ConvOp(wraw, np.zeros(L.cout, np.float32), "f8", L.stride, L.pad, L.act, scale=np.full(L.cout, 1.0 / np.sqrt(K), np.float32))
                    x = torch.randint(0, 0x48, (n, h, w, cin), device="cuda", dtype=torch.uint8, generator=gen)       # magnitudes up to 3.75
                    x |= torch.randint(0, 2, (n, h, w, cin), device="cuda", dtype=torch.uint8, generator=gen) << 7
                    y = torch.empty((n, ho, wo, L.cout), device="cuda", dtype=torch.uint8)
                    res = torch.randint(0, 0x48, (n, ho, wo, L.cout), device="cuda", dtype=torch.uint8, generator=gen) if has_res else None
                kw = dict(res=res, res_mode=L.res_mode if has_res else 0, res_scale=1.0, y_inv_scale=1.0)
                kid = binding.op_conv(layer, x, y, **kw)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
                ev[0].record()
                for r in range(reps):
                    binding.op_conv(layer, x, y, **kw)
                    ev[r + 1].record()
                torch.cuda.synchronize()
                ms = float(np.median([ev[r].elapsed_time(ev[r + 1]) for r in range(reps)]))
                nbytes = es * (x.numel() + y.numel() + (res.numel() if has_res else 0))
                row[dt] = {"ms": ms, "tflops": flop / ms / 1e9, "gb_per_s": nbytes / ms / 1e6, "kernel": conv_name(kid, dt)}
                del x, y, res, layer
            row["speedup"] = row["bf16"]["ms"] / row["f8"]["ms"]
            seen[key] = row
            rows.append(row)
            print("%-10s %3d  n %4d %4dx%-4d %4d>%-4d k%d s%d %s  bf16 %7.3f ms %6.0f TF  e4m3 %7.3f ms %6.0f TF  x%.2f" %
                  (m.name, li, n, h, w, cin, L.cout, L.kh, L.stride, "r" if has_res else " ", row["bf16"]["ms"], row["bf16"]["tflops"],
                   row["f8"]["ms"], row["f8"]["tflops"], row["speedup"]), file=sys.stderr)
    tot16 = sum(r["bf16"]["ms"] * r["count"] for r in rows)
    tot8 = sum(r["f8"]["ms"] * r["count"] for r in rows)
    flops = sum(r["gflop"] * r["count"] for r in rows) * 1e9
    # the E4M3 kernel variant that takes the most time
    by_kernel = {}
    for r in rows:
        d = by_kernel.setdefault(r["f8"]["kernel"], [0.0, 0.0, 0.0])
        d[0] += r["f8"]["ms"] * r["count"]; d[1] += r["gflop"] * r["count"] * 1e9; d[2] += r["count"]
    dom = max(by_kernel, key=lambda k_: by_kernel[k_][0])
    ach = by_kernel[dom][1] / by_kernel[dom][0] / 1e9
    print(json.dumps({
        "metric": "pipeline frames/s within 200 ms SLO on 1 GPU", "value": 32.0 / (tot8 * 1e-3), "unit": "frames/s (convolution layers only, E4M3)",
        "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": tot8, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f8e4m3", "data": "synthetic",
        "config": {"workload": "convolution layers of the high-resolution cascade (32 frames, 4170 ROIs; all but the two 3-channel first layers), "
                               "each alone through octo_op_conv, E4M3 against bf16"},
        "bf16_ms": tot16, "e4m3_ms": tot8, "speedup": tot16 / tot8, "conv_tflops_bf16": flops / tot16 / 1e9, "conv_tflops_e4m3": flops / tot8 / 1e9,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": 5000.0, "unit": "TFLOP/s", "frac": ach / 5000.0, "traffic": None,
                     "frac_of_measured": ach / peak8, "launches": by_kernel[dom][2], "ms": by_kernel[dom][0]},
        "measured_peaks": {"mfma_e4m3_tflops": peak8, "mfma_bf16_tflops": peak16},
        "layers": rows}))


def run_surge(args):
    """A workload surge between two runs of the scheduler (Sec. III-D, IV-A): traffic cascade + detector-only pipeline
    on half of the GPU; the cameras of the first send --surge-factor x as many frames during the middle third.  Served by
    the scheduled instances alone, with lazy dropping of late requests, and with the run-time scaler (a stand-by copy
    that Algorithm 2 places into free portions)."""
    from paper_2502_01277_amd import binding, executor
    dur, scale = args.duration, max(1, args.camera_scale)
    t0, t1 = dur / 3.0, 2.0 * dur / 3.0
    co = executor.make_colocation(dur, n_cameras=(6 * scale, 0, 4 * scale), pool_frames=8, det_batch=args.det_batch,
                                  slo_ms=args.slo_ms, surge=(0, t0, t1, args.surge_factor))
    specs = [co.specs[0], co.specs[2]]
    cams = [executor.Camera(0 if c.pipeline == 0 else 1, c.arrivals_s, c.pool) for c in co.cameras]
    pools = [co.head_pools[0], co.head_pools[2]]
    pipes = [binding.Pipeline(s) for s in specs]
    spares = [binding.Pipeline(specs[0]), None]
    profiles = [executor.profile_pipeline(P, widths=(64, 128, 256), iters=2) for P in pipes]
    sch = executor.plan(specs, profiles, [co.frame_rates[0], co.frame_rates[2]], [co.objects_per_frame[0], co.objects_per_frame[2]],
                        [co.burstiness[0], co.burstiness[2]], n_streams=8)
    res = {}
    for tag, kw in (("scheduled_only", {}), ("lazy_dropping", dict(drop_late=True)), ("scaler", dict(spares=spares)),
                    ("scaler_and_dropping", dict(spares=spares, drop_late=True))):
        ex = executor.Executor(pipes, sch, cams, pools, slotted=True, masked=True, **kw)
        res[tag] = ex.serve(dur)
        res[tag]["stream_cus"] = {str(k): v for k, v in ex.stream_cus.items()}
        ex.close()
    out = res["scaler"]
    print(json.dumps({
        "metric": "pipeline frames/s within %g ms SLO on 1 GPU" % args.slo_ms, "value": out["effective_frames_per_s"], "unit": "frames/s",
        "n_gpus": 1, "steps": int(1e3 * dur / sch.duty_ms), "warmup": 1, "ms_per_step": sch.duty_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "surge: traffic cascade (%d cameras) + detector-only pipeline (%d cameras) at 15 fps, %.0f s; "
                               "the traffic cameras send %gx the frames for %.2f s <= t < %.2f s; planted heads Poisson(8)" %
                               (6 * scale, 4 * scale, dur, args.surge_factor, t0, t1), "slo_ms": args.slo_ms, "heads": "planted"},
        "schedule": {"duty_ms": sch.duty_ms, "bz": sch.bz, "batches_per_cycle": sch.batches_per_cycle,
                     "placements": sch.placements, "stream_cus": {str(k): v for k, v in sch.stream_cus.items()}},
        **res}))
    for P in pipes + [spares[0]]:
        P.close()


def hbm_rooflines(spec, scene, pipe, stage, names, n, measured_copy):
    """Achieved HBM GB/s of the three large pre/post-processing kernels, from their algorithmic bytes (what the step must
    move whatever the kernel: unique source pixels tapped + output elements for letterbox, every head element + one
    record per candidate for decode, min(4 taps per output pixel, the box's own pixels) + output elements per ROI for
    crop-resize) and the event-timed duration of their stage on the pipeline's stream."""
    from paper_2502_01277_amd import binding
    det = spec.models[0]
    es = 4 if det.dtype == "f32" else 2
    st = dict(zip(names, stage))
    out = []
    # letterbox (K1): the resized image is nw x nh inside the det.in_h x det.in_w canvas
    r = min(det.in_h / spec.src_h, det.in_w / spec.src_w)
    nw, nh = int(spec.src_w * r + 0.5), int(spec.src_h * r + 0.5)
    kx = spec.src_w / nw
    taps = 1 if (spec.src_w % nw == 0 and spec.src_h % nh == 0 and int(kx) % 2 == 1) else 4     # odd integer ratio: taps fall on pixel centres
    usrc = min(nw * nh * taps, spec.src_w * spec.src_h)
    out.append(("letterbox_kernel", "letterbox", n * (3 * usrc + det.in_h * det.in_w * 3 * es)))
    # decode (K5)
    cands = sum(int(pipe.get_detections(0, f)[0]) for f in range(n))
    out.append(("decode_stream_kernel", "decode", n * det.n_cand() * (5 + det.n_classes) * es + 32 * cands))
    # crop-resize (K9), first edge
    if spec.edges:
        child = spec.models[spec.edges[0].child]
        ces = 4 if child.dtype == "f32" else 2
        rois = pipe.get_rois(0)
        w = np.maximum(rois["x2"] - rois["x1"], 1.0); h = np.maximum(rois["y2"] - rois["y1"], 1.0)
        src = np.minimum(4.0 * child.in_h * child.in_w, np.ceil(w) * np.ceil(h)) * 3
        out.append(("crop_resize_rows_kernel", "crop0", float(src.sum()) + len(rois) * child.in_h * child.in_w * 3 * ces))
    res = []
    for kernel, key, nbytes in out:
        us = 1e3 * float(st[key])
        gbps = nbytes / (us * 1e-6) / 1e9 if us > 0 else 0.0
        res.append({"kernel": kernel, "stage": key, "bound": "hbm", "algorithmic_bytes": float(nbytes), "stage_us": us, "achieved": gbps,
                    "peak": HBM_PEAK, "unit": "GB/s", "frac": gbps / HBM_PEAK,
                    "frac_of_measured": gbps / measured_copy if measured_copy else None})
    return res


def bench_cascade(args, workload, steps, warmup, ninst, measured, with_cpu):
    """One workload: `warmup` untimed and `steps` timed batches of the whole cascade, then the same steps with timing
    events for the per-kernel figures.  Returns the JSON object of the run."""
    import torch
    from paper_2502_01277_amd import binding
    spec, scene, heads, desc = make_workload(workload)
    det = spec.models[0]
    n = scene.frames.shape[0]
    pipes, keep_heads = [], []
    for _ in range(ninst):
        P = binding.Pipeline(spec)
        if getattr(args, "det_exec", 0):
            P.set_detector_batch(args.det_exec)
        if heads is not None:
            dh = [binding.to_device(h, det.dtype) for h in heads]
            for l, h in enumerate(dh):
                P.set_head(0, l, h)
            keep_heads.append(dh)
        pipes.append(P)
    dev = [torch.from_numpy(f).cuda() for f in scene.frames]
    # one stream per instance, created by the library over all compute units: each gets a hardware queue of its own
    # (streams from a framework's pool may share one, which serialises the instances that land on it)
    n_cu = binding.device_cu_count()
    streams = [binding.stream_create_range(0, n_cu) for _ in range(ninst)]
    now = binding.lib().octo_now_ms

    def region(k_steps, on_collect, use=None):
        """`k_steps` batches, taken in turn by the instances in `use`; each instance keeps at most two uncollected
        batches, so the host prepares and collects while the GPU works."""
        use = list(range(ninst)) if use is None else use
        pend = {j: 0 for j in use}
        for k in range(k_steps):
            j = use[k % len(use)]
            if pend[j] >= 2:
                fr, bx, st = pipes[j].collect()
                pend[j] -= len(fr) // n
                on_collect(j, fr)
            pipes[j].submit(dev, arrival_ms=[now()] * n)
            pipes[j].run(streams[j])
            pend[j] += 1
        for j in use:
            while pend[j] > 0:
                fr, bx, st = pipes[j].collect()
                pend[j] -= len(fr) // n
                on_collect(j, fr)

    region(warmup, lambda j, fr: None)
    if args.calib_copy_mib and workload == args.workload:
        src = torch.full((args.calib_copy_mib << 18,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)           # one elementwise kernel: reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    # ---- timed region: K steps, inputs resident in HBM ----
    lat, tot = [], {"met": 0, "boxes": 0, "frames": 0}

    def tally(j, fr):
        lat.extend(fr["latency_ms"].tolist())
        tot["met"] += int(fr["slo_met"].sum()); tot["boxes"] += int(fr["n_boxes"].sum()); tot["frames"] += len(fr)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    region(steps, tally)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert tot["frames"] == n * steps
    # ---- the same steps again with timing events on every layer: once with one instance alone (a kernel's own
    # duration, which is what a profiler that serialises dispatches reports) and once with all instances overlapping
    items = [n] + [0] * (len(spec.models) - 1)          # items each model processes per step (same batch every step)
    for e, edge in enumerate(spec.edges):
        items[edge.child] = len(pipes[0].get_rois(e))

    def timing_pass(k_steps, use):
        agg, stage = {}, []      # kernel id -> [time ms, flops, bytes, launches]

        def per_layer(j, fr):
            stage.append(pipes[j].stage_ms())            # timings of the newest batch of this collect
            for mi, m in enumerate(spec.models):
                ms, kid, fl, by, wb = pipes[j].layer_info(mi)
                for q in range(len(ms)):
                    if kid[q] == 0:
                        continue
                    a = agg.setdefault(int(kid[q]), [0.0, 0.0, 0.0, 0])
                    a[0] += float(ms[q]); a[1] += fl[q] * items[mi]; a[2] += by[q] * items[mi] + wb[q]; a[3] += 1

        for P in pipes:
            P.set_layer_timing(True); P.set_stage_timing(True)
        region(k_steps, per_layer, use)
        for P in pipes:
            P.set_layer_timing(False); P.set_stage_timing(False)
        return agg, np.mean(np.stack(stage), axis=0), len(stage)

    agg, stage, nsamp = timing_pass(max(4, min(steps, 60)), [0])
    agg_ov, stage_ov, nsamp_ov = timing_pass(min(steps, 120), None) if ninst > 1 else (agg, stage, nsamp)
    conv = {k: v for k, v in agg.items() if k >= 1000000000}
    dom = max(conv, key=lambda k: conv[k][0])
    t_ms, fl, by, launches = conv[dom]
    kname = conv_name(dom, det.dtype)
    achieved = fl / (t_ms * 1e-3) / 1e12
    traffic, traffic_source = traffic_per_launch(kname)
    roofline = {"bound": "mfma", "kernel": kname, "achieved": achieved, "peak": PEAK[det.dtype], "unit": "TFLOP/s",
                "frac": achieved / PEAK[det.dtype], "traffic": traffic, "traffic_source": traffic_source,
                "frac_of_measured": achieved / measured["mfma_tflops"] if measured.get("mfma_tflops") else None,
                "avg_launch_us": 1e3 * t_ms / launches, "launches_per_step": launches / nsamp,
                "avg_launch_us_overlapped": 1e3 * agg_ov[dom][0] / agg_ov[dom][3],
                "flop_per_launch": fl / launches, "bytes_per_launch": by / launches,
                # the same launches against the memory roofline (algorithmic bytes: input + output + residual + weights):
                # many of them are 1x1 layers whose bound is HBM, not the matrix cores
                "algorithmic_gbps": by / (t_ms * 1e-3) / 1e9, "hbm_frac": by / (t_ms * 1e-3) / 1e9 / 8000.0,
                "hbm_frac_of_measured": by / (t_ms * 1e-3) / 1e9 / measured["copy_gbps"] if measured.get("copy_gbps") else None,
                "share_of_conv_time": t_ms / sum(v[0] for v in conv.values()),
                "all_conv_tflops_per_kernel": sum(v[1] for v in conv.values()) / (sum(v[0] for v in conv.values()) * 1e-3) / 1e12,
                "conv_flop_per_step": sum(v[1] for v in conv.values()) / nsamp,
                "conv_tflops_whole_step": sum(v[1] for v in conv.values()) / nsamp / (dt / steps) / 1e12}
    names = ["letterbox", "detector_layers", "decode", "topk", "nms", "compact"]
    for e in range(len(spec.edges)):
        names += ["crop%d" % e, "child%d_layers" % e, "child%d_tail" % e]
    out = {
        "metric": "pipeline frames/s within 200 ms SLO on 1 GPU", "value": tot["met"] / dt, "unit": "frames/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * dt / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": det.dtype, "data": "synthetic",
        "config": {"workload": desc, "batch_frames": n, "slo_ms": spec.slo_ms, "instances": ninst,
                   "heads": "planted" if heads is not None else "natural"},
        "total_frames_per_s": n * steps / dt, "objects_per_s": tot["boxes"] / dt,
        "latency_ms_p50": float(np.percentile(lat, 50)), "latency_ms_p99": float(np.percentile(lat, 99)),
        "stage_ms": {k: round(float(v), 4) for k, v in zip(names, stage)},
        "stage_ms_overlapped": {k: round(float(v), 4) for k, v in zip(names, stage_ov)},
        "roofline": roofline,
        "roofline_hbm": hbm_rooflines(spec, scene, pipes[0], stage, names, n, measured.get("copy_gbps")),
        "conv_kernels": [{"kernel": conv_name(k, det.dtype), "ms_per_step": v[0] / nsamp, "tflops": v[1] / max(v[0], 1e-9) / 1e9,
                          "launches_per_step": v[3] / nsamp} for k, v in sorted(conv.items(), key=lambda kv: -kv[1][0])],
    }
    if args.layers:
        for k, v in sorted(agg.items()):
            nm = conv_name(k, det.dtype) if k >= 1000000000 else {1: "maxpool", 2: "upsample2x", 3: "copy", 4: "add", 5: "gap"}.get(k, str(k))
            print("%-80s %8.3f ms/step  %7.1f TFLOP/s  %7.1f GB/s  %5.1f launches/step  %7.1f us/launch" %
                  (nm, v[0] / nsamp, v[1] / max(v[0], 1e-9) / 1e9, v[2] / max(v[0], 1e-9) / 1e6, v[3] / nsamp, 1e3 * v[0] / max(v[3], 1)), file=sys.stderr)
    if with_cpu:
        out["cpu_baseline"], _ = cpu_baseline(spec, scene, heads, subset=workload == "hires",
                                              rois_per_frame=float(np.mean(items[1:])) / n if len(items) > 1 else 0.0)
        if workload == "tiny":                   # the small configuration is also timed on one thread
            threads = torch.get_num_threads()
            torch.set_num_threads(1)
            out["cpu_baseline_1_thread"], _ = cpu_baseline(spec, scene, heads, min_seconds=5.0)
            torch.set_num_threads(threads)
    torch.cuda.synchronize()
    for P in pipes:
        P.close()
    for st in streams:
        binding.stream_destroy(st)
    del pipes, keep_heads, dev
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed batches (default: 200 for the high-resolution workload, about 7 s; 4000 for "
                    "the traffic one; 400 otherwise)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed batches before them (default: steps / 20)")
    ap.add_argument("--workload", default="hires", help="hires (default: 32 x 3840x2160 frames, the largest configuration), traffic, tiny, placement, "
                    "sweep, colocate, surge")
    ap.add_argument("--instances", type=int, default=None,
                    help="copies of the pipeline (own activations and tables) that take batches in turn, each on its own "
                         "stream, so that kernels of different batches overlap on the GPU (default: 4 for the traffic and "
                         "sweep workloads, 1 for the high-resolution one, whose batches fill the GPU by themselves)")
    ap.add_argument("--det-exec", type=int, default=0, help="frames per execution of the detector's layers (0: the whole batch at once)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-traffic", action="store_true", help="high-resolution workload: do not also run the traffic workload for the extra key")
    ap.add_argument("--traffic-steps", type=int, default=400, help="timed batches of the traffic workload run beside the high-resolution one")
    ap.add_argument("--layers", action="store_true", help="print the per-kernel table to stderr")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device pass over this many MiB before the timed region (a known-size kernel "
                         "against which hardware traffic counters are scaled)")
    ap.add_argument("--duration", type=float, default=5.0, help="co-location workload: seconds of arrivals to serve")
    ap.add_argument("--camera-scale", type=int, default=1, help="co-location workload: multiply the sixteen cameras")
    ap.add_argument("--det-batch", type=int, default=16, help="co-location workload: largest detector batch")
    ap.add_argument("--slo-ms", type=float, default=200.0, help="co-location workload: the pipelines' latency objective")
    ap.add_argument("--edge-cus", type=int, default=8, help="placement simulation: compute units of the stream that stands in for the edge device")
    ap.add_argument("--alpha", type=float, default=1.0, help="placement simulation: how much more network a model's output may cost than its input")
    ap.add_argument("--surge-factor", type=float, default=2.5, help="surge workload: rate multiplier during the middle third")
    args = ap.parse_args()
    if args.instances is None:
        args.instances = 1 if args.workload in ("hires", "tiny") else 4
    if args.steps is None:
        args.steps = {"traffic": 4000, "hires": 200}.get(args.workload, 400)
    if args.warmup is None:
        args.warmup = max(4, args.steps // 20)
    if args.gpus != 1:
        print("bench.py measures one GPU only (frames are independent: more GPUs = more copies of this run); --gpus %d refused" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2502_01277_amd import binding
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    if args.workload == "sweep":
        return run_sweep(args)
    if args.workload == "colocate":
        return run_colocate(args)
    if args.workload == "placement":
        return run_placement(args)
    if args.workload == "surge":
        return run_surge(args)
    if args.workload == "conv8":
        return run_conv8(args)
    # what this machine sustains, measured now: a plain copy and a register-only MFMA loop with random operands
    measured = {"copy_gbps": binding.probe_copy(512, 5), "mfma_tflops": binding.probe_mfma("bf16", 20000, 3),
                "note": "library microbenchmarks run before the timed region: 512 MiB device copy (read + write bytes), register-only "
                        "32x32x16 bf16 MFMA loop with random operand values"}
    out = bench_cascade(args, args.workload, args.steps, args.warmup, max(1, args.instances), measured, not args.no_cpu_baseline)
    out["measured_peaks"] = measured
    if args.workload == "hires" and not args.no_traffic:
        # the traffic cascade (8 x 1080p, fp16, four instances) in the same run, as an extra key
        tsteps = max(20, args.traffic_steps)
        t = bench_cascade(args, "traffic", tsteps, max(8, tsteps // 10), 4, measured, False)
        out["traffic"] = {k: t[k] for k in ("value", "unit", "steps", "ms_per_step", "dtype", "config", "total_frames_per_s", "objects_per_s",
                                            "latency_ms_p50", "latency_ms_p99", "stage_ms", "roofline", "roofline_hbm")}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
