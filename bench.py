#!/usr/bin/env python3
"""Benchmark of the cascade hot path on one MI355X.

A step is one pass of the whole path (letterbox, detector, decode, top-k, NMS, ROI compaction, crop-resize,
classifier and plate detector, result copy) over one batch of the traffic workload: 8 synthetic 1920x1080 frames
from 4 cameras, fp16, planted detector heads (Poisson(8) objects per frame).  Prints one JSON line.
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
    from paper_2502_01277_amd import synth, zoo
    if name == "traffic":
        spec = zoo.traffic_cascade()
        rng = np.random.default_rng(zoo.SEED0 + 2)
        counts = synth.counts_poisson(rng, 8, 8.0, 64)
        scene = synth.make_scene(rng, 8, 1080, 1920, counts, 24, 360, log_uniform=True)
        heads = synth.planted_heads(rng, spec.models[0], scene, 1080, 1920)
        desc = "traffic cascade: 8x1920x1080 u8 frames (4 cameras x 2), CSP-s detector 640 fp16, planted heads Poisson(8), " \
               "ResNet-18-shaped classifier 224 + 6-layer plate detector 128 on every ROI"
    elif name == "hires":
        spec = zoo.hires_cascade()
        rng = np.random.default_rng(zoo.SEED0 + 5)
        counts = synth.counts_pareto(rng, 32)
        scene = synth.make_scene(rng, 32, 2160, 3840, counts, 48, 720, log_uniform=True)
        heads = synth.planted_heads(rng, spec.models[0], scene, 2160, 3840, n_clutter=1100)
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
    bc, bp, kv, minb, vec = d // 1000000, (d // 1000) % 1000, (d // 100) % 10, (d // 10) % 10, d % 10
    wc, wp = (1, 4) if bc == 32 else (2, 2)
    ctype = {"f16": "_Float16", "bf16": "__bf16", "f32": "float"}[dtype]
    return "octo::conv_mfma_kernel<%s, %d, %d, %d, %d, %d, 2, %d, %s>" % (ctype, bc, bp, wc, wp, kv, minb, "true" if vec else "false")


def cpu_baseline(spec, scene, heads):
    """The oracle, as it stands, on the same batch (bounded to about 10-30 s of CPU work)."""
    import torch
    from oracle import cascade
    n = scene.frames.shape[0]
    t0 = time.time()
    ref = cascade.run_cascade(spec, scene.frames, planted_heads=heads)
    dt = time.time() - t0
    return {"value": n / dt, "unit": "frames/s", "cores": int(torch.get_num_threads()), "kind": "oracle",
            "sample": "one full batch of %d frames through the whole cascade (%d ROIs per child), %.1f s" %
                      (n, len(ref.children[0].rois) if ref.children else 0, dt)}, ref


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="traffic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", action="store_true", help="print the per-layer table to stderr")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the timed region (a known-size kernel "
                         "against which hardware traffic counters are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only (frames are independent: more GPUs = more copies of this run); --gpus %d refused" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2502_01277_amd import binding
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    spec, scene, heads, desc = make_workload(args.workload)
    det = spec.models[0]
    n = scene.frames.shape[0]
    P = binding.Pipeline(spec)
    d_heads = None
    if heads is not None:
        d_heads = [binding.to_device(h, det.dtype) for h in heads]
        for l, h in enumerate(d_heads):
            P.set_head(0, l, h)
    dev = [torch.from_numpy(f).cuda() for f in scene.frames]
    stream = torch.cuda.Stream()
    now = binding.lib().octo_now_ms

    def step_submit():
        P.submit(dev, arrival_ms=[now()] * n)
        P.run(stream)

    for _ in range(args.warmup):
        step_submit()
        P.collect()
    if args.calib_copy_mib:
        src = torch.full((args.calib_copy_mib << 18,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)           # one elementwise kernel: reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    # ---- timed region: K steps, two batches in flight, inputs resident in HBM ----
    lat, met, total_boxes = [], 0, 0
    submitted = collected = 0

    def drain(max_in_flight):
        nonlocal collected, met, total_boxes
        while submitted - collected > max_in_flight * n:
            fr, bx, st = P.collect()            # blocking: returns at least the oldest batch
            collected += len(fr)
            lat.extend(fr["latency_ms"].tolist())
            met += int(fr["slo_met"].sum())
            total_boxes += int(fr["n_boxes"].sum())

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_submit()
        submitted += n
        drain(1)                                # one batch stays in flight while the next is prepared
    drain(0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # ---- same region again with an event between layers: per-kernel durations ----
    P.set_layer_timing(True)
    P.set_stage_timing(True)
    agg = {}      # kernel id -> [time ms, flops, bytes, launches]
    stage = []
    ksteps = min(args.steps, 50)
    items = [n] + [0] * (len(spec.models) - 1)          # items each model processes per step (same batch every step)
    for e, edge in enumerate(spec.edges):
        items[edge.child] = len(P.get_rois(e))
    for i in range(ksteps):
        step_submit()
        P.collect()
        stage.append(P.stage_ms())
        for mi, m in enumerate(spec.models):
            ms, kid, fl, by, wb = P.layer_info(mi)
            for j in range(len(ms)):
                if kid[j] == 0:
                    continue
                a = agg.setdefault(int(kid[j]), [0.0, 0.0, 0.0, 0])
                a[0] += float(ms[j]); a[1] += fl[j] * items[mi]; a[2] += by[j] * items[mi] + wb[j]; a[3] += 1
    P.set_layer_timing(False)
    P.set_stage_timing(False)
    stage = np.mean(np.stack(stage), axis=0)
    conv = {k: v for k, v in agg.items() if k >= 1000000000}
    dom = max(conv, key=lambda k: conv[k][0])
    t_ms, fl, by, launches = conv[dom]
    kname = conv_name(dom, det.dtype)
    roofline = {"bound": "mfma", "kernel": kname, "achieved": fl / (t_ms * 1e-3) / 1e12, "peak": PEAK[det.dtype], "unit": "TFLOP/s",
                "frac": fl / (t_ms * 1e-3) / 1e12 / PEAK[det.dtype], "traffic": None,
                "avg_launch_us": 1e3 * t_ms / launches, "launches_per_step": launches / ksteps,
                "all_conv_tflops": sum(v[1] for v in conv.values()) / (sum(v[0] for v in conv.values()) * 1e-3) / 1e12,
                "conv_ms_per_step": sum(v[0] for v in conv.values()) / ksteps}
    names = ["letterbox", "detector_layers", "decode", "topk", "nms", "compact"]
    for e in range(len(spec.edges)):
        names += ["crop%d" % e, "child%d_layers" % e, "child%d_tail" % e]
    out = {
        "metric": "pipeline frames/s within 200 ms SLO on 1 GPU", "value": met / dt, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": det.dtype, "data": "synthetic",
        "config": {"workload": desc, "batch_frames": n, "slo_ms": spec.slo_ms, "batches_in_flight": 2,
                   "heads": "planted" if heads is not None else "natural"},
        "total_frames_per_s": n * args.steps / dt, "objects_per_s": total_boxes / dt,
        "latency_ms_p50": float(np.percentile(lat, 50)), "latency_ms_p99": float(np.percentile(lat, 99)),
        "stage_ms": {k: round(float(v), 4) for k, v in zip(names, stage)},
        "roofline": roofline,
    }
    if args.layers:
        for k, v in sorted(agg.items()):
            nm = conv_name(k, det.dtype) if k >= 1000000000 else {1: "maxpool", 2: "upsample2x", 3: "copy", 4: "add", 5: "gap"}.get(k, str(k))
            print("%-80s %8.3f ms/step  %7.1f TFLOP/s  %7.1f GB/s  %5.1f launches/step  %7.1f us/launch" %
                  (nm, v[0] / ksteps, v[1] / max(v[0], 1e-9) / 1e9, v[2] / max(v[0], 1e-9) / 1e6, v[3] / ksteps, 1e3 * v[0] / max(v[3], 1)), file=sys.stderr)
    if not args.no_cpu_baseline:
        out["cpu_baseline"], _ = cpu_baseline(spec, scene, heads)
    P.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
