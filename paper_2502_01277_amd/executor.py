"""Co-located serving of several pipelines on one GPU: profiling, scheduler-lite and the slot executor.

The paper shares a GPU between models in space and time (Sec. III-C): every model gets a *portion* - a time slot
inside the duty cycle of an inference stream (length = its batch latency) with a width (the share of compute it
needs) - found by Algorithm 2 after Algorithm 1 has chosen the batch sizes.  Here a stream's width is a real
restriction: a HIP stream created on a contiguous range of compute units.  All decisions come from the library
(`octo_cwd_search`, `octo_coral_schedule`, the run-time rules) and the serving loop itself is the library's
(`octo_executor_*`); this module measures the profiles they need, turns the placements into streams and slot times and
marshals the description of pipelines, instances and cameras.

Two things differ from the paper's runtime and are stated here once:
  * a child model consumes the ROIs of its parent's batch in one launch whose size is taken on the device, so a
    child's batch size from Algorithm 1 sizes its portion (ceil(ROIs per cycle / bz) back-to-back batches) rather
    than splitting the launch;
  * the schedule holds one instance per model: where the arrival rate needs more than one batch per duty cycle, the
    portion is sized for k = ceil(rate * cycle / bz) back-to-back batches instead of k instances.  Further instances
    appear only at run time, from the horizontal scaler (Sec. III-D), which is given stand-by copies of the pipelines.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import binding
from .colocation import Camera, Colocation, make_colocation    # noqa: F401  (the workload that feeds the executor)

CU_GRAIN = 8          # stream widths are multiples of 8 compute units (one per die)


def _pow2_upto(cap: int, limit: int = 8) -> List[int]:
    out, b = [], 1
    while b <= cap and len(out) < limit:
        out.append(b)
        b *= 2
    return out


# Every decision of the serving loop is the library's (include/octo.h, "run-time rules of the serving loop"); this module
# only moves data between the pipelines, the scheduler calls and those rules.
def width_to_cus(util: float, total: int) -> int:
    return binding.width_to_cus(util, total, CU_GRAIN)


coefficient_of_variation = binding.burstiness
late_prefix = binding.late_prefix
SurgeDetector = binding.Scaler


@dataclass
class ModelProfile:
    latency_ms: Dict[int, float]        # batch size -> batch latency at the chosen width
    util: float                         # chosen width as a share of the GPU
    by_width: Dict[int, Dict[int, float]] = field(default_factory=dict)    # compute units -> {batch size -> latency}


def choose_width(by_width: Dict[int, Dict[int, float]], ref_bz: int, total: int, rule: str = "efficient", tol: float = 0.10) -> int:
    """Portion width of a model from its latency at several stream widths (octo_choose_width) at batch size ref_bz."""
    return binding.choose_width({w: by_width[w][ref_bz] for w in by_width}, rule, tol)


def profile_pipeline(P: binding.Pipeline, widths: Sequence[int] = (64, 128, 256), iters: int = 2,
                     det_batches: Optional[Sequence[int]] = None, child_batches: Optional[Sequence[int]] = None,
                     rule: str = "efficient", tol: float = 0.10) -> List[ModelProfile]:
    """Batch-latency profile L_m(bz) of every model (the paper's offline profiling, Sec. III-C), measured by running
    the model's layers on bz items on streams of several widths, and the width chosen from it."""
    import torch
    total = binding.device_cu_count()
    streams = {}
    for w in widths:
        streams[min(w, total)] = binding.stream_create_range(0, min(w, total))
    out = []
    try:
        for mi, m in enumerate(P.spec.models):
            cap = m.batch_size
            grid = list(det_batches if (mi == 0 and det_batches) else child_batches if (mi > 0 and child_batches) else _pow2_upto(cap))
            grid = [b for b in grid if b <= cap]
            by_width = {}
            for w, s in streams.items():
                lat = {}
                for b in grid:
                    P.profile_layers(mi, b, 1, s)                       # warm-up
                    lat[b] = float(P.profile_layers(mi, b, iters, s)[0].sum())
                by_width[w] = lat
            w = choose_width(by_width, grid[-1], total, rule, tol)
            out.append(ModelProfile(dict(by_width[w]), w / total, by_width))
    finally:
        torch.cuda.synchronize()
        for s in streams.values():
            binding.stream_destroy(s)
    return out


@dataclass
class Schedule:
    duty_ms: float
    bz: List[List[int]]                                   # per pipeline, per model
    batches_per_cycle: List[List[int]]                    # per pipeline, per model
    placements: List[Tuple[int, int, int, float, float, float]]   # (pipeline, model, stream, start, end, duty)
    stream_cus: Dict[int, Tuple[int, int]]                # stream -> (first compute unit, count)
    est_latency_ms: List[float]
    est_throughput: List[float]
    coral_inputs: List = field(default_factory=list)      # what Algorithm 2 was given: (models, slo_ms) per pipeline
    gpu_mem_mb: float = 288e3
    n_streams: int = 8

    def placement(self, pipeline: int, model: int):
        for pl in self.placements:
            if pl[0] == pipeline and pl[1] == model:
                return pl
        raise KeyError((pipeline, model))


def plan(specs, profiles: List[List[ModelProfile]], frame_rates: Sequence[float], objects_per_frame: Sequence[float],
         burstiness: Sequence[Sequence[float]], n_streams: int = 8, gpu_mem_mb: float = 288e3,
         fixed_bz: Optional[List[List[int]]] = None, cycle_share: float = 0.5) -> Schedule:
    """Scheduler-lite: per pipeline octo_plan_pipeline (Algorithm 1's batch-size search under load-aware widths), then
    Algorithm 2 over all pipelines, then one contiguous range of compute units per stream that got a portion."""
    total = binding.device_cu_count()
    sched_in, all_bz, all_k, est_l, est_t = [], [], [], [], []
    duty = min(s.slo_ms for s in specs) / 2.0
    for i, spec in enumerate(specs):
        parent = {e.child: e.parent for e in spec.edges}
        widths = sorted(set(w for m in profiles[i] for w in m.by_width)) or [total]
        models = []
        for mi, m in enumerate(spec.models):
            pr = profiles[i][mi]
            wmem = sum(L.weight.size for L in m.layers if getattr(L, "weight", None) is not None) * (4 if m.dtype == "f32" else 2) / 1e6
            models.append(dict(parent=parent.get(mi, -1), rate=frame_rates[i] * (objects_per_frame[i] if mi > 0 else 1.0),
                               burstiness=burstiness[i][mi], weight_mem=wmem, inter_mem=0.0, width=int(round(pr.util * total)),
                               by_width=pr.by_width or {total: pr.latency_ms}))
        out, ks, lat, thr = binding.plan_pipeline(models, spec.slo_ms, duty, cycle_share, widths, total, None if fixed_bz is None else fixed_bz[i])
        sched_in.append((out, spec.slo_ms))
        all_bz.append([m["bz"] for m in out])
        all_k.append(ks)
        est_l.append(lat)
        est_t.append(thr)
    placements = binding.coral_schedule(sched_in, gpu_mem_mb, 1.0, n_streams)
    widest: Dict[int, float] = {}
    for (pi, mi, st, a, b, d) in placements:
        if st >= 0:
            widest[st] = max(widest.get(st, 0.0), sched_in[pi][0][mi]["util"])
    stream_cus, first = {}, 0
    for st in sorted(widest):
        n = width_to_cus(widest[st], total)
        if first + n > total:                               # rounding to the stream granularity overshot the GPU
            first = max(0, total - n)
        stream_cus[st] = (first, n)
        first = min(total - CU_GRAIN, first + n)
    return Schedule(duty, all_bz, all_k, placements, stream_cus, est_l, est_t, sched_in, gpu_mem_mb, n_streams)


PipelineStats, Executor = binding.PipelineStats, binding.SlotExecutor
