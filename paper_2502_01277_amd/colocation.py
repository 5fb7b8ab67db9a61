"""The co-location workload: three pipelines fed by sixteen cameras (and multiples of them), with planted detector heads."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

from . import binding


@dataclass
class Camera:
    pipeline: int
    arrivals_s: np.ndarray              # arrival times in seconds from the start of serving
    pool: List                          # device uint8 frames this camera cycles through
    pool_offset: int = 0                # where in the pipeline's planted-head pool this camera's frames start



@dataclass
class Colocation:
    specs: List
    cameras: List[Camera]
    head_pools: List[Optional[List]]
    scenes: List
    heads_host: List[Optional[List[np.ndarray]]]
    frame_rates: List[float]
    objects_per_frame: List[float]
    burstiness: List[List[float]]


def make_colocation(duration_s: float, n_cameras=(6, 6, 4), pool_frames: int = 8, det_batch: int = 16, dtype: str = "bf16",
                    seed: int = 20250201 + 4, mean_objects: float = 8.0, base_fps: float = 15.0,
                    src_hw=(1080, 1920), slo_ms: float = 200.0, surge: Optional[Tuple[int, float, float, float]] = None) -> Colocation:
    """Traffic cascade, surveillance cascade and a detector-only pipeline fed by cameras whose frame rate swings
    sinusoidally around 15 fps (inhomogeneous Poisson arrivals); frames cycle through a small pool per pipeline and
    the detector heads are planted per pool frame with Poisson object counts.

    surge = (pipeline, t0, t1, factor): the cameras of that pipeline send factor x as many frames for t0 <= t < t1;
    the rates and burstiness handed to the scheduler are then those of the time before t0 (the scheduler ran before
    the surge and could not know of it)."""
    import torch
    from . import synth, zoo
    rng = np.random.default_rng(seed)
    specs = [zoo.traffic_cascade(dtype=dtype, det_batch=det_batch), zoo.surveillance_cascade(dtype=dtype, det_batch=det_batch),
             zoo.detector_only(dtype=dtype, det_batch=det_batch)]
    for sp in specs:
        sp.slo_ms = slo_ms
    h, w = src_hw
    boost = None
    if surge is not None:
        owner = [i for i, n in enumerate(n_cameras) for _ in range(n)]
        boost = [tuple(surge[1:]) if owner[c] == surge[0] else None for c in range(sum(n_cameras))]
    arrivals = synth.sinusoid_arrivals(rng, sum(n_cameras), duration_s, base_fps=base_fps, boost=boost)
    cams, pools, scenes, heads_host = [], [], [], []
    ci = 0
    for i, spec in enumerate(specs):
        counts = synth.counts_poisson(rng, pool_frames, mean=mean_objects, cap=spec.max_rois_per_frame)
        scene = synth.make_scene(rng, pool_frames, h, w, counts, 24, 360, log_uniform=True)
        scenes.append(scene)
        dev = [torch.from_numpy(f).cuda() for f in scene.frames]
        hh = synth.planted_heads(rng, spec.models[0], scene, h, w, binding.letterbox_geometry(h, w, spec.models[0].in_h, spec.models[0].in_w))
        heads_host.append(hh)
        pools.append([binding.to_device(x, spec.models[0].dtype) for x in hh])
        for _ in range(n_cameras[i]):
            cams.append(Camera(i, arrivals[ci], dev, 0))
            ci += 1
    rates, objs, burst = [], [], []
    for i, spec in enumerate(specs):
        mine = np.sort(np.concatenate([c.arrivals_s for c in cams if c.pipeline == i])) if n_cameras[i] else np.zeros(0)
        span = duration_s
        if surge is not None and surge[0] == i and surge[1] > 0:
            mine, span = mine[mine < surge[1]], surge[1]
        rates.append(len(mine) / max(span, 1e-9))
        per_frame = np.array([len(r) for r in scenes[i].rects], np.float64)
        objs.append(float(per_frame.mean()))
        # objects of one frame reach the child together, so its inter-arrival times are mostly zero: a much
        # burstier sequence than the frames themselves
        k = rng.choice(per_frame.astype(np.int64), size=len(mine)) if len(mine) else np.zeros(0, np.int64)
        child_times = np.repeat(mine, k)
        burst.append([binding.burstiness(mine)] + [binding.burstiness(child_times)] * (len(spec.models) - 1))
    return Colocation(specs, cams, pools, scenes, heads_host, rates, objs, burst)
