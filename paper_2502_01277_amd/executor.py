"""Co-located serving of several pipelines on one GPU: profiling, scheduler-lite and the slot executor.

The paper shares a GPU between models in space and time (Sec. III-C): every model gets a *portion* - a time slot
inside the duty cycle of an inference stream (length = its batch latency) with a width (the share of compute it
needs) - found by Algorithm 2 after Algorithm 1 has chosen the batch sizes.  Here a stream's width is a real
restriction: a HIP stream created on a contiguous range of compute units.  All decisions come from the library
(`octo_cwd_search`, `octo_coral_schedule`); this module measures the profiles they need, turns the placements into
streams and slot times, and drives `octo_run_model` at the slot starts.

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
import time
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import binding

CU_GRAIN = 8          # stream widths are multiples of 8 compute units (one per die)
MAX_IN_FLIGHT = 6     # uncollected batches per pipeline (the library holds result slots for 7)


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
    """Scheduler-lite: Algorithm 1's batch-size search per pipeline, then Algorithm 2 over all pipelines.

    Widths: every model starts at the width its profile chose; if the pipeline's work per duty cycle (sum over its
    models of batches-per-cycle x batch latency at that width) does not fit in cycle_share of the cycle, all its models
    are moved to the next profiled width and the batch sizes are searched again with the latencies of that width."""
    total = binding.device_cu_count()
    sched_in, all_bz, all_k, est_l, est_t = [], [], [], [], []
    duty = min(s.slo_ms for s in specs) / 2.0
    for i, spec in enumerate(specs):
        parent = {e.child: e.parent for e in spec.edges}
        widths = sorted(set(w for m in profiles[i] for w in m.by_width)) or [total]
        for w_floor in widths:
            models = []
            for mi, m in enumerate(spec.models):
                pr = profiles[i][mi]
                w = max(w_floor, int(round(pr.util * total)))
                lat = pr.by_width.get(w, pr.latency_ms)
                rate = frame_rates[i] * (objects_per_frame[i] if mi > 0 else 1.0)
                wmem = sum(L.weight.size for L in m.layers if getattr(L, "weight", None) is not None) * (4 if m.dtype == "f32" else 2) / 1e6
                models.append(dict(parent=parent.get(mi, -1), profile=dict(lat), rate=max(rate, 1e-3),
                                   burstiness=burstiness[i][mi], util=w / total, weight_mem=wmem, inter_mem=0.0, bz=1))
            bzs = binding.cwd_search(models, spec.slo_ms) if fixed_bz is None else list(fixed_bz[i])
            ks = [binding.batches_per_cycle(m["rate"], duty, b) for m, b in zip(models, bzs)]
            work = sum(k * m["profile"][b] for m, b, k in zip(models, bzs, ks))
            if work <= cycle_share * duty or w_floor == widths[-1]:
                break
        keep: list = []
        for m, b in zip(models, bzs):
            m["bz"] = b
        sp = binding.sched_pipeline(models, spec.slo_ms, keep)
        est_l.append(float(binding.lib().octo_est_latency_ms(binding.C.byref(sp))))
        est_t.append(float(binding.lib().octo_est_throughput(binding.C.byref(sp))))
        for m, b, k in zip(models, bzs, ks):
            m["profile"] = dict(m["profile"])
            m["profile"][b] = k * m["profile"][b]          # the portion holds k back-to-back batches
        sched_in.append((models, spec.slo_ms))
        all_bz.append(bzs)
        all_k.append(ks)
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


@dataclass
class Camera:
    pipeline: int
    arrivals_s: np.ndarray              # arrival times in seconds from the start of serving
    pool: List                          # device uint8 frames this camera cycles through
    pool_offset: int = 0                # where in the pipeline's planted-head pool this camera's frames start


@dataclass
class PipelineStats:
    submitted: int = 0
    served: int = 0
    slo_met: int = 0
    boxes: int = 0
    dropped: int = 0                    # requests dropped at batch formation because they were already late
    latency_ms: List[float] = field(default_factory=list)
    results: Dict[int, Tuple[int, np.ndarray]] = field(default_factory=dict)   # frame id -> (pool index, boxes)


@dataclass
class _Instance:
    """One running copy of a pipeline: the scheduled one, or a stand-by copy the scaler switches on and off."""
    pipe: binding.Pipeline
    logical: int                        # which pipeline's queue it serves
    clone: bool
    override: Optional[List]            # planted mode: the buffers its decode reads
    streams: List[int] = field(default_factory=list)     # per model: stream handle
    slot_ms: float = 0.0                # start of its first model's portion inside the duty cycle
    active: bool = True
    inflight: int = 0
    batch_last: set = field(default_factory=set)


class Executor:
    """Slot executor (Sec. III-C 'Inference Stream'): every duty cycle, at a portion's start, the model is launched on
    what is queued (at most its batch size per batch); downstream models follow their parent on their own streams.

    drop_late: requests already older than the objective when a batch is formed are dropped (Sec. IV-A).
    spares: one stand-by copy per pipeline (or None) for the run-time scaler (Sec. III-D); when a pipeline's arrivals
    outgrow its portion the copy is given portions of its own by Algorithm 2, run over the scheduled pipelines followed
    by the active copies, and it then takes batches from the same queue at its own slot; when the surge is over the copy
    is switched off and its portions are free again.  Only the slotted mode scales: without slots nothing limits how
    many batches a pipeline launches."""

    def __init__(self, pipes: List[binding.Pipeline], schedule: Schedule, cameras: List[Camera],
                 head_pools: Optional[List[Optional[List]]] = None, slotted: bool = True, masked: bool = True,
                 keep_results: bool = False, drop_late: bool = False,
                 spares: Optional[List[Optional[binding.Pipeline]]] = None, scaler: Optional[dict] = None):
        import torch
        self.t = torch
        self.pipes, self.sch, self.cams = pipes, schedule, cameras
        self.slotted, self.masked, self.keep_results, self.drop_late = slotted, masked, keep_results, drop_late
        self.total_cus = binding.device_cu_count()
        self.streams: Dict[int, int] = {}
        self.stream_cus: Dict[int, Tuple[int, int]] = dict(schedule.stream_cus)
        self._owned: List[int] = []
        self._plain = torch.cuda.Stream()
        for st, (first, n) in schedule.stream_cus.items():
            self.streams[st] = self._make_stream(first, n)
        self.head_pools = head_pools or [None] * len(pipes)
        self.inst: List[_Instance] = []
        for i, P in enumerate(pipes):
            I = _Instance(P, i, False, self._make_override(P, i))
            I.streams = [self._stream_of(i, mi) for mi in range(len(P.spec.models))]
            I.slot_ms = schedule.placement(i, 0)[3]
            self.inst.append(I)
        self.spare_of: Dict[int, _Instance] = {}
        if spares is not None and slotted:
            for i, P in enumerate(spares):
                if P is None:
                    continue
                I = _Instance(P, i, True, self._make_override(P, i), list(self.inst[i].streams), self.inst[i].slot_ms, False)
                self.inst.append(I)
                self.spare_of[i] = I
        for I in self.inst:
            I.pipe.set_batch_size(0, min(schedule.bz[I.logical][0], I.pipe.spec.models[0].batch_size))
        self.detectors: Dict[int, SurgeDetector] = {
            i: SurgeDetector((schedule.batches_per_cycle[i][0] + 1) * schedule.bz[i][0], **(scaler or {})) for i in self.spare_of}
        self.scale_events: List[Tuple[float, int, int]] = []      # (seconds since start, pipeline, +1 / -1 / 0 = no room)
        self.stats = [PipelineStats() for _ in pipes]
        self._warmup()

    def _make_stream(self, first: int, n: int) -> int:
        if not self.masked:
            return int(self._plain.cuda_stream)
        h = binding.stream_create_range(first, n)
        self._owned.append(h)
        return h

    def _make_override(self, P: binding.Pipeline, i: int) -> Optional[List]:
        hp = self.head_pools[i]
        if hp is None:
            return None
        bufs = [self.t.empty((P.spec.max_frames,) + tuple(h.shape[1:]), dtype=h.dtype, device=h.device) for h in hp]
        for l, b in enumerate(bufs):
            P.set_head(0, l, b)
        return bufs

    def _gather_heads(self, I: _Instance, idx_dev, stream: int):
        """Planted mode: copy the head tensors of the batch's frames from the pool into the buffers decode reads.
        idx_dev: device int64 tensor of pool indices (prepared ahead, so nothing is copied from the host here)."""
        if I.override is None:
            return
        t = self.t
        with t.cuda.stream(t.cuda.ExternalStream(stream)):
            for l, pool in enumerate(self.head_pools[I.logical]):
                t.index_select(pool, 0, idx_dev, out=I.override[l][:idx_dev.shape[0]])

    def _warmup(self):
        """One frame through every pipeline copy on the streams it will use, so that the first served batch does not
        pay for stream and code-object set-up."""
        for I in self.inst:
            cam = next((c for c in self.cams if c.pipeline == I.logical), None)
            if cam is None:
                continue
            self._gather_heads(I, self.t.tensor([cam.pool_offset], dtype=self.t.int64).cuda(), I.streams[0])
            I.pipe.submit([cam.pool[0]], frame_ids=[-1])
            for mi in range(len(I.pipe.spec.models)):
                I.pipe.run_model(mi, I.streams[mi])
            I.pipe.collect(blocking=True)

    def close(self):
        self.t.cuda.synchronize()
        for h in self._owned:
            binding.stream_destroy(h)
        self._owned = []
        for I in self.inst:
            if I.override is not None:
                for l in range(len(I.override)):
                    I.pipe.set_head(0, l, None)

    def _stream_of(self, pipeline: int, model: int) -> int:
        """Stream of a model's portion; a model Algorithm 2 could not place follows its parent on the parent's stream
        (a root: on the first stream), i.e. it is served best-effort without a slot of its own."""
        st = self.sch.placement(pipeline, model)[2]
        if st >= 0:
            return self.streams[st]
        parent = {e.child: e.parent for e in self.pipes[pipeline].spec.edges}.get(model, -1)
        if parent >= 0:
            return self._stream_of(pipeline, parent)
        return self.streams[min(self.streams)] if self.streams else int(self._plain.cuda_stream)

    # ---- run-time scaling -------------------------------------------------------------------------------------
    def _place_clones(self) -> None:
        """Algorithm 2 over the scheduled pipelines followed by the active copies.  It visits pipelines in order, so
        the scheduled ones get the placements they already have and the copies get what is free.  A copy whose first
        model finds no portion is switched off again; a later model without a portion follows its parent's stream.  A
        stream the schedule did not use yet gets the compute units after the ones in use (the last ones if the GPU is
        full), as wide as the widest model placed on it; streams that exist keep their width."""
        base = self.sch.coral_inputs
        clones = [I for I in self.inst if I.clone and I.active]
        if not clones:
            return
        pl = binding.coral_schedule(list(base) + [base[I.logical] for I in clones], self.sch.gpu_mem_mb, 1.0, self.sch.n_streams)
        for ci, I in enumerate(clones):
            mine = {m: (st, a) for (pi, m, st, a, b, d) in pl if pi == len(base) + ci}
            if mine[0][0] < 0:
                I.active = False
                continue
            models = base[I.logical][0]
            for m, (st, _) in mine.items():
                if st >= 0 and st not in self.streams:
                    n = width_to_cus(max(models[q]["util"] for q, (s2, _) in mine.items() if s2 == st), self.total_cus)
                    first = max([f + c for (f, c) in self.stream_cus.values()] + [0])
                    if first + n > self.total_cus:
                        first = self.total_cus - n
                    self.stream_cus[st] = (first, n)
                    self.streams[st] = self._make_stream(first, n)
            parent = {e.child: e.parent for e in I.pipe.spec.edges}
            handles: List[int] = []
            for m in range(len(models)):
                st = mine[m][0]
                handles.append(self.streams[st] if st >= 0 else handles[parent[m]])
            I.streams, I.slot_ms = handles, mine[0][1]

    def _autoscale(self, now_s: float) -> None:
        """Once per duty cycle: tell every pipeline's detector what arrived and what is queued, and act on its decision."""
        ups, downs = [], []
        for i, det in self.detectors.items():
            self._admit(i, now_s)
            arrived = self.next_arrival[i] - self._arrival_mark[i]
            self._arrival_mark[i] = self.next_arrival[i]
            I = self.spare_of[i]
            d = det.observe(arrived, len(self.mirror[i]), 2 if I.active else 1)
            if d > 0 and not I.active:
                I.active = True
                ups.append(i)
            elif d < 0 and I.active:
                I.active = False
                downs.append(i)
        if ups or downs:
            self._place_clones()             # the copies that stay may move into what a removed one has freed
            self.scale_events += [(now_s, i, -1) for i in downs] + [(now_s, i, 1 if self.spare_of[i].active else 0) for i in ups]

    # ---- serving ----------------------------------------------------------------------------------------------
    def _poll(self):
        for I in self.inst:
            if I.inflight == 0:
                continue
            fr, bx, st = I.pipe.collect(blocking=False)
            if st == binding.ENOTREADY or len(fr) == 0:
                continue
            i = I.logical
            S = self.stats[i]
            S.served += len(fr)
            S.slo_met += int(fr["slo_met"].sum())
            S.boxes += int(fr["n_boxes"].sum())
            S.latency_ms.extend(fr["latency_ms"].tolist())
            batches_done = 0
            for f in fr:
                fid = int(f["frame_id"])
                if fid in I.batch_last:
                    batches_done += 1
                    I.batch_last.discard(fid)
                if self.keep_results:
                    S.results[fid] = (self.pool_of[i].pop(fid), bx[f["box_offset"]: f["box_offset"] + f["n_boxes"]].copy())
            I.inflight -= batches_done

    def _admit(self, i: int, now_s: float):
        """Move frames that have arrived by now from the camera streams into the pipeline's host-side queue."""
        arr, ptr = self.merged[i], self.next_arrival[i]
        while ptr < len(arr) and arr[ptr][0] <= now_s:
            t_s, cam, seq = arr[ptr]
            c = self.cams[cam]
            k = seq % len(c.pool)
            fid = self.next_id[i]
            self.next_id[i] += 1
            self.mirror[i].append((fid, c.pool_offset + k, c.pool[k], self.t0_ms + 1e3 * t_s))
            ptr += 1
        self.stats[i].submitted += ptr - self.next_arrival[i]
        self.next_arrival[i] = ptr

    def _launch_batch(self, I: _Instance) -> int:
        i, P = I.logical, I.pipe
        queue = self.mirror[i]
        if self.drop_late and queue:
            late = late_prefix([q[3] for q in queue], binding.lib().octo_now_ms(), P.spec.slo_ms)
            if late:
                del queue[:late]
                self.stats[i].dropped += late
        n = min(self.sch.bz[i][0], len(queue))
        if n == 0 or I.inflight >= MAX_IN_FLIGHT:
            return 0
        batch = queue[:n]
        del queue[:n]
        if I.override is not None:
            self._gather_heads(I, self.seq_dev[i][batch[0][0]: batch[0][0] + n], I.streams[0])   # ids in a batch are consecutive
        P.submit([b[2] for b in batch], arrival_ms=[b[3] for b in batch], frame_ids=[b[0] for b in batch])
        got = P.run_model(0, I.streams[0])
        assert got == n, (got, n)
        for mi in range(1, len(P.spec.models)):
            P.run_model(mi, I.streams[mi])
        I.inflight += 1
        I.batch_last.add(batch[-1][0])
        if self.keep_results:
            for b in batch:
                self.pool_of[i][b[0]] = b[1]
        return n

    def _fire(self, I: _Instance, now_s: float):
        self._admit(I.logical, now_s)
        for _ in range(self.sch.batches_per_cycle[I.logical][0] + 1):
            spins = 0
            while I.inflight >= MAX_IN_FLIGHT and spins < 100000:    # result slots are full: take finished batches first
                self._poll()
                spins += 1
            if self._launch_batch(I) == 0:
                break

    def _all_done(self) -> bool:
        return all(self.next_arrival[i] == len(self.merged[i]) and not self.mirror[i] for i in range(len(self.pipes))) and \
            all(I.inflight == 0 for I in self.inst)

    def serve(self, duration_s: float, drain_s: float = 2.0) -> dict:
        npipe = len(self.pipes)
        self.merged = [[] for _ in range(npipe)]
        for ci, c in enumerate(self.cams):
            self.merged[c.pipeline] += [(float(t_), ci, k) for k, t_ in enumerate(c.arrivals_s) if t_ < duration_s]
        for m in self.merged:
            m.sort()
        # frame ids are handed out in arrival order, so the pool index of every frame is known now: one upload
        self.seq_dev = []
        for i in range(npipe):
            seq = [self.cams[ci].pool_offset + k % len(self.cams[ci].pool) for (_, ci, k) in self.merged[i]]
            self.seq_dev.append(self.t.tensor(seq if seq else [0], dtype=self.t.int64).cuda())
        self.next_arrival = [0] * npipe
        self._arrival_mark = [0] * npipe
        self.next_id = [0] * npipe
        self.mirror = [[] for _ in range(npipe)]
        self.pool_of = [dict() for _ in range(npipe)]
        now = binding.lib().octo_now_ms
        duty = self.sch.duty_ms
        self.t0_ms = now() + 2.0
        t_end_ms = self.t0_ms + 1e3 * (duration_s + drain_s)
        if self.slotted:
            c = 0
            while True:
                for off, k in sorted((I.slot_ms, k) for k, I in enumerate(self.inst) if I.active):
                    target = self.t0_ms + c * duty + off
                    while now() < target:
                        self._poll()
                        time.sleep(0.0002)
                    self._fire(self.inst[k], (now() - self.t0_ms) / 1e3)
                c += 1
                if self.detectors:
                    while now() < self.t0_ms + c * duty:           # decisions are taken on whole cycles
                        self._poll()
                        time.sleep(0.0002)
                    self._autoscale((now() - self.t0_ms) / 1e3)
                if (self._all_done() and c * duty >= 1e3 * duration_s) or now() > t_end_ms:
                    break
        else:
            while True:
                for I in self.inst:
                    self._admit(I.logical, (now() - self.t0_ms) / 1e3)
                    self._launch_batch(I)
                self._poll()
                time.sleep(0.0002)
                if (self._all_done() and now() - self.t0_ms >= 1e3 * duration_s) or now() > t_end_ms:
                    break
        wall_s = (now() - self.t0_ms) / 1e3
        for _ in range(1000):
            if all(I.inflight == 0 for I in self.inst):
                break
            self._poll()
            time.sleep(0.001)
        per = []
        for i, S in enumerate(self.stats):
            lat = np.asarray(S.latency_ms) if S.latency_ms else np.zeros(1)
            per.append(dict(pipeline=self.pipes[i].spec.name, submitted=S.submitted, served=S.served, slo_met=S.slo_met,
                            dropped=S.dropped, objects=S.boxes, latency_ms_p50=float(np.percentile(lat, 50)),
                            latency_ms_p99=float(np.percentile(lat, 99)), latency_ms_max=float(lat.max())))
        span = max(duration_s, 1e-9)
        return dict(duration_s=duration_s, wall_s=wall_s, per_pipeline=per,
                    effective_frames_per_s=sum(S.slo_met for S in self.stats) / span,
                    total_frames_per_s=sum(S.served for S in self.stats) / span,
                    objects_per_s=sum(S.boxes for S in self.stats) / span,
                    slo_attainment=sum(S.slo_met for S in self.stats) / max(1, sum(S.submitted for S in self.stats)),
                    dropped=sum(S.dropped for S in self.stats),
                    scale_events=[(round(t_, 3), i, d) for (t_, i, d) in self.scale_events])


# ---------------------------------------------------------------------------
# the co-location workload: three pipelines, sixteen cameras
# ---------------------------------------------------------------------------
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
        burst.append([coefficient_of_variation(mine)] + [coefficient_of_variation(child_times)] * (len(spec.models) - 1))
    return Colocation(specs, cams, pools, scenes, heads_host, rates, objs, burst)
