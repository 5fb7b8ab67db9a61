"""Oracle: batch-size search and spatiotemporal portion scheduling (test infrastructure).

`cwd_lite` is the batch-size part of the paper's Algorithm 1 with device and GPU
fixed to the one GPU and one instance per model; `coral` is Algorithm 2.  Both
take the algorithm's steps in the paper's order.  Readings taken where the
listing is silent or garbled are marked READING.

parity unpinned (against the paper): neither algorithm has a printed worked
example; the tests pin them by invariants, exhaustive search on small cases and
a hand-computed schedule.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

INF = math.inf


@dataclass
class SModel:
    name: str
    parent: int                       # index of the upstream model in the pipeline, -1 for the root
    profile: Dict[int, float]         # batch size -> batch latency L_{m|bz} in ms (Sec. II)
    rate: float = 15.0                # requests per second reaching this model
    burstiness: float = 0.0           # coefficient of variation of inter-arrival times (Sec. III-B)
    util: float = 0.25                # U_m: share of the GPU's compute the model needs (portion width)
    weight_mem: float = 0.0           # W_m
    inter_mem: float = 0.0            # I_m
    bz: int = 1


@dataclass
class SPipeline:
    name: str
    models: List[SModel]              # topological order, root first
    slo_ms: float


def est_latency(p: SPipeline) -> float:
    """READING (EstLat is not defined in the paper): worst case of the first request of a batch (Sec. II,
    constraint a) along the longest root-to-leaf path: sum of batch latency plus the wait for bz-1 further
    requests at the model's arrival rate."""
    def path_cost(i):
        m = p.models[i]
        own = m.profile[m.bz] + (m.bz - 1) * 1000.0 / m.rate
        return own + (path_cost(m.parent) if m.parent >= 0 else 0.0)
    leaves = [i for i in range(len(p.models)) if all(c.parent != i for c in p.models)]
    return max(path_cost(i) for i in leaves)


def est_throughput(p: SPipeline) -> float:
    """Eq. (2) for one pipeline with the same-device IO term dropped: 1 / sum_m (L_{m|bz} / bz); per second."""
    return 1000.0 / sum(m.profile[m.bz] / m.bz for m in p.models)


def cwd_lite(p: SPipeline) -> List[int]:
    """Algorithm 1, batch-size part.  Start from bz = 1 everywhere; visit models from the burstiest down;
    double a model's batch; drop the trial if the estimated latency exceeds SLO/2, adopt it if the estimated
    throughput beats the best so far; repeat sweeps until one adopts nothing.

    READING: a trial that is feasible but no better is reverted too, so the running state always equals the
    adopted configuration; a batch size with no profile entry is infeasible; 'max' starts at the throughput of
    the all-ones configuration; ties in burstiness keep pipeline order.
    """
    for m in p.models:
        m.bz = 1
    best = est_throughput(p)
    order = sorted(range(len(p.models)), key=lambda i: -p.models[i].burstiness)
    while True:
        adopted = False
        for i in order:
            m = p.models[i]
            m.bz *= 2
            if m.bz not in m.profile or est_latency(p) > p.slo_ms / 2:
                m.bz //= 2
                continue
            thr = est_throughput(p)
            if thr > best:
                best = thr
                adopted = True
            else:
                m.bz //= 2
        if not adopted:
            break
    return [m.bz for m in p.models]


# ---------------------------------------------------------------------------
# CORAL
# ---------------------------------------------------------------------------
@dataclass
class Portion:
    stream: int
    start: float
    end: float


@dataclass
class Stream:
    duty_cycle: float = 0.0      # 0 = not set yet
    inter_mem: float = 0.0       # I_s: largest intermediate memory of the models on the stream (shared)
    max_util: float = 0.0        # widest portion on the stream


@dataclass
class Placement:
    pipeline: int
    model: int
    stream: int                  # -1: not found
    start: float = 0.0
    end: float = 0.0
    duty_cycle: float = 0.0


@dataclass
class Gpu:
    mem: float
    util_max: float = 1.0
    n_streams: int = 8
    W: float = 0.0
    I: float = 0.0
    U: float = 0.0
    streams: List[Stream] = field(default_factory=list)
    free: List[Portion] = field(default_factory=list)


def _portion_key(pt: Portion):
    # READING ("best fit", "minimal empty space"): free portions are kept ordered by length, then start,
    # then stream, so the first acceptable portion is the tightest one.
    return (pt.end - pt.start, pt.start, pt.stream)


def model_window(p: SPipeline, i: int):
    """Start = sum of the portion lengths of the model's ancestors (downstream runs right after upstream,
    Sec. III-C 'Inference Stream'); end = start + L_{m|bz}."""
    m = p.models[i]
    start = 0.0
    a = m.parent
    while a >= 0:
        start += p.models[a].profile[p.models[a].bz]
        a = p.models[a].parent
    return start, start + m.profile[m.bz]


def coral_place(g: Gpu, p: SPipeline, pi: int, mi: int) -> Placement:
    """Function CORAL(m, instanceNumber) of Algorithm 2 for a single-instance model."""
    m = p.models[mi]
    m_start, m_end = model_window(p, mi)
    duty_r = p.slo_ms / 2.0                                   # a stream's duty cycle is half the SLO (Sec. III-C)
    for pt in list(g.free):
        s = g.streams[pt.stream]
        w_g = g.W + m.weight_mem
        i_g = g.I - s.inter_mem + max(s.inter_mem, m.inter_mem)
        # READING (indices in the listing are garbled): every stream reserves the width of its widest portion.
        u_g = sum(t.max_util for k, t in enumerate(g.streams) if k != pt.stream) + max(s.max_util, m.util)
        duty_s = s.duty_cycle
        # READING: on a stream with no duty cycle yet the portion must also end inside the cycle it would set.
        fits_cycle = m_end <= (duty_s if duty_s > 0 else duty_r)
        if (pt.start <= m_start and pt.end >= m_end and fits_cycle
                and w_g + i_g <= g.mem and u_g <= g.util_max + 1e-12
                and duty_r >= duty_s):
            if duty_s == 0:
                s.duty_cycle = duty_r
                # READING (DividePortion / open-ended portions): once the cycle is known, the stream's
                # open-ended free portion is cut at the cycle's end.
                for q in g.free:
                    if q.stream == pt.stream and q.end == INF:
                        q.end = duty_r
            g.W, g.I, g.U = w_g, i_g, u_g
            s.inter_mem = max(s.inter_mem, m.inter_mem)
            s.max_util = max(s.max_util, m.util)
            g.free.remove(pt)
            for a, b in ((pt.start, m_start), (m_end, pt.end)):    # leftovers; zero-length ones are discarded
                if b > a:
                    g.free.append(Portion(pt.stream, a, b))
            g.free.sort(key=_portion_key)
            return Placement(pi, mi, pt.stream, m_start, m_end, s.duty_cycle)
    return Placement(pi, mi, -1)


def coral(pipelines: List[SPipeline], mem: float, util_max: float = 1.0, n_streams: int = 8):
    """Function Main of Algorithm 2: instance number 0, 1, ... ; per round one instance of every model of every
    pipeline (fairness).  Here every model has exactly one instance, so there is one round."""
    g = Gpu(mem=mem, util_max=util_max, n_streams=n_streams)
    g.streams = [Stream() for _ in range(n_streams)]
    g.free = [Portion(s, 0.0, INF) for s in range(n_streams)]
    g.free.sort(key=_portion_key)
    out = []
    for pi, p in enumerate(pipelines):
        for mi in range(len(p.models)):
            out.append(coral_place(g, p, pi, mi))
    return out, g
