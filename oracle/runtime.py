"""Oracle: the run-time rules of the serving loop (test infrastructure).

Plain, slow reference implementations of the small decisions an executor takes around the scheduler's output: the
burstiness of an arrival sequence (Sec. III-B), how many back-to-back batches a model's portion must hold (Sec. III-C:
a portion's length is the model's batch latency), which compute units a portion's width maps to, which width a
model takes given its latency at several widths, lazy dropping of late requests (Sec. IV-A) and the horizontal
scaling decision between two runs of the scheduler (Sec. III-D).

parity unpinned (against the paper): the paper gives none of these as a formula or a worked example - burstiness is
named as "the coefficient of variation of inter-request arrival times", lazy dropping in one sentence, the scaler in
one paragraph without a rule.  Each function states its reading; the tests pin them by hand-computed cases.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence


def burstiness(times: Sequence[float]) -> float:
    """Coefficient of variation (population standard deviation / mean) of the gaps between consecutive arrival times,
    taken in ascending order.  Fewer than three arrivals (fewer than two gaps), or a zero mean gap, give 0."""
    t = sorted(float(x) for x in times)
    if len(t) < 3:
        return 0.0
    gaps = [t[i + 1] - t[i] for i in range(len(t) - 1)]
    mean = sum(gaps) / len(gaps)
    if mean <= 0.0:
        return 0.0
    var = sum((g - mean) ** 2 for g in gaps) / len(gaps)
    return math.sqrt(var) / mean


def batches_per_cycle(rate_per_s: float, duty_ms: float, bz: int) -> int:
    """READING: with one instance per model, the requests of one duty cycle (rate x cycle) need ceil(that / bz) batches,
    at least one; the model's portion is that many batch latencies long."""
    need = rate_per_s * duty_ms / 1000.0 / bz
    return max(1, int(math.ceil(need - 1e-9)))


def width_to_cus(util: float, total: int, grain: int = 8) -> int:
    """READING: a portion's width (share of the GPU's compute, 0..1) is rounded up to whole multiples of `grain`
    compute units (one per die), at least one grain and at most the GPU."""
    n = int(math.ceil(util * total / grain - 1e-9)) * grain
    return max(grain, min(total, n))


def choose_width(latency_by_width: Dict[int, float], rule: str = "efficient", tol: float = 0.10) -> int:
    """READING: a model's width from its batch latency on streams of several widths (compute units -> ms).
    'latency': the narrowest width whose latency is within tol of the widest width's.  'efficient': the narrowest width
    whose cost width x latency is within tol of the cheapest cost."""
    ws = sorted(latency_by_width)
    if rule == "latency":
        full = latency_by_width[ws[-1]]
        for w in ws:
            if latency_by_width[w] <= (1.0 + tol) * full:
                return w
    best = min(w * latency_by_width[w] for w in ws)
    for w in ws:
        if w * latency_by_width[w] <= (1.0 + tol) * best:
            return w
    return ws[-1]


def late_prefix(arrival_ms: Sequence[float], now_ms: float, slo_ms: float) -> int:
    """Lazy dropping (Sec. IV-A): the number of requests at the head of an arrival-ordered queue that are already older
    than the latency objective when a batch is formed.  A request exactly one objective old is still served; counting
    stops at the first request that is not late (nothing is taken out of the middle of the queue)."""
    n = 0
    for a in arrival_ms:
        if now_ms - a <= slo_ms:
            break
        n += 1
    return n


class Scaler:
    """READING of the horizontal scaler (Sec. III-D): once per duty cycle it sees how many requests arrived and how many
    are queued.  One instance serves `capacity` requests per cycle.  Over the last `window` cycles: add an instance if
    fewer than `max_instances` run and (mean arrivals > up x capacity of the running instances, or the queue never fell
    to that capacity or below); otherwise remove one if more than one runs, mean arrivals < down x capacity of one instance
    fewer, and the current queue fits that capacity.  A decision empties the window; before the window is full nothing
    is decided."""

    def __init__(self, capacity: float, window: int = 5, up: float = 1.0, down: float = 0.75, max_instances: int = 2):
        self.capacity, self.window, self.up, self.down, self.max_instances = float(capacity), int(window), float(up), float(down), int(max_instances)
        self.arrived: List[int] = []
        self.backlog: List[int] = []

    def observe(self, arrived: int, backlog: int, n_active: int) -> int:
        self.arrived.append(int(arrived))
        self.backlog.append(int(backlog))
        if len(self.arrived) < self.window:
            return 0
        self.arrived = self.arrived[-self.window:]
        self.backlog = self.backlog[-self.window:]
        mean = sum(self.arrived) / self.window
        have = self.capacity * n_active
        if n_active < self.max_instances and (mean > self.up * have or min(self.backlog) > have):
            self.arrived, self.backlog = [], []
            return 1
        less = self.capacity * (n_active - 1)
        if n_active > 1 and mean < self.down * less and self.backlog[-1] <= less:
            self.arrived, self.backlog = [], []
            return -1
        return 0


def plan_pipeline(models: List[dict], slo_ms: float, duty_ms: float, cycle_share: float, widths: Sequence[int], total_cus: int,
                  fixed_bz: Sequence[int] = None):
    """Load-aware widths around Algorithm 1's batch-size search (READING: the paper takes a model's measured utilisation
    as its width U_m and does not say what happens when a pipeline's work does not fit its duty cycle at those widths).

    models: dicts with parent, rate, burstiness, weight_mem, inter_mem, width (the compute units the model's own profile
    chose) and by_width {compute units: {batch size: latency ms}}.  For every profiled width taken as a floor, in
    ascending order: each model runs at max(floor, its own width); Algorithm 1 picks the batch sizes with the latencies
    of those widths (or fixed_bz is taken); a model needs k = batches_per_cycle batches per cycle; the floor is accepted
    if the pipeline's work per duty cycle, sum k x L(bz), is at most cycle_share x duty, and the widest floor is accepted
    whatever its work.  Returns (models as oracle.sched.SModel with bz set and the batch latency at bz multiplied by k -
    the portion holds k back-to-back batches -, k per model, estimated latency, estimated throughput); the two
    estimates are taken before the multiplication."""
    from . import sched
    ws = sorted(widths)
    for floor in ws:
        sm = []
        for i, m in enumerate(models):
            w = max(floor, m["width"])
            sm.append(sched.SModel("m%d" % i, m["parent"], dict(m["by_width"][w]), max(m["rate"], 1e-3), m["burstiness"], w / total_cus,
                                   m["weight_mem"], m["inter_mem"], 1))
        p = sched.SPipeline("p", sm, slo_ms)
        bzs = sched.cwd_lite(p) if fixed_bz is None else list(fixed_bz)
        for m, b in zip(sm, bzs):
            m.bz = b
        ks = [batches_per_cycle(m.rate, duty_ms, m.bz) for m in sm]
        work = sum(k * m.profile[m.bz] for m, k in zip(sm, ks))
        if work <= cycle_share * duty_ms or floor == ws[-1]:
            break
    lat, thr = sched.est_latency(p), sched.est_throughput(p)
    for m, k in zip(sm, ks):
        m.profile[m.bz] = k * m.profile[m.bz]
    return sm, ks, lat, thr
