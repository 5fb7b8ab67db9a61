"""Pins for the oracle's batch-size search (Algorithm 1, batch part) and portion scheduler (Algorithm 2).

parity unpinned against the paper (it prints no worked example): pinned by invariants, exhaustive search on
small cases and a schedule computed by hand below.
"""
import itertools
import math

import numpy as np

from oracle import sched


def _profile(base, slope, bzs=(1, 2, 4, 8, 16, 32, 64)):
    return {b: base + slope * b for b in bzs}


def _pipe(rng, n_models, slo=200.0):
    ms = []
    for i in range(n_models):
        ms.append(sched.SModel("m%d" % i, parent=-1 if i == 0 else int(rng.integers(0, i)),
                               profile=_profile(rng.uniform(1, 6), rng.uniform(0.2, 2.0)),
                               rate=float(rng.uniform(15, 400)), burstiness=float(rng.uniform(0, 3))))
    return sched.SPipeline("p", ms, slo)


def test_estimators_closed_form():
    a = sched.SModel("a", -1, {1: 10.0, 2: 14.0}, rate=100.0)
    b = sched.SModel("b", 0, {1: 5.0, 4: 8.0}, rate=50.0)
    c = sched.SModel("c", 0, {1: 1.0}, rate=10.0)
    p = sched.SPipeline("p", [a, b, c], 200.0)
    a.bz, b.bz, c.bz = 2, 4, 1
    # path a->b: (14 + 1*10ms) + (8 + 3*20ms) = 92 ; path a->c: 24 + 1 = 25
    assert math.isclose(sched.est_latency(p), 92.0)
    assert math.isclose(sched.est_throughput(p), 1000.0 / (14 / 2 + 8 / 4 + 1 / 1))


def test_cwd_hand_case_burstiest_first():
    # two models; doubling either is feasible once, but not both (SLO/2 = 20 ms).
    a = sched.SModel("a", -1, {1: 4.0, 2: 5.0, 4: 30.0}, rate=1000.0, burstiness=0.1)
    b = sched.SModel("b", 0, {1: 4.0, 2: 5.0, 4: 30.0}, rate=1000.0, burstiness=2.0)
    p = sched.SPipeline("p", [a, b], 40.0)
    # sweep 1: b first: (4)+(5+1)=10 ok, thr 1000/(4+2.5) > 1000/8 adopt; a: (5+1)+(6)=12 ok, thr 1000/5 adopt
    # sweep 2: b->4: lat 6 + 30+3 > 20 drop; a->4 likewise drop; stop.
    assert sched.cwd_lite(p) == [2, 2]
    a.profile = {1: 4.0, 2: 17.0}; b.profile = {1: 4.0, 2: 7.0}
    # b->2: 4 + (7+1) = 12 ok, thr 1000/7.5 > 125 adopt; a->2: (17+1) + 8 > 20 drop -> only the bursty model grows
    assert sched.cwd_lite(p) == [1, 2]


def test_cwd_invariants_on_random_profiles():
    rng = np.random.default_rng(0)
    for _ in range(60):
        p = _pipe(rng, int(rng.integers(1, 5)), slo=float(rng.choice([100, 200, 300])))
        bz = sched.cwd_lite(p)
        assert all(b in (1, 2, 4, 8, 16, 32, 64) for b in bz)
        ones = sched.SPipeline("q", [sched.SModel(m.name, m.parent, m.profile, m.rate) for m in p.models], p.slo_ms)
        if any(b > 1 for b in bz):
            assert sched.est_latency(p) <= p.slo_ms / 2
        assert sched.est_throughput(p) >= sched.est_throughput(ones)
        assert sched.cwd_lite(p) == bz                                  # deterministic / idempotent
        # local optimality of the stopping rule: no single doubling is feasible and better
        best = sched.est_throughput(p)
        for m in p.models:
            m.bz *= 2
            if m.bz in m.profile and sched.est_latency(p) <= p.slo_ms / 2:
                assert sched.est_throughput(p) <= best
            m.bz //= 2


def test_cwd_against_exhaustive_search_small():
    rng = np.random.default_rng(1)
    for _ in range(20):
        p = _pipe(rng, 3)
        bz = sched.cwd_lite(p)
        got = sched.est_throughput(p)
        feas = []
        for combo in itertools.product((1, 2, 4, 8, 16, 32, 64), repeat=3):
            for m, b in zip(p.models, combo):
                m.bz = b
            if sched.est_latency(p) <= p.slo_ms / 2:
                feas.append(sched.est_throughput(p))
        for m, b in zip(p.models, bz):
            m.bz = b
        assert feas and got <= max(feas) + 1e-9            # greedy never beats the optimum and is feasible


def _validate(pipes, placed, g, mem, util_max):
    by_stream = {}
    for pl in placed:
        if pl.stream < 0:
            continue
        p = pipes[pl.pipeline]; m = p.models[pl.model]
        s, e = sched.model_window(p, pl.model)
        assert (pl.start, pl.end) == (s, e) and pl.duty_cycle <= p.slo_ms / 2 and e <= pl.duty_cycle
        if m.parent >= 0:
            par = [q for q in placed if q.pipeline == pl.pipeline and q.model == m.parent][0]
            if par.stream >= 0:
                assert pl.start >= par.end                 # downstream never before upstream
        by_stream.setdefault(pl.stream, []).append((s, e, m))
    for s, items in by_stream.items():
        items.sort(key=lambda t: t[0])
        for (s0, e0, _), (s1, e1, _) in zip(items, items[1:]):
            assert e0 <= s1                                 # no overlap inside a stream
    util = sum(max(m.util for _, _, m in items) for items in by_stream.values())
    assert util <= util_max + 1e-9 and math.isclose(util, g.U, abs_tol=1e-9)
    w = sum(m.weight_mem for items in by_stream.values() for _, _, m in items)
    i = sum(max(m.inter_mem for _, _, m in items) for items in by_stream.values())
    assert math.isclose(w, g.W) and math.isclose(i, g.I) and w + i <= mem


def test_coral_hand_computed_schedule():
    A = sched.SModel("A", -1, {1: 30.0}, util=0.5, weight_mem=10, inter_mem=4)
    B = sched.SModel("B", 0, {1: 20.0}, util=0.3, weight_mem=5, inter_mem=6)
    C = sched.SModel("C", -1, {1: 40.0}, util=0.5, weight_mem=7, inter_mem=3)
    D = sched.SModel("D", -1, {1: 45.0}, util=0.2, weight_mem=1, inter_mem=1)
    E = sched.SModel("E", -1, {1: 40.0}, util=0.2, weight_mem=1, inter_mem=1)
    F = sched.SModel("F", 0, {1: 10.0}, util=0.5, weight_mem=1, inter_mem=1)
    p0 = sched.SPipeline("p0", [A, B], 200.0)       # duty 100
    p1 = sched.SPipeline("p1", [C], 300.0)          # duty 150
    p2 = sched.SPipeline("p2", [D], 250.0)          # duty 125
    p3 = sched.SPipeline("p3", [E, F], 400.0)       # duty 200
    placed, g = sched.coral([p0, p1, p2, p3], mem=100.0, util_max=1.0, n_streams=2)
    got = [(q.stream, q.start, q.end, q.duty_cycle) for q in placed]
    # A: stream 0 [0,30), sets duty 100, free s0:[30,100).  B: window [30,50) fits s0 tightly.
    # C: s0:[50,100) does not contain [0,40); s1 open: u = 0.5 + 0.5 = 1.0 ok -> s1 [0,40), duty 150, free s1:[40,150).
    # D: window [0,45): no free portion starts at 0 -> not found.
    # E: window [0,40): none starts at 0 -> not found.  F (child of E): window [40,50):
    #    s0:[50,100) no; s1:[40,150) contains it, duty 200 >= 150, u = 0.5 + max(0.5,0.5) = 1.0 -> s1 [40,50).
    assert got == [(0, 0.0, 30.0, 100.0), (0, 30.0, 50.0, 100.0), (1, 0.0, 40.0, 150.0),
                   (-1, 0.0, 0.0, 0.0), (-1, 0.0, 0.0, 0.0), (1, 40.0, 50.0, 150.0)]
    assert sorted((q.stream, q.start, q.end) for q in g.free) == [(0, 50.0, 100.0), (1, 50.0, 150.0)]
    assert (g.W, g.I, g.U) == (10 + 5 + 7 + 1, 6 + 3, 1.0)
    _validate([p0, p1, p2, p3], placed, g, 100.0, 1.0)


def test_coral_rejections_each_condition():
    big = sched.SModel("big", -1, {1: 10.0}, util=0.7, weight_mem=50, inter_mem=10)
    wide = sched.SModel("wide", -1, {1: 10.0}, util=0.4, weight_mem=1, inter_mem=1)
    fat = sched.SModel("fat", -1, {1: 10.0}, util=0.1, weight_mem=45, inter_mem=1)
    long_ = sched.SModel("long", -1, {1: 120.0}, util=0.1, weight_mem=1, inter_mem=1)
    short = sched.SModel("short", -1, {1: 5.0}, util=0.1, weight_mem=1, inter_mem=1)
    ps = [sched.SPipeline("a", [big], 200.0), sched.SPipeline("b", [wide], 200.0),
          sched.SPipeline("c", [fat], 200.0), sched.SPipeline("d", [long_], 200.0),
          sched.SPipeline("e", [short], 100.0)]
    placed, g = sched.coral(ps, mem=100.0, util_max=1.0, n_streams=3)
    # wide: 0.7 + 0.4 > 1 on any other stream, and stream 0 has no portion starting at 0 -> rejected (utilisation)
    # fat: 60 + 45 + 1 > 100 -> rejected (memory); long: 120 > duty 100 -> rejected (cycle)
    # short (duty 50): stream 0 has duty 100 > 50 and no portion at 0; stream 1 is fresh -> placed there
    assert [q.stream for q in placed] == [0, -1, -1, -1, 1]
    assert placed[4].duty_cycle == 50.0
    _validate(ps, placed, g, 100.0, 1.0)


def test_coral_random_schedules_validate():
    rng = np.random.default_rng(3)
    for _ in range(40):
        pipes = []
        for k in range(int(rng.integers(1, 5))):
            p = _pipe(rng, int(rng.integers(1, 4)), slo=float(rng.choice([200, 300])))
            for m in p.models:
                m.util = float(rng.choice([0.125, 0.25, 0.5]))
                m.weight_mem = float(rng.uniform(1, 10)); m.inter_mem = float(rng.uniform(1, 10))
            sched.cwd_lite(p)
            pipes.append(p)
        placed, g = sched.coral(pipes, mem=60.0, util_max=1.0, n_streams=int(rng.integers(1, 6)))
        assert len(placed) == sum(len(p.models) for p in pipes)
        _validate(pipes, placed, g, 60.0, 1.0)
