"""Host logic of the slot executor that needs no GPU, through the C ABI: the run-time rules (burstiness, batches per
cycle, widths, lazy dropping, the scaling decision) equal the oracle's on hand cases and on random inputs; the property
of the portion scheduler the scaler relies on; the surge in the synthetic arrivals."""
import numpy as np

from oracle import runtime as ort, sched
from paper_2502_01277_amd import binding, executor, synth


# ---- the library's run-time rules against the oracle's (exact equality) ----
def test_runtime_rules_equal_the_oracle_on_random_inputs():
    rng = np.random.default_rng(11)
    for _ in range(300):
        n = int(rng.integers(0, 40))
        t = np.round(rng.uniform(0, 10, n), 3)
        if n and rng.random() < 0.3:
            t[rng.integers(0, n, n // 2)] = t[0]                     # bursts: equal arrival times
        assert abs(binding.burstiness(t) - ort.burstiness(t.tolist())) <= 1e-12
        rate, duty, bz = float(rng.uniform(0, 2000)), float(rng.choice([25.0, 50.0, 100.0])), int(2 ** rng.integers(0, 7))
        assert binding.batches_per_cycle(rate, duty, bz) == ort.batches_per_cycle(rate, duty, bz)
        util, total = float(rng.uniform(0, 1.2)), int(rng.choice([64, 256, 304]))
        assert binding.width_to_cus(util, total, 8) == ort.width_to_cus(util, total, 8)
        lat = {int(w): float(rng.uniform(0.5, 20)) for w in rng.choice([8, 16, 32, 64, 128, 256], size=int(rng.integers(1, 5)), replace=False)}
        for rule in ("efficient", "latency"):
            assert binding.choose_width(lat, rule, 0.1) == ort.choose_width(lat, rule, 0.1), (lat, rule)
        arr = np.sort(rng.uniform(0, 1000, n))
        now, slo = float(rng.uniform(0, 1200)), float(rng.choice([50.0, 200.0]))
        assert binding.late_prefix(arr, now, slo) == ort.late_prefix(arr.tolist(), now, slo)
    assert binding.batches_per_cycle(160.0, 100.0, 16) == 1 and binding.batches_per_cycle(161.0, 100.0, 16) == 2
    assert binding.width_to_cus(0.26, 256) == 72 and binding.choose_width({64: 10.0, 128: 3.0, 256: 3.0}) == 128


def _random_plan_case(rng):
    """A pipeline of 1-3 models with latencies (multiples of 1/8 ms, exact in fp32) that fall with the width and grow with the batch."""
    n = int(rng.integers(1, 4))
    widths = [64, 128, 256][: int(rng.integers(1, 4))]
    bzs = [1, 2, 4, 8, 16, 32][: int(rng.integers(2, 7))]
    models = []
    for i in range(n):
        base = float(rng.integers(2, 40)) / 8.0
        by_width = {}
        for j, w in enumerate(widths):
            speed = 1.0 + 0.6 * j * float(rng.uniform(0.2, 1.0))
            by_width[w] = {b: round(8 * base * (1 + 0.35 * np.log2(b) * b ** 0.5) / speed) / 8.0 + 0.125 for b in bzs}
        models.append(dict(parent=-1 if i == 0 else int(rng.integers(0, i)), rate=float(rng.integers(5, 4000)), burstiness=float(rng.integers(0, 30)) / 8.0,
                           weight_mem=float(rng.integers(1, 200)), inter_mem=0.0, width=int(rng.choice(widths)), by_width=by_width))
    return models, widths, bzs


def test_plan_pipeline_equals_the_oracle_and_its_hand_case():
    """Load-aware widths around Algorithm 1 through the C ABI against oracle/runtime.plan_pipeline: batch sizes, batches per
    cycle, accepted widths, the k-fold portion lengths and both estimates on random pipelines; then a case worked by hand."""
    rng = np.random.default_rng(14)
    moved = 0
    for _ in range(200):
        models, widths, bzs = _random_plan_case(rng)
        slo, share = float(rng.choice([50.0, 100.0, 200.0])), float(rng.choice([0.25, 0.5, 0.8]))
        fixed = None if rng.random() < 0.7 else [int(rng.choice(bzs)) for _ in models]
        got, ks, lat, thr = binding.plan_pipeline(models, slo, slo / 2, share, widths, 256, fixed)
        ref, rks, rlat, rthr = ort.plan_pipeline(models, slo, slo / 2, share, widths, 256, fixed)
        assert ks == rks and [g["bz"] for g in got] == [r.bz for r in ref]
        assert [round(g["util"] * 256) for g in got] == [round(r.util * 256) for r in ref]
        for g, r in zip(got, ref):
            assert all(abs(g["profile"][b] - r.profile[b]) <= 1e-4 * r.profile[b] for b in r.profile)
        assert abs(lat - rlat) <= 1e-4 * rlat and abs(thr - rthr) <= 1e-4 * rthr
        moved += any(round(g["util"] * 256) > m["width"] for g, m in zip(got, models))
    assert moved > 10                                        # the width floor really moved in some of the cases
    # by hand: one model, 1000 requests/s, duty 100 ms -> 100 requests per cycle.  At 64 units L(8) = 10 ms, L(16) = 30 ms; Algorithm 1
    # (SLO 200: latency bound 100 ms; wait of a batch's first request (bz - 1) ms) doubles 1 -> 2 -> 4 -> 8 while throughput
    # grows (L/bz: 2, 1.5, 1.25 at bz 1, 2, 4; 1.25 at 8 is no better, so it stops at 4): k = ceil(100 / 4) = 25 batches of 5 ms =
    # 125 ms of work > 0.5 x 100 -> next width.  At 128 units L = 1, 1.5, 2, 3, 8 ms: L/bz = 1, .75, .5, .375, .5 -> bz 8, k = 13,
    # work 39 ms <= 50: accepted; the portion is 13 x 3 = 39 ms long.
    m = [dict(parent=-1, rate=1000.0, burstiness=0.0, weight_mem=1.0, inter_mem=0.0, width=64,
              by_width={64: {1: 2.0, 2: 3.0, 4: 5.0, 8: 10.0, 16: 30.0}, 128: {1: 1.0, 2: 1.5, 4: 2.0, 8: 3.0, 16: 8.0}})]
    for plan in (binding.plan_pipeline, ort.plan_pipeline):
        out, ks, lat, thr = plan(m, 200.0, 100.0, 0.5, [64, 128], 256)
        o = out[0] if isinstance(out[0], dict) else dict(bz=out[0].bz, util=out[0].util, profile=out[0].profile)
        assert o["bz"] == 8 and ks == [13] and abs(o["util"] - 0.5) < 1e-6 and abs(o["profile"][8] - 39.0) < 1e-4
        assert abs(lat - (3.0 + 7.0)) < 1e-4 and abs(thr - 1000.0 / (3.0 / 8)) < 0.1
    out, ks, _, _ = binding.plan_pipeline(m, 200.0, 100.0, 2.0, [64, 128], 256)           # a generous share keeps the narrow width
    assert out[0]["bz"] == 4 and ks == [25] and abs(out[0]["util"] - 0.25) < 1e-6


def test_scaler_equals_the_oracle_on_random_sequences():
    rng = np.random.default_rng(12)
    for _ in range(60):
        cap, win = float(rng.integers(4, 64)), int(rng.integers(1, 7))
        up, down, mx = float(rng.uniform(0.8, 1.3)), float(rng.uniform(0.3, 0.79)), int(rng.integers(1, 4))
        a, b = binding.Scaler(cap, win, up, down, mx), ort.Scaler(cap, win, up, down, mx)
        n_active = 1
        for _ in range(80):
            arrived, backlog = int(rng.integers(0, 3 * cap)), int(rng.integers(0, 3 * cap))
            da, db = a.observe(arrived, backlog, n_active), b.observe(arrived, backlog, n_active)
            assert da == db
            n_active += da
            assert 1 <= n_active <= max(1, mx)
        a.close()
    for bad in ((0.0, 5, 1.0, 0.75, 2), (8.0, 0, 1.0, 0.75, 2), (8.0, 5, 0.5, 0.75, 2), (8.0, 5, 1.0, 0.75, 0)):
        try:
            binding.Scaler(*bad)
            assert False, bad
        except binding.OctoError:
            pass


# ---- lazy dropping (Sec. IV-A) ----
def test_late_prefix_counts_only_the_expired_head_of_the_queue():
    now, slo = 1000.0, 200.0
    assert executor.late_prefix([], now, slo) == 0
    assert executor.late_prefix([900.0, 950.0], now, slo) == 0
    assert executor.late_prefix([799.0, 799.9, 800.0, 900.0], now, slo) == 2          # exactly the SLO old is still served
    assert executor.late_prefix([100.0, 200.0, 300.0], now, slo) == 3
    # the queue is in arrival order, so an expired request behind a live one cannot happen; the count stops at the
    # first live request in any case (nothing is taken out of the middle of a batch)
    assert executor.late_prefix([700.0, 900.0, 750.0], now, slo) == 1


# ---- run-time scaling decision (Sec. III-D) ----
def _run(det, arrivals, backlog=None, n_active=1):
    """Feeds a sequence of per-cycle arrivals and applies the decisions; returns (decisions, instances over time)."""
    out, act = [], []
    for t, a in enumerate(arrivals):
        d = det.observe(a, 0 if backlog is None else backlog[t], n_active)
        n_active += d
        out.append(d)
        act.append(n_active)
    return out, act


def test_steady_load_within_capacity_never_scales():
    det = executor.SurgeDetector(capacity=32, window=5)
    dec, act = _run(det, [30, 32, 28, 31, 32, 29, 32, 30] * 5)
    assert not any(dec) and set(act) == {1}


def test_surge_adds_one_instance_after_a_full_window_and_dip_removes_it():
    det = executor.SurgeDetector(capacity=32, window=4, up=1.0, down=0.7, max_instances=2)
    arr = [30] * 6 + [60] * 12 + [20] * 10
    dec, act = _run(det, arr)
    # the first surge cycle already lifts the mean of the last 4 cycles over the capacity: (30*3 + 60)/4 = 37.5 > 32
    up_at = dec.index(1)
    assert up_at == 6
    assert dec.count(1) == 1, "two instances are the limit"
    # removal: the first whole window below 0.7 * 32 = 22.4 is cycles 18..21 (all 20); (60 + 20*3)/4 = 30 is not
    assert dec.index(-1) == 21 and act[-1] == 1 and dec.count(-1) == 1
    assert all(d == 0 for d in dec[up_at + 1: up_at + 4]), "no decision inside the window after another"


def test_load_between_the_two_thresholds_changes_nothing_in_either_state():
    for n_active in (1, 2):
        det = executor.SurgeDetector(capacity=40, window=3, up=1.0, down=0.7)
        # one instance: 30 < 40; two instances: 30 > 0.7*40 = 28 and 30 < 80
        dec, _ = _run(det, [30] * 30, n_active=n_active)
        assert not any(dec)


def test_a_queue_that_never_drains_scales_up_even_if_arrivals_look_fine():
    det = executor.SurgeDetector(capacity=16, window=3)
    dec, _ = _run(det, [10] * 6, backlog=[20, 25, 17, 30, 40, 50])
    assert dec[:3] == [0, 0, 1]
    det = executor.SurgeDetector(capacity=16, window=3)
    dec, _ = _run(det, [10] * 6, backlog=[20, 25, 16, 30, 3, 50])           # drained to within capacity in between
    assert not any(dec)


def test_scale_down_waits_until_the_queue_fits_the_remaining_instance():
    det = executor.SurgeDetector(capacity=16, window=2)
    dec, _ = _run(det, [2, 2, 2, 2], backlog=[50, 40, 17, 16], n_active=2)
    assert dec == [0, 0, 0, -1]


def test_random_sequences_keep_the_instance_count_in_range_and_decisions_apart():
    rng = np.random.default_rng(5)
    for _ in range(50):
        w = int(rng.integers(1, 7))
        det = executor.SurgeDetector(capacity=float(rng.integers(4, 64)), window=w, max_instances=3)
        arr = rng.poisson(rng.choice([5, 20, 60, 150]), size=200) * (rng.random(200) < 0.9)
        dec, act = _run(det, arr.tolist(), backlog=rng.integers(0, 80, size=200).tolist())
        assert min(act) >= 1 and max(act) <= 3
        idx = [t for t, d in enumerate(dec) if d]
        assert all(b - a >= w for a, b in zip(idx, idx[1:]))


# ---- what the scaler relies on: copies appended to the pipeline list do not move what is already scheduled ----
def _models(rng, n):
    ms = []
    for i in range(n):
        base, slope = rng.uniform(1, 6), rng.uniform(0.2, 2.0)
        ms.append(dict(parent=-1 if i == 0 else int(rng.integers(0, i)), profile={b: base + slope * b for b in (1, 2, 4, 8, 16)},
                       rate=float(rng.uniform(15, 300)), burstiness=float(rng.uniform(0, 3)), util=float(rng.uniform(0.1, 0.5)),
                       weight_mem=float(rng.uniform(1, 5)), inter_mem=float(rng.uniform(0.5, 3)), bz=int(rng.choice([1, 2, 4, 8]))))
    return ms


def test_appending_a_copy_leaves_scheduled_portions_where_they_are():
    rng = np.random.default_rng(11)
    placed_copies = 0
    for _ in range(40):
        pipes = [(_models(rng, int(rng.integers(1, 4))), float(rng.choice([200, 300]))) for _ in range(int(rng.integers(1, 4)))]
        ns = int(rng.integers(2, 7))
        base = binding.coral_schedule(pipes, 80.0, 1.0, ns)
        k = int(rng.integers(0, len(pipes)))
        ext = binding.coral_schedule(pipes + [pipes[k]], 80.0, 1.0, ns)
        assert ext[:len(base)] == base
        copy = ext[len(base):]
        assert [c[0] for c in copy] == [len(pipes)] * len(pipes[k][0])
        # the copy's portions do not overlap anything on their streams
        for c in copy:
            if c[2] < 0:
                continue
            placed_copies += 1
            for o in ext:
                if o is not c and o[2] == c[2]:
                    assert c[4] <= o[3] + 1e-4 or o[4] <= c[3] + 1e-4, (c, o)
    assert placed_copies > 10


# ---- surge in the synthetic arrivals ----
def test_boosted_arrivals_multiply_the_rate_inside_the_window_only():
    n, dur = 40, 30.0
    plain = synth.sinusoid_arrivals(np.random.default_rng(3), n, dur, base_fps=15.0, depth=0.0)
    boost = synth.sinusoid_arrivals(np.random.default_rng(3), n, dur, base_fps=15.0, depth=0.0, boost=[(10.0, 20.0, 3.0)] * n)
    def rate(streams, a, b):
        return sum(int(((s >= a) & (s < b)).sum()) for s in streams) / (len(streams) * (b - a))
    for s in boost:
        assert np.all(np.diff(s) >= 0) and s.min() >= 0 and s.max() < dur
    assert abs(rate(plain, 0, 30) - 15.0) < 0.6
    assert abs(rate(boost, 0, 10) - 15.0) < 1.0 and abs(rate(boost, 20, 30) - 15.0) < 1.0
    assert abs(rate(boost, 10, 20) - 45.0) < 2.0
    # streams without a boost entry are drawn exactly as before while no boosted stream precedes them
    mixed = synth.sinusoid_arrivals(np.random.default_rng(3), 3, dur, boost=[None, None, (1.0, 2.0, 2.0)])
    ref = synth.sinusoid_arrivals(np.random.default_rng(3), 3, dur)
    assert np.array_equal(mixed[0], ref[0]) and np.array_equal(mixed[1], ref[1]) and len(mixed[2]) > len(ref[2]) - 10
