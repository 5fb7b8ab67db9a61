"""Pins of the oracle's run-time rules (oracle/runtime.py) by hand-computed cases."""
import math

from oracle import runtime as rt


def test_burstiness_hand_cases():
    assert rt.burstiness([]) == 0.0 and rt.burstiness([1.0, 2.0]) == 0.0               # fewer than two gaps
    assert rt.burstiness([0.0, 1.0, 2.0, 3.0]) == 0.0                                  # regular arrivals: no variation
    # gaps 1, 3: mean 2, population variance ((1)^2 + (1)^2) / 2 = 1 -> CV 1/2; order of the input does not matter
    assert abs(rt.burstiness([4.0, 0.0, 1.0]) - 0.5) < 1e-12
    # gaps 0, 0, 0, 4 (a burst of four, then a pause): mean 1, variance (3 * 1 + 9) / 4 = 3 -> CV sqrt(3)
    assert abs(rt.burstiness([0.0, 0.0, 0.0, 0.0, 4.0]) - math.sqrt(3.0)) < 1e-12
    assert rt.burstiness([5.0, 5.0, 5.0]) == 0.0                                       # all at once: zero mean gap


def test_batches_per_cycle_hand_cases():
    assert rt.batches_per_cycle(90.0, 100.0, 16) == 1        # 9 requests per cycle fit one batch of 16
    assert rt.batches_per_cycle(160.0, 100.0, 16) == 1       # exactly 16
    assert rt.batches_per_cycle(161.0, 100.0, 16) == 2
    assert rt.batches_per_cycle(0.001, 100.0, 8) == 1        # never less than one
    assert rt.batches_per_cycle(720.0, 100.0, 8) == 9


def test_width_to_cus_hand_cases():
    assert rt.width_to_cus(0.25, 256) == 64 and rt.width_to_cus(1.0, 256) == 256 and rt.width_to_cus(0.5, 256) == 128
    assert rt.width_to_cus(0.26, 256) == 72                  # 66.56 units -> 9 groups of 8
    assert rt.width_to_cus(0.001, 256) == 8 and rt.width_to_cus(1.7, 256) == 256
    assert rt.width_to_cus(0.3, 64, grain=8) == 24


def test_choose_width_hand_cases():
    # a model that scales perfectly costs the same everywhere: the narrowest width
    assert rt.choose_width({64: 8.0, 128: 4.0, 256: 2.0}) == 64
    # a model that does not scale at all: also the narrowest (more units only cost more)
    assert rt.choose_width({64: 3.0, 128: 3.0, 256: 3.0}) == 64
    # super-linear gain from 64 to 128 (cost 640 -> 384), none beyond (768): 128
    assert rt.choose_width({64: 10.0, 128: 3.0, 256: 3.0}) == 128
    # within the tolerance of the cheapest: 64 x 4.3 = 275 <= 1.1 x 256
    assert rt.choose_width({64: 4.3, 128: 2.0, 256: 1.5}) == 64
    assert rt.choose_width({64: 4.5, 128: 2.0, 256: 1.5}) == 128
    # 'latency': the narrowest width within 10 % of the whole GPU's latency
    assert rt.choose_width({64: 4.0, 128: 2.1, 256: 2.0}, rule="latency") == 128
    assert rt.choose_width({64: 2.2, 128: 2.1, 256: 2.0}, rule="latency") == 64


def test_late_prefix_hand_cases():
    now, slo = 1000.0, 200.0
    assert rt.late_prefix([], now, slo) == 0
    assert rt.late_prefix([900.0, 950.0], now, slo) == 0
    assert rt.late_prefix([799.0, 799.9, 800.0, 900.0], now, slo) == 2                  # exactly the objective old is still served
    assert rt.late_prefix([100.0, 200.0, 300.0], now, slo) == 3
    assert rt.late_prefix([700.0, 900.0, 750.0], now, slo) == 1                         # stops at the first live request


def _run(s, arrivals, backlog=None, n_active=1):
    out = []
    for t, a in enumerate(arrivals):
        d = s.observe(a, 0 if backlog is None else backlog[t], n_active)
        n_active += d
        out.append(d)
    return out, n_active


def test_scaler_hand_cases():
    # capacity 32, window 4: nothing before four cycles; mean of (40, 40, 40, 40) = 40 > 32 -> +1 at the fourth cycle
    assert _run(rt.Scaler(32, window=4), [40, 40, 40, 40]) == ([0, 0, 0, 1], 2)
    # the window empties on a decision: the next one needs four new cycles; with two instances 64 per cycle are served,
    # mean 40 is neither above 64 nor below 0.75 x 32 = 24 -> nothing
    assert _run(rt.Scaler(32, window=4), [40] * 12)[0] == [0, 0, 0, 1] + [0] * 8
    # dip: mean 20 < 24 with an empty queue -> -1 once the window has refilled
    assert _run(rt.Scaler(32, window=4), [40] * 4 + [20] * 4)[0] == [0, 0, 0, 1, 0, 0, 0, -1]
    # between the thresholds (24 <= mean <= 32) nothing changes in either state
    assert not any(_run(rt.Scaler(32, window=4), [30] * 10)[0])
    assert not any(_run(rt.Scaler(32, window=4), [30] * 10, n_active=2)[0])
    # arrivals look fine (30) but the queue never falls to the capacity: +1
    assert _run(rt.Scaler(32, window=4), [30] * 4, backlog=[50, 45, 40, 33])[0] == [0, 0, 0, 1]
    assert _run(rt.Scaler(32, window=4), [30] * 4, backlog=[50, 45, 32, 33])[0] == [0, 0, 0, 0]
    # no removal while the queue does not fit the remaining instance
    assert _run(rt.Scaler(32, window=4), [10] * 4, backlog=[0, 0, 0, 33], n_active=2)[0] == [0, 0, 0, 0]
    assert _run(rt.Scaler(32, window=4), [10] * 4, backlog=[0, 0, 0, 32], n_active=2)[0] == [0, 0, 0, -1]
    # never more than max_instances, never fewer than one
    assert not any(_run(rt.Scaler(32, window=2, max_instances=2), [100] * 6, n_active=2)[0])
    assert not any(_run(rt.Scaler(32, window=2), [0] * 6, n_active=1)[0])
