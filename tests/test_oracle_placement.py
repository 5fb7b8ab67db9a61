"""Cross-device placement (Algorithm 1, function ToEdge): the oracle against cases worked by hand, and the library's
octo_to_edge against the oracle on random pipelines (exact placements and batch sizes, estimates to fp32 rounding).

parity unpinned against the paper (it has no worked example); the hand cases pin the readings stated in oracle/placement.py."""
import copy

import numpy as np
import pytest

from oracle import placement as opl
from paper_2502_01277_amd import binding


def _pipeline(c_rate=40.0, d_edge=None, alpha=1.0):
    """Detector (10 frames/s of 1 MB) feeding a classifier (100 KB crops, 100-byte results); 10 MB/s link; objective 400 ms."""
    D = opl.PModel(-1, 10.0, 0.0, {1: 10.0, 2: 16.0}, d_edge or {1: 50.0, 2: 90.0}, 1e6)
    C = opl.PModel(0, c_rate, 0.5, {1: 2.0, 2: 3.0}, {1: 10.0, 2: 12.0}, 1e5, 100.0)
    return [D, C]


def test_estimates_with_the_network_term_by_hand():
    m = _pipeline()
    # everything on the server: the frame crosses the link (1e6 / 1e7 s = 100 ms), the crop does not
    assert opl.est_latency(m, 1e7) == pytest.approx(10 + 100 + 2)
    assert opl.est_throughput(m, 1e7) == pytest.approx(1000 / 112)
    m[0].on_edge = True                          # split after the detector: the crop crosses instead (10 ms)
    assert opl.est_latency(m, 1e7) == pytest.approx(50 + 2 + 10)
    assert opl.edge_load(m) == pytest.approx(10 * 50 / 1000)
    m[1].on_edge, m[1].bz = True, 2              # both on the edge: nothing crosses; the classifier's first request waits 1 / 40 s
    assert opl.est_latency(m, 1e7) == pytest.approx(50 + 12 + 25)
    assert opl.est_throughput(m, 1e7) == pytest.approx(1000 / (50 + 6))
    assert opl.edge_load(m) == pytest.approx(0.5 + 40 * 6 / 1000)


def test_to_edge_hand_cases():
    # light load: the detector fits the edge at bz 1 (bz 2: 90 + 100 wait + 12 > 200), the classifier at bz 2 (best throughput)
    m = opl.to_edge(_pipeline(), 400.0, 1e7, 1.0)
    assert [(x.on_edge, x.bz) for x in m] == [(True, 1), (True, 2)]
    # rush hour (Insight 2): 200 crops/s need 2.5 s (bz 1) or 1.7 s (bz 2) of edge compute per second with the detector's 0.5 - no
    # configuration; the detector's output (2e7 B/s) now exceeds its input (1e7 B/s) and nothing downstream is on the edge: back to the server
    m = opl.to_edge(_pipeline(c_rate=200.0), 400.0, 1e7, 1.0)
    assert [(x.on_edge, x.bz) for x in m] == [(False, 1), (False, 1)]
    # a tolerant alpha keeps the split after the detector
    m = opl.to_edge(_pipeline(c_rate=200.0), 400.0, 1e7, 3.0)
    assert [(x.on_edge, x.bz) for x in m] == [(True, 1), (False, 1)]
    # an edge device too slow for the detector (1.5 s of compute per second): nothing moves, downstream is never visited
    m = opl.to_edge(_pipeline(d_edge={1: 150.0, 2: 280.0}), 400.0, 1e7, 1.0)
    assert [(x.on_edge, x.bz) for x in m] == [(False, 1), (False, 1)]


def _random_pipeline(rng):
    n = int(rng.integers(1, 6))
    bzs = [1, 2, 4, 8, 16][: int(rng.integers(1, 6))]
    models = []
    for i in range(n):
        base = float(rng.integers(4, 80)) / 8.0
        slow = float(rng.integers(3, 12)) / 2.0
        srv = {b: round(8 * base * (1 + 0.4 * np.log2(b) * b ** 0.5)) / 8.0 for b in bzs}
        models.append(opl.PModel(-1 if i == 0 else int(rng.integers(0, i)), float(rng.integers(1, 60)), float(rng.integers(0, 16)) / 8.0,
                                 srv, {b: v * slow for b, v in srv.items()}, float(rng.integers(1, 4000)) * 1024.0,
                                 float(rng.integers(1, 64)) * 16.0, int(rng.choice(bzs))))
    return models


def test_library_placement_equals_the_oracle_on_random_pipelines():
    rng = np.random.default_rng(21)
    moved = partial = 0
    for _ in range(400):
        models = _random_pipeline(rng)
        slo = float(rng.choice([100.0, 200.0, 400.0, 1000.0]))
        bw = float(rng.choice([1e5, 1e6, 1e7, 1e8, 1e9]))
        alpha = float(rng.choice([0.5, 1.0, 2.0]))
        as_dicts = [dict(parent=m.parent, rate=m.rate, burstiness=m.burstiness, server_ms=m.server_ms, edge_ms=m.edge_ms, in_bytes=m.in_bytes,
                         result_bytes=m.result_bytes, bz=m.bz) for m in models]
        got, lat, thr = binding.to_edge(as_dicts, slo, bw, alpha)
        ref = opl.to_edge(copy.deepcopy(models), slo, bw, alpha)
        assert got == [(m.on_edge, m.bz) for m in ref]
        rl, rt = opl.est_latency(ref, bw), opl.est_throughput(ref, bw)
        assert abs(lat - rl) <= 1e-5 * rl and abs(thr - rt) <= 1e-5 * rt
        # what the method guarantees: the edge models form a subtree from the root, and the edge device is not overloaded
        for m in ref:
            assert not m.on_edge or m.parent < 0 or ref[m.parent].on_edge
        assert opl.edge_load(ref) <= 1.0 + 1e-9
        on = sum(m.on_edge for m in ref)
        moved += on > 0
        partial += 0 < on < len(ref)
    assert moved > 40 and partial > 10               # the cases really exercise all three outcomes


def test_octo_to_edge_rejects_bad_descriptions():
    ok = [dict(parent=-1, rate=10.0, burstiness=0.0, server_ms={1: 1.0}, edge_ms={1: 2.0}, in_bytes=1e5, result_bytes=10.0, bz=1)]
    binding.to_edge(ok, 200.0, 1e7, 1.0)
    for bad in (dict(ok[0], rate=0.0), dict(ok[0], bz=2), dict(ok[0], parent=0), dict(ok[0], in_bytes=-1.0)):
        with pytest.raises(binding.OctoError):
            binding.to_edge([bad], 200.0, 1e7, 1.0)
    for args in ((0.0, 1e7, 1.0), (200.0, 0.0, 1.0), (200.0, 1e7, 0.0)):
        with pytest.raises(binding.OctoError):
            binding.to_edge(ok, *args)
