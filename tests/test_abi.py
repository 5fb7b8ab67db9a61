"""CPU-only checks of the C ABI: the library loads, exports what the header declares, validates arguments on
the host, and its two scheduling entry points agree with the oracle (host logic, no GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import sched
from paper_2502_01277_amd import binding, zoo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    src = open(os.path.join(ROOT, "include", "octo.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(octo_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    declared = _header_functions()
    assert len(declared) >= 30
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(binding.EXPORTS) == declared


def test_letterbox_geometry_matches_the_oracle():
    from oracle import preprocess as pre
    rng = np.random.default_rng(5)
    shapes = [(1080, 1920, 640, 640), (2160, 3840, 1280, 1280), (720, 1280, 640, 640), (320, 320, 320, 320), (100, 37, 64, 64), (45, 83, 64, 64)]
    shapes += [tuple(int(v) for v in rng.integers(8, 900, 4)) for _ in range(200)]
    for (sh, sw, dh, dw) in shapes:
        assert binding.letterbox_geometry(sh, sw, dh, dw) == tuple(pre.letterbox_geometry(sh, sw, dh, dw)[1:]), (sh, sw, dh, dw)
    with pytest.raises(binding.OctoError):
        binding.letterbox_geometry(0, 10, 10, 10)


def test_record_sizes_match_header():
    assert binding.CAND_DTYPE.itemsize == 32 and binding.ROI_DTYPE.itemsize == 32 and binding.BOX_DTYPE.itemsize == 32
    assert binding.FRAME_DTYPE.itemsize == 32


def test_workspace_size_and_host_validation():
    L = binding.lib()
    n = C.c_size_t()
    keep = []
    d = binding.pipeline_desc(zoo.tiny_cascade(), keep)
    assert L.octo_pipeline_workspace_size(C.byref(d), C.byref(n)) == binding.OK and 1e6 < n.value < 1e9
    assert L.octo_pipeline_workspace_size(None, C.byref(n)) == binding.EINVAL
    assert L.octo_pipeline_workspace_size(C.byref(d), None) == binding.EINVAL
    d.models[0].layers[1].in_[0] = 7                       # forward reference
    assert L.octo_pipeline_workspace_size(C.byref(d), C.byref(n)) == binding.EINVAL
    assert b"layer input id" in L.octo_last_error(None)
    d = binding.pipeline_desc(zoo.tiny_cascade(), keep)
    d.models[0].topk = 5000                                # beyond what the sorter handles
    d.models[0].dtype = 7
    assert L.octo_pipeline_workspace_size(C.byref(d), C.byref(n)) == binding.EINVAL
    d = binding.pipeline_desc(zoo.tiny_cascade(), keep)
    d.edges[0].parent = 1                                  # only root-to-child edges
    assert L.octo_pipeline_workspace_size(C.byref(d), C.byref(n)) == binding.EINVAL
    out = C.c_void_p()
    assert L.octo_pipeline_create(C.byref(d), None, 0, C.byref(out)) == binding.EINVAL
    assert L.octo_op_nms_scratch_bytes(8, 1024) == 8 * 1024 * 16 * 8
    assert L.octo_now_ms() > 0


def test_stream_masks_are_validated_on_the_host():
    """A compute-unit mask that leaves one of the eight dies without units is refused before any HIP call (bit i of a
    mask selects unit i / 8 of die i % 8), and so are empty arguments."""
    L = binding.lib()
    out = C.c_void_p()
    one_die = (C.c_uint32 * 8)(*([0x01010101] * 8))            # bits 0, 8, 16, ...: die 0 only
    assert L.octo_stream_create_masked(one_die, 8, C.byref(out)) == binding.EINVAL
    two_dies = (C.c_uint32 * 8)(*([0x03030303] * 8))
    assert L.octo_stream_create_masked(two_dies, 8, C.byref(out)) == binding.EINVAL
    assert L.octo_stream_create_masked(None, 8, C.byref(out)) == binding.EINVAL
    assert L.octo_stream_create_masked(one_die, 0, C.byref(out)) == binding.EINVAL
    assert L.octo_stream_destroy(None) == binding.EINVAL
    assert out.value is None


def _rand_models(rng, n):
    ms = []
    for i in range(n):
        base, slope = rng.uniform(1, 6), rng.uniform(0.2, 2.0)
        ms.append(dict(parent=-1 if i == 0 else int(rng.integers(0, i)),
                       profile={b: float(np.float32(base + slope * b)) for b in (1, 2, 4, 8, 16, 32, 64)},
                       rate=float(np.float32(rng.uniform(15, 400))), burstiness=float(np.float32(rng.uniform(0, 3))),
                       util=float(rng.choice([0.125, 0.25, 0.5])), weight_mem=float(np.float32(rng.uniform(1, 10))),
                       inter_mem=float(np.float32(rng.uniform(1, 10)))))
    return ms


def _oracle_pipe(ms, slo):
    return sched.SPipeline("p", [sched.SModel("m", m["parent"], dict(m["profile"]), m["rate"], m["burstiness"], m["util"],
                                              m["weight_mem"], m["inter_mem"], m.get("bz", 1)) for m in ms], slo)


def test_cwd_search_matches_oracle():
    rng = np.random.default_rng(0)
    for _ in range(60):
        ms = _rand_models(rng, int(rng.integers(1, 5)))
        slo = float(rng.choice([60, 100, 200, 300]))
        assert binding.cwd_search(ms, slo) == sched.cwd_lite(_oracle_pipe(ms, slo))


def test_coral_schedule_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(40):
        pipes = []
        for k in range(int(rng.integers(1, 5))):
            ms = _rand_models(rng, int(rng.integers(1, 4)))
            slo = float(rng.choice([200, 300]))
            for m, b in zip(ms, sched.cwd_lite(_oracle_pipe(ms, slo))):
                m["bz"] = b
            pipes.append((ms, slo))
        ns = int(rng.integers(1, 6))
        got = binding.coral_schedule(pipes, 60.0, 1.0, ns)
        ref, _ = sched.coral([_oracle_pipe(ms, slo) for ms, slo in pipes], mem=60.0, util_max=1.0, n_streams=ns)
        assert len(got) == len(ref)
        for g, r in zip(got, ref):
            assert g[:3] == (r.pipeline, r.model, r.stream)
            if r.stream >= 0:
                assert abs(g[3] - r.start) < 1e-3 and abs(g[4] - r.end) < 1e-3 and abs(g[5] - r.duty_cycle) < 1e-3


def test_coral_hand_example_through_the_abi():
    A = dict(parent=-1, profile={1: 30.0}, util=0.5, weight_mem=10, inter_mem=4)
    B = dict(parent=0, profile={1: 20.0}, util=0.3, weight_mem=5, inter_mem=6)
    Cm = dict(parent=-1, profile={1: 40.0}, util=0.5, weight_mem=7, inter_mem=3)
    D = dict(parent=-1, profile={1: 45.0}, util=0.2, weight_mem=1, inter_mem=1)
    got = binding.coral_schedule([([A, B], 200.0), ([Cm], 300.0), ([D], 250.0)], 100.0, 1.0, 2)
    assert [g[2:] for g in got] == [(0, 0.0, 30.0, 100.0), (0, 30.0, 50.0, 100.0), (1, 0.0, 40.0, 150.0), (-1, 0.0, 0.0, 0.0)]
