"""Shared test plumbing: conversions between oracle objects and the library's device records, tolerances."""
import numpy as np

from oracle import postprocess as pp
from paper_2502_01277_amd import binding

# max-abs tolerance relative to max(1, max|oracle|): the bar the workloads state for fp16/bf16 and fp32
TOL = {"f32": 1e-4, "f16": 2e-2, "bf16": 2e-2}


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    return float(np.abs(got - ref).max() / max(1.0, np.abs(ref).max()))


def cands_to_records(c: pp.Candidates) -> np.ndarray:
    r = np.zeros(len(c), binding.CAND_DTYPE)
    if len(c):
        r["x1"], r["y1"], r["x2"], r["y2"] = c.box[:, 0], c.box[:, 1], c.box[:, 2], c.box[:, 3]
        r["score"], r["cls"], r["idx"] = c.score, c.cls, c.idx
    return r


def records_to_cands(r: np.ndarray) -> pp.Candidates:
    box = np.stack([r["x1"], r["y1"], r["x2"], r["y2"]], axis=1).astype(np.float32).reshape(-1, 4)
    return pp.Candidates(box, r["score"].astype(np.float32), r["cls"].astype(np.int32), r["idx"].astype(np.int32))


def small_root(dtype="f32"):
    """A tiny root detector so that other models can ride in a pipeline as detached models."""
    from paper_2502_01277_amd import zoo
    return zoo.plain_detector("root", dtype, 32, (8,), 2, seed=99, batch_size=1)
