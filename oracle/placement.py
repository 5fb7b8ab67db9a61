"""Oracle: cross-device placement of a pipeline's models (test infrastructure).

The second half of the paper's Algorithm 1 (function ToEdge, Sec. III-B): after the batch-size search has configured
every model on the server, models are moved to the edge device where the data source is, depth first from the root,
as long as a configuration for them exists there; on the way back a model whose output costs more network than its
input (times alpha) and whose downstream models all stayed on the server is sent back to the server (Insights 2, 3).

parity unpinned (against the paper): the paper gives no worked example and leaves "find a new configuration only for
m", Overhead() and the latency estimate undefined.  READINGS, all stated where they are used:
  * latency and throughput estimates follow Eq. (1): a model whose upstream model (for the root: the data source, which
    is on the edge) sits on the other device pays size(In_m) / BW per request; on the same device the IO term is zero;
  * EstLat is the worst case of a batch's first request along the longest root-to-leaf path (Sec. II, constraint a),
    EstThrpt is 1 / sum_m L_m (Eq. 2), exactly as in oracle/sched.py, plus the IO terms;
  * "a new configuration only for m" on the edge: only m's device and batch size change; among the batch sizes profiled
    on the edge, those that keep EstLat within SLO/2 and the edge device within its compute (sum over edge models of
    rate x L(bz)/bz at most one second per second) are feasible; the one with the largest EstThrpt is taken, the
    smallest on ties; none feasible = NULL;
  * Overhead(In_m) = rate_m x size(In_m) and Overhead(Out_m) = sum over downstream models of rate x size(In), or
    rate_m x result bytes for a leaf: bytes per second either would put on the network;
  * "downstreams are not on Edge" = no downstream model of m is on the edge (true for a leaf).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List


@dataclass
class PModel:
    parent: int                       # index of the upstream model, -1 for the root
    rate: float                       # requests per second reaching the model
    burstiness: float
    server_ms: Dict[int, float]       # batch size -> batch latency on the server
    edge_ms: Dict[int, float]         # batch size -> batch latency on the edge device
    in_bytes: float                   # size(In_m): bytes of one request entering the model
    result_bytes: float = 0.0         # bytes of one result leaving the pipeline here (leaves)
    bz: int = 1
    on_edge: bool = False

    def batch_ms(self) -> float:
        return (self.edge_ms if self.on_edge else self.server_ms)[self.bz]


def _io_ms(models: List[PModel], i: int, bandwidth: float) -> float:
    """Eq. (1), second term, in ms: the request crosses the network iff the model and its upstream are on different devices."""
    m = models[i]
    upstream_on_edge = True if m.parent < 0 else models[m.parent].on_edge
    return 1000.0 * m.in_bytes / bandwidth if upstream_on_edge != m.on_edge else 0.0


def est_latency(models: List[PModel], bandwidth: float) -> float:
    def path(i):
        m = models[i]
        own = m.batch_ms() + (m.bz - 1) * 1000.0 / m.rate + _io_ms(models, i, bandwidth)
        return own + (path(m.parent) if m.parent >= 0 else 0.0)
    leaves = [i for i in range(len(models)) if all(c.parent != i for c in models)]
    return max(path(i) for i in leaves)


def est_throughput(models: List[PModel], bandwidth: float) -> float:
    return 1000.0 / sum(m.batch_ms() / m.bz + _io_ms(models, i, bandwidth) for i, m in enumerate(models))


def edge_load(models: List[PModel]) -> float:
    """Seconds of edge compute needed per second."""
    return sum(m.rate * m.batch_ms() / m.bz / 1000.0 for m in models if m.on_edge)


def to_edge(models: List[PModel], slo_ms: float, bandwidth: float, alpha: float) -> List[PModel]:
    """ToEdge(root).  models: topological order, every model on the server with its batch size chosen.  Modifies and returns them."""
    children = lambda i: [c for c in range(len(models)) if models[c].parent == i]

    def visit(i):
        m = models[i]
        kept = (m.bz, m.on_edge)
        # a new configuration only for m, on the edge
        best = None
        for bz in sorted(m.edge_ms):
            m.bz, m.on_edge = bz, True
            if est_latency(models, bandwidth) <= slo_ms / 2 and edge_load(models) <= 1.0:
                thr = est_throughput(models, bandwidth)
                if best is None or thr > best[0]:
                    best = (thr, bz)
        if best is None:
            m.bz, m.on_edge = kept
            return
        m.bz, m.on_edge = best[1], True
        for c in sorted(children(i), key=lambda c: models[c].burstiness):        # the least bursty first (Insight 1)
            visit(c)
        kids = children(i)
        out = sum(models[c].rate * models[c].in_bytes for c in kids) if kids else m.rate * m.result_bytes
        if m.rate * m.in_bytes * alpha < out and not any(models[c].on_edge for c in kids):
            m.bz, m.on_edge = kept                                               # not a split point worth having (Insights 2, 3)

    visit(0)
    return models
