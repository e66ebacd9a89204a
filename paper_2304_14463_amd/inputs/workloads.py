"""The five synthetic workloads and a helper for ad-hoc test workloads.

Shapes follow the paper's evaluation (Section 3, Table 2): C = 2 copies per
node in every run of the paper, budgets at a percentage of the no-remat peak
of a random input topological order, (n, m) = (442, 1247) for the real-world
graph the headline figure uses, random layered graphs up to n = 1000.  The two
largest workloads go beyond the paper's sizes.

Budget rounding: M = floor(pct * P / 100).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

from . import graphs as G
from .candidates import base_candidate, candidate_tables, gen_candidates

BASE_SEED = 0x230414463000


@dataclass
class Workload:
    name: str
    seed: int
    graph: G.Graph
    C: int
    B: int
    pct: int
    order: list
    no_remat_peak: int
    budget: int
    pos: np.ndarray
    out_ptr: np.ndarray
    cons_pos: np.ndarray
    win_hi: np.ndarray
    ncut: np.ndarray
    R: int = 0  # neighbourhood radius (0: plain evaluation workload)
    dense: bool = False  # the dense batch: nearly every copy live (see candidates.py)

    @property
    def n(self):
        return self.graph.n

    @property
    def m(self):
        return self.graph.m

    @property
    def T(self):
        return self.graph.n * self.C

    def base(self):
        return base_candidate(self.n, self.C, self.pos, self.out_ptr, self.cons_pos)

    def candidates(self, b0=0, count=None):
        if count is None:
            count = self.B - b0
        return gen_candidates(self.seed, self.n, self.C, self.B, self.pos, self.out_ptr,
                              self.cons_pos, self.win_hi, self.ncut, b0, count, dense=self.dense)


def workload_from_graph(name, seed, graph, C, B, pct, R=0, order=None):
    if order is None:
        order = G.random_topological_order(seed, graph)
    P = G.no_remat_peak(graph, order)
    pos, out_ptr, cons_pos, win_hi, ncut = candidate_tables(graph, order, C)
    return Workload(name, seed, graph, C, B, pct, order, P, (pct * P) // 100, pos, out_ptr, cons_pos,
                    win_hi, ncut, R)


def _layered(cfg, n, layers, dmin, dmax, skew, single_sink, target_m, size_fn, dur_hi):
    seed = BASE_SEED + cfg
    edges = G.layered_dag_edges(seed, n, layers, dmin, dmax, skew, single_sink, target_m)
    size = size_fn(seed, n)
    dur = G.uniform_ints(seed, G.S_DUR, n, 1, dur_hi)
    return seed, G.graph_from_edges(n, edges, size, dur)


def make_workload(cfg: int, B: int | None = None, dense: bool = False) -> Workload:
    """cfg 0..4; B overrides the batch size (the type-A/type-B split follows B); dense: same
    graph, order and budget with the dense candidate batch."""
    if dense:
        w = make_workload(cfg, B)
        w.dense = True
        w.name += "-dense"
        return w
    if cfg == 0:
        seed, g = _layered(0, 50, 10, 1, 3, False, True, None,
                           lambda s, n: G.uniform_ints(s, G.S_SIZE, n, 1, 100), 50)
        return workload_from_graph("layered-n50-C2", seed, g, 2, B or 1024, 80)
    if cfg == 1:
        seed, g = _layered(1, 442, 20, 1, 5, True, False, 1247,
                           lambda s, n: G.lognormal_sizes(s, n, math.log(64), 1.0), 100)
        return workload_from_graph("layered-n442-m1247-C2", seed, g, 2, B or 16384, 80)
    if cfg == 2:
        seed = BASE_SEED + 2
        L = 500
        edges = G.training_dag_edges(L)
        size = G.lognormal_sizes(seed, 2 * L, math.log(256), 0.7)
        dur = G.proportional_durations(seed, size)
        g = G.graph_from_edges(2 * L, edges, size, dur)
        return workload_from_graph("training-n1000-C2", seed, g, 2, B or 65536, 60)
    if cfg == 3:
        seed, g = _layered(3, 2000, 40, 1, 6, True, False, 6000,
                           lambda s, n: G.lognormal_sizes(s, n, math.log(128), 1.2), 200)
        return workload_from_graph("layered-n2000-C2-neighbours", seed, g, 2, B or 8192, 70, R=8)
    if cfg == 4:
        seed, g = _layered(4, 5000, 100, 1, 6, True, False, 15000,
                           lambda s, n: G.lognormal_sizes(s, n, math.log(128), 1.0), 200)
        return workload_from_graph("layered-n5000-C3", seed, g, 3, B or 262144, 50)
    raise ValueError(f"unknown workload {cfg}")
