"""Seeded synthetic compute DAGs shaped like the paper's evaluation graphs.

The paper evaluates on random layered graphs (G1..G4, up to n=1000, m=5875),
real-world inference graphs (e.g. n=442, m=1247) and training graphs with
forward/backward "U-net-like" structure (Section 3.1, Table 2).  None of those
graphs is public in a form usable here, so these generators produce stand-ins
with the same node/edge counts and structure.  Host only; plain Python loops
(n <= a few thousand).  Node ids are always a topological order.

This module holds no arithmetic of the evaluated method.
"""
from __future__ import annotations

import heapq
import math
from dataclasses import dataclass

import numpy as np

from .hashrng import hash3, uniform01

# hash streams (first counter) used by the graph generators
S_DEG, S_PRED, S_ORPHAN, S_TRIM, S_PAD, S_SIZE, S_DUR, S_ORDER = range(1, 9)


@dataclass
class Graph:
    """CSR by in-edges: predecessors of v are in_idx[in_ptr[v]:in_ptr[v+1]]."""

    n: int
    in_ptr: np.ndarray  # int32 [n+1]
    in_idx: np.ndarray  # int32 [m]
    size: np.ndarray    # int32 [n]  output size m_v
    dur: np.ndarray     # int32 [n]  duration w_v

    @property
    def m(self) -> int:
        return int(self.in_idx.shape[0])

    def edges(self):
        """List of (u, v) pairs."""
        out = []
        for v in range(self.n):
            for e in range(self.in_ptr[v], self.in_ptr[v + 1]):
                out.append((int(self.in_idx[e]), v))
        return out

    def consumers(self):
        """out[u] = sorted list of v with (u, v) in E."""
        out = [[] for _ in range(self.n)]
        for u, v in self.edges():
            out[u].append(v)
        return out


def graph_from_edges(n, edges, size, dur) -> Graph:
    preds = [[] for _ in range(n)]
    for u, v in edges:
        preds[v].append(u)
    in_ptr = np.zeros(n + 1, dtype=np.int32)
    idx = []
    for v in range(n):
        ps = sorted(preds[v])
        idx.extend(ps)
        in_ptr[v + 1] = len(idx)
    return Graph(n, in_ptr, np.asarray(idx, dtype=np.int32).reshape(-1),
                 np.asarray(size, dtype=np.int32), np.asarray(dur, dtype=np.int32))


def _layers(n, n_layers):
    base, rem = divmod(n, n_layers)
    sizes = [base + (1 if l < rem else 0) for l in range(n_layers)]
    start = [0]
    for s in sizes:
        start.append(start[-1] + s)
    layer_of = []
    for l, s in enumerate(sizes):
        layer_of.extend([l] * s)
    return sizes, start, layer_of


def layered_dag_edges(seed, n, n_layers, dmin, dmax, skew, single_sink, target_m=None):
    """Random layered DAG.

    Node ids run layer by layer.  A node of layer l >= 1 draws an in-degree
    uniformly in [dmin, dmax] and that many distinct predecessors from earlier
    layers: the layer uniformly (skew=False) or at gap g with P proportional to
    2^-g (skew=True), the node uniformly inside the layer.  Nodes left without a
    consumer get one edge to a later node (single_sink: to node n-1).  When
    target_m is given, random legal edges are removed/added until m == target_m.
    """
    sizes, start, layer_of = _layers(n, n_layers)
    edges = set()
    indeg = [0] * n
    outdeg = [0] * n

    def add(u, v):
        edges.add((u, v)); indeg[v] += 1; outdeg[u] += 1

    for v in range(start[1], n):
        lv = layer_of[v]
        d = dmin + hash3(seed, S_DEG, v, 0) % (dmax - dmin + 1)
        d = min(d, start[lv])
        t = 0
        while indeg[v] < d:
            r = hash3(seed, S_PRED, v, t); t += 1
            if skew:
                g, bits = 1, r >> 40
                while (bits & 1) and g < lv:
                    g += 1; bits >>= 1
                l = lv - g
            else:
                l = (r >> 40) % lv
            u = start[l] + (r & 0xFFFFFFFF) % sizes[l]
            if (u, v) not in edges:
                add(u, v)

    last = n_layers - 1
    for u in range(n):
        if outdeg[u]:
            continue
        if single_sink:
            if u != n - 1:
                add(u, n - 1)
            continue
        lu = layer_of[u]
        if lu == last:
            continue
        t = 0
        while True:
            r = hash3(seed, S_ORPHAN, u, t); t += 1
            l = lu + 1 + (r >> 40) % (last - lu)
            v = start[l] + (r & 0xFFFFFFFF) % sizes[l]
            if indeg[v] < dmax or t > 16:
                add(u, v)
                break

    if target_m is not None:
        t = 0
        cand = sorted(edges)
        while len(cand) > target_m:
            r = hash3(seed, S_TRIM, t, 0); t += 1
            i = r % len(cand)
            u, v = cand[i]
            if indeg[v] > 1 and outdeg[u] > 1:
                edges.remove((u, v)); indeg[v] -= 1; outdeg[u] -= 1
                cand[i] = cand[-1]
                cand.pop()
        t = 0
        while len(edges) < target_m:
            r = hash3(seed, S_PAD, t, 0); t += 1
            v = start[1] + (r & 0xFFFFFFFF) % (n - start[1])
            lv = layer_of[v]
            u = (r >> 32) % start[lv]
            if indeg[v] < dmax and (u, v) not in edges:
                add(u, v)
    return sorted(edges)


def training_dag_edges(L):
    """Forward chain f_0..f_{L-1} (ids 0..L-1) with a skip edge every 4 ops and
    the mirrored backward chain b_{L-1}..b_0 (ids L..2L-1 in execution order).
    b_i consumes f_i (its output activation), f_{i-1} (its input activation),
    the previously computed backward op b_{i+1}, and b_{i+4} where the forward
    pass had a skip edge."""
    def f(i): return i
    def b(i): return L + (L - 1 - i)
    edges = set()
    for i in range(1, L):
        edges.add((f(i - 1), f(i)))
        if i % 4 == 0 and i >= 4:
            edges.add((f(i - 4), f(i)))
    for i in range(L - 1, -1, -1):
        edges.add((f(i), b(i)))
        if i >= 1:
            edges.add((f(i - 1), b(i)))
        if i + 1 < L:
            edges.add((b(i + 1), b(i)))
        if i % 4 == 0 and i + 4 < L:
            edges.add((b(i + 4), b(i)))
    return sorted(edges)


def _std_normal(seed, stream, v):
    """Box-Muller on two hash uniforms (host only, float64)."""
    u1 = uniform01(hash3(seed, stream, v, 0))
    u2 = uniform01(hash3(seed, stream, v, 1))
    return math.sqrt(-2.0 * math.log(1.0 - u1)) * math.cos(2.0 * math.pi * u2)


def lognormal_sizes(seed, n, mu, sigma):
    return [max(1, int(round(math.exp(mu + sigma * _std_normal(seed, S_SIZE, v))))) for v in range(n)]


def uniform_ints(seed, stream, n, lo, hi):
    return [lo + hash3(seed, stream, v, 0) % (hi - lo + 1) for v in range(n)]


def proportional_durations(seed, sizes):
    """duration = size * (0.8 + 0.4 u), u uniform, at least 1."""
    return [max(1, int(round(s * (0.8 + 0.4 * uniform01(hash3(seed, S_DUR, v, 0))))))
            for v, s in enumerate(sizes)]


def random_topological_order(seed, g: Graph):
    """Kahn's algorithm; among ready nodes the one with the smallest hash goes
    first, which gives a seeded random topological order."""
    cons = g.consumers()
    missing = [int(g.in_ptr[v + 1] - g.in_ptr[v]) for v in range(g.n)]
    heap = [(hash3(seed, S_ORDER, v, 0), v) for v in range(g.n) if missing[v] == 0]
    heapq.heapify(heap)
    order = []
    while heap:
        _, u = heapq.heappop(heap)
        order.append(u)
        for v in cons[u]:
            missing[v] -= 1
            if missing[v] == 0:
                heapq.heappush(heap, (hash3(seed, S_ORDER, v, 0), v))
    if len(order) != g.n:
        raise ValueError("graph has a cycle")
    return order


def no_remat_peak(g: Graph, order):
    """Peak memory of executing `order` once, every output kept from its compute
    step through the step of its last consumer (a sink: its own step only)."""
    step = [0] * g.n
    for j, v in enumerate(order):
        step[v] = j
    last = list(step)
    for u, v in g.edges():
        last[u] = max(last[u], step[v])
    delta = [0] * (g.n + 1)
    for v in range(g.n):
        delta[step[v]] += int(g.size[v])
        delta[last[v] + 1] -= int(g.size[v])
    peak = cur = 0
    for j in range(g.n):
        cur += delta[j]
        peak = max(peak, cur)
    return peak
