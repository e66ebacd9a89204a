"""Oracle evaluator vs brute force over rematerialisation sequences.

The sequence side (oracle/moc_bruteforce.cpp) works on the problem as stated
in Section 1 of arXiv 2304.14463 -- an ordered list of nodes, inputs must be in
memory, footprint by liveness -- and never looks at intervals; the evaluator
works on Eq. (1)-(8).  The two must agree through the correspondence
"event = index in the sequence" (Section 2, compute events).
"""
import numpy as np
import pytest

import oracle
from paper_2304_14463_amd.inputs import graph_from_edges
from paper_2304_14463_amd.inputs.hashrng import hash3

F = {name: i for i, name in enumerate(oracle.FIELDS)}


def tiny_dag(n, seed, density=3):
    """Seeded random DAG on n nodes (ids topological), sizes/durations small and distinct-ish."""
    edges = set()
    for v in range(1, n):
        for t in range(density):
            r = hash3(seed, v, t, 0)
            if t == 0 or (r >> 8) % 3 == 0:
                edges.add((r % v, v))
    size = [1 + hash3(seed, 100, v, 0) % 9 for v in range(n)]
    dur = [1 + hash3(seed, 200, v, 0) % 7 for v in range(n)]
    return graph_from_edges(n, sorted(edges), size, dur)


DIAMOND = [(0, 1), (0, 2), (1, 3), (2, 3)]
PAPER4 = [(0, 1), (1, 2), (2, 3), (0, 3)]


@pytest.mark.parametrize("case", [
    ("paper4", 4, PAPER4, 2, 4), ("diamond", 4, DIAMOND, 2, 4), ("diamond-C3", 4, DIAMOND, 3, 3),
    ("seed5a", 5, None, 2, 5), ("seed5b", 5, None, 2, 5), ("seed6", 6, None, 2, 3),
    ("seed7", 7, None, 2, 2), ("seed8", 8, None, 2, 2), ("seed6-C3", 6, None, 3, 2),
])
def test_sequences_evaluate_to_their_simulation(case):
    name, n, edges, C, max_extra = case
    if edges is None:
        g = tiny_dag(n, sum(map(ord, name)))
    else:
        g = graph_from_edges(n, edges, [3, 5, 2, 7][:n], [2, 3, 5, 7][:n])
    en = oracle.enumerate_sequences(g, C, max_extra)
    assert en["count"] > 100
    res = oracle.evaluate(g, 10**9, C, en["starts"], en["ends"], en["active"])
    bad = np.flatnonzero((res[:, F["violations"]] != 0) | (res[:, F["peak"]] != en["peak"]) |
                         (res[:, F["duration"]] != en["duration"]))
    assert bad.size == 0, (name, en["seqs"][bad[:3]], res[bad[:3]], en["peak"][bad[:3]])
    # budget feasibility follows the simulated peak
    for budget in (int(en["peak"].min()), int(np.median(en["peak"])), int(en["peak"].min()) - 1):
        res = oracle.evaluate(g, budget, C, en["starts"], en["ends"], en["active"])
        assert (res[:, F["feasible"]] == (en["peak"] <= budget)).all()


def test_shrinking_a_served_interval_is_caught():
    """Cutting one unit off any interval that serves a later use must break
    exactly the uses it no longer covers."""
    g = graph_from_edges(4, PAPER4, [1, 1, 1, 1], [1, 1, 1, 1])
    en = oracle.enumerate_sequences(g, 2, 4)
    checked = 0
    for b in range(0, en["count"], 17):
        s, e, a = en["starts"][b].copy(), en["ends"][b].copy(), en["active"][b]
        for k in range(8):
            if a[k] and e[k] > s[k]:
                e2 = e.copy(); e2[k] -= 1
                r = oracle.evaluate(g, 10**9, 2, s, e2, a)[0]
                # the canonical end is a use: at least that one is now uncovered
                assert r[F["v_prec"]] >= 1 and r[F["violations"]] == r[F["v_prec"]]
                checked += 1
    assert checked > 50


def test_path_graph_gains_nothing():
    """Section 1.1: on a line graph rematerialisation cannot lower the
    footprint below max over edges of m_u + m_v."""
    sizes = [4, 9, 2, 7, 5]
    g = graph_from_edges(5, [(i, i + 1) for i in range(4)], sizes, [1] * 5)
    en = oracle.enumerate_sequences(g, 2, 5)
    res = oracle.evaluate(g, 10**9, 2, en["starts"], en["ends"], en["active"])
    bound = max(sizes[i] + sizes[i + 1] for i in range(4))
    assert (res[:, F["violations"]] == 0).all()
    assert res[:, F["peak"]].min() == bound


@pytest.mark.parametrize("edges", [[(0, 1), (1, 2), (0, 2)], [(0, 1), (0, 2)]])
def test_every_assignment_on_three_nodes(edges):
    """All 9.9e7 assignments with C = 2 on a 3-node DAG: every violation-free
    one decodes to a valid sequence of the same duration whose footprint is not
    above the assignment's peak; and per set of recomputed nodes the best
    assignment reaches exactly the best sequence's footprint."""
    g = graph_from_edges(3, edges, [3, 5, 2], [2, 3, 5])
    counts, min_peak = oracle.exhaustive_c2(g, n_threads=8)
    assert counts[0] == (21 * 22) ** 3
    assert counts[1] > 0 and counts[2] == 0
    en = oracle.enumerate_sequences(g, 2, 3)
    best = {}
    for b in range(en["count"]):
        mask = sum(1 << v for v in range(3) if en["active"][b][2 * v + 1])
        best[mask] = min(best.get(mask, 10**9), int(en["peak"][b]))
    for mask in range(8):
        assert min_peak[mask] == best.get(mask, -1), (mask, min_peak, best)
