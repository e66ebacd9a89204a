"""Pins of the oracle's greedy descent by cuts (orc_search_cuts): what must hold
of any run, whatever moves it picks -- it is a descent on
(violations, max(peak, M), positions at the peak), max(peak, M) being the
quantity Phase 1 of Section 2.4 of arXiv 2304.14463 minimises; a violation-free start stays violation-free and
still decodes to a valid sequence; every step is the best single cut of the
table that orc_cuts gives for the candidate at that point."""
import numpy as np
import pytest

import oracle

F = {name: i for i, name in enumerate(oracle.FIELDS)}


@pytest.mark.parametrize("cfg", [0, 1])
def test_descent_from_the_plain_schedule(workloads, cfg):
    w = workloads(cfg)
    g, C = w.graph, w.C
    s, e, a = (x.copy() for x in w.base())
    start = oracle.evaluate(g, w.budget, C, s, e, a)[0]
    assert start[F["violations"]] == 0 and start[F["peak"]] > w.budget
    total, fs, fe, fa = oracle.search_cuts(g, w.budget, C, s, e, a, 400)
    assert 0 < total < 400                                  # it stops by itself
    prev = start
    for step in range(1, total + 2):
        # step by step: one call with max_steps = step continues the same path
        k, ts, te, ta = oracle.search_cuts(g, w.budget, C, s, e, a, step)
        assert k == min(step, total)
        now = oracle.evaluate(g, w.budget, C, ts, te, ta)[0]
        if step <= total:
            # the step taken is the first minimum of the table of the candidate before it
            k0, ps, pe, pa = oracle.search_cuts(g, w.budget, C, s, e, a, step - 1)
            table = oracle.cuts(g, w.budget, C, ps, pe, pa, with_at_peak=True)
            ok = np.flatnonzero(table[:, 0] >= 0)
            q = min(ok, key=lambda q: (table[q, 0], table[q, 1], table[q, 3], q))
            assert list(table[q][:3]) == [now[F["violations"]], now[F["peak"]], now[F["duration"]]]
            assert now[F["violations"]] == 0
            # a descent: the peak falls, or it stays and fewer positions reach it
            _, prof_prev = oracle.profile(g, w.budget, C, ps, pe, pa)
            _, prof_now = oracle.profile(g, w.budget, C, ts, te, ta)
            assert prev[F["peak"]] > w.budget
            assert now[F["peak"]] < prev[F["peak"]] or (
                now[F["peak"]] == prev[F["peak"]] and
                (prof_now >= prev[F["peak"]]).sum() < (prof_prev >= prev[F["peak"]]).sum())
            assert table[q][3] == (prof_now >= prev[F["peak"]]).sum()
            assert now[F["duration"]] > prev[F["duration"]]
            assert int(ta.sum()) == int(a.sum()) + step
            d, _ = oracle.decode(g, C, ts, ta)
            assert d[0][0] == 1 and d[0][1] == w.n + step and d[0][2] <= now[F["peak"]]
            assert d[0][3] == now[F["duration"]]
            prev = now
        else:
            assert (ts == fs).all() and (te == fe).all() and (ta == fa).all()
    # where it stops, it is under the budget or no violation-free cut lowers the peak or the
    # number of positions that reach it
    table = oracle.cuts(g, w.budget, C, fs, fe, fa, with_at_peak=True)
    ok = table[:, 0] == 0
    _, prof = oracle.profile(g, w.budget, C, fs, fe, fa)
    if prev[F["peak"]] > w.budget:
        assert not (table[ok, 1] < prev[F["peak"]]).any()
        assert not (table[ok, 3] < (prof >= prev[F["peak"]]).sum()).any()


def test_nothing_to_do():
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(3, [(0, 1), (1, 2)], [4, 4, 4], [1, 1, 1])
    s, e, a = [0, 0, 2, 0, 4, 0], [2, 0, 4, 0, 4, 0], [1, 0, 1, 0, 1, 0]
    # a chain gains nothing from recomputation (Section 1.1): every cut leaves the peak at 8
    k, s2, e2, a2 = oracle.search_cuts(g, 5, 2, s, e, a, 10)
    assert k == 0 and list(s2) == s and list(e2) == e and list(a2) == a
    # under the budget already: max(peak, M) cannot fall
    assert oracle.search_cuts(g, 100, 2, s, e, a, 10)[0] == 0
    assert oracle.search_cuts(g, 5, 2, s, e, a, 0)[0] == 0
