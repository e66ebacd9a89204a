"""Pins of the two moves the two-phase descent adds to the oracle, and of the descent itself.

Phase 1 of Section 2.4 of arXiv 2304.14463 minimises max(peak, M), Phase 2 minimises the
duration, Eq. (1), from a solution within the budget.  The moves are this library's:
  * the cut that keeps the producer's inputs (oracle cut mode 1): as the plain cut, but the
    recomputation goes to the last free position before the use, and every input of the producer
    that is gone by then is kept until there instead;
  * the merge: a recomputation is undone, its output held across the gap instead.
Both are scored by full evaluation through the pinned evaluator; what is pinned here is which
copies and positions they touch (hand-counted cases) and what any such move must do to the
memory profile, the duration and the decoded sequence (separate code: profile, decoder).
"""
import numpy as np
import pytest

import oracle
from paper_2304_14463_amd.inputs import graph_from_edges
from test_oracle_cuts import edge_index

F = {name: i for i, name in enumerate(oracle.FIELDS)}


def waits_case():
    """Node 2 needs nodes 0 and 1; node 3 uses node 2 late; node 1 (small) is dropped early."""
    g = graph_from_edges(4, [(0, 2), (1, 2), (2, 3)], [1, 1, 6, 1], [1, 1, 5, 1])
    #             0a 0b 1a 1b 2a 2b 3a 3b
    s = np.array([0, 0, 2, 0, 3, 0, 7, 0], np.int32)
    e = np.array([7, 0, 4, 0, 7, 0, 7, 0], np.int32)
    a = np.array([1, 0, 1, 0, 1, 0, 1, 0], np.uint8)
    return g, 2, s, e, a


def test_keeping_cut_by_hand():
    g, C, s, e, a = waits_case()
    x = edge_index(g, 2, 3)
    # plain cut: waits at position 4 where node 1 is still held (pinned elsewhere); keeping cut:
    # the last free position before 7 is 6; node 0 is held there, node 1 ([2,4]) is kept until 6
    ok, s2, e2, a2 = oracle.cut_apply(g, C, s, e, a, x, 0, mode=1)
    assert ok
    assert (s2[5], e2[5], a2[5]) == (6, 7, 1) and e2[4] == 3            # node 2: [3,3] and [6,7]
    assert e2[2] == 6 and (np.delete(e2, [2, 4, 5]) == np.delete(e, [2, 4, 5])).all()
    assert (np.delete(s2, 5) == np.delete(s, 5)).all() and (np.delete(a2, 5) == np.delete(a, 5)).all()
    # memory before: 1, 1, 2, 8, 8, 7, 7, 8; after: node 2 gone on 4..5, node 1 added on 5..6
    base, prof0 = oracle.profile(g, 100, C, s, e, a)
    res, prof1 = oracle.profile(g, 100, C, s2, e2, a2)
    assert list(prof0) == [1, 1, 2, 8, 8, 7, 7, 8]
    assert list(prof1) == [1, 1, 2, 8, 2, 2, 8, 8]
    assert list(oracle.cuts(g, 100, C, s, e, a, mode=1)[x * C]) == [0, 8, 8 + 5]
    # all inputs held at the last free position: the two kinds of cut are the same move
    e_all = e.copy(); e_all[2] = 7
    for arrs in zip(oracle.cut_apply(g, C, s, e_all, a, x, 0, mode=0), oracle.cut_apply(g, C, s, e_all, a, x, 0, mode=1)):
        assert np.array_equal(*arrs)
    # an input that was never computed before the position cannot be kept: look further down.
    # node 1 computed at 5 only: at 6 it is held ([5,7]); make it [5,5]: kept from 5 until 6
    s3, e3 = s.copy(), e.copy(); s3[2], e3[2] = 5, 5
    ok, s4, e4, a4 = oracle.cut_apply(g, C, s3, e3, a, x, 0, mode=1)
    assert ok and (s4[5], e4[2]) == (6, 6)
    # node 1 computed at 6 itself (taken) and never before: positions 5 and 4 have no copy of node 1
    # to keep; nothing applies
    s3[2], e3[2] = 6, 7
    assert not oracle.cut_apply(g, C, s3, e3, a, x, 0, mode=1)[0]
    # two copies of an input end before the position: the later end is kept (the higher index among equals)
    g3 = graph_from_edges(4, [(0, 2), (1, 2), (2, 3)], [1, 1, 6, 1], [1, 1, 5, 1])
    s5 = np.array([0, 0, 0, 1, 2, 0, 3, 0, 0, 9, 0, 0], np.int32)     # C = 3; node 1 at 1 and 2
    e5 = np.array([9, 0, 0, 1, 4, 0, 9, 0, 0, 9, 0, 0], np.int32)
    a5 = np.array([1, 0, 0, 1, 1, 0, 1, 0, 0, 1, 0, 0], np.uint8)
    ok, s6, e6, a6 = oracle.cut_apply(g3, 3, s5, e5, a5, edge_index(g3, 2, 3), 0, mode=1)
    assert ok and (s6[7], e6[7], a6[7]) == (8, 9, 1) and e6[4] == 8 and e6[3] == 1 and e6[6] == 3


@pytest.mark.parametrize("cfg", [0, 1])
def test_what_every_keeping_cut_must_satisfy(workloads, cfg):
    """On workload candidates: the memory falls by m_u strictly between the cut copy's new end
    and the recomputation, rises by m_w from behind the old end of every kept input up to the
    recomputation, and changes nowhere else; the duration grows by w_u; no precedence is lost;
    a violation-free result decodes to the base's sequence with u inserted."""
    w = workloads(cfg)
    g, C, T = w.graph, w.C, w.T
    ss, ee, aa = w.candidates(0, 24)
    ev = oracle.evaluate(g, w.budget, C, ss, ee, aa)
    rows = [b for b in range(24) if ev[b, F["violations"]] == 0][:3] + [b for b in range(24) if ev[b, F["violations"]]][:2]
    m = int(g.in_ptr[-1])
    consumer = np.repeat(np.arange(g.n), np.diff(g.in_ptr))
    applicable = kept_something = differs = 0
    for b in rows:
        s, e, a = ss[b], ee[b], aa[b]
        base, prof0 = oracle.profile(g, w.budget, C, s, e, a)
        sc = oracle.cuts(g, w.budget, C, s, e, a, mode=1)
        sc0 = oracle.cuts(g, w.budget, C, s, e, a, mode=0)
        assert ((sc0[:, 0] >= 0) <= (sc[:, 0] >= 0)).all()          # wherever the plain cut applies, so does this one
        differs += int((sc != sc0).any())
        for q in np.flatnonzero(sc[:, 0] >= 0)[::max(1, m * C // 150)]:
            x, i = divmod(int(q), C)
            u, v = int(g.in_idx[x]), int(consumer[x])
            ok, s2, e2, a2 = oracle.cut_apply(g, C, s, e, a, x, i, mode=1)
            assert ok
            j = int(np.flatnonzero(a2 != a)[0])
            assert j // C == u and (s2 != s).sum() == 1 and s2[j] < s[v * C + i]
            p = int(s2[j])
            res, prof1 = oracle.profile(g, w.budget, C, s2, e2, a2)
            assert list(res[:3]) == list(sc[q][[1, 2, 0]])
            assert res[F["duration"]] == base[F["duration"]] + g.dur[u]
            want = prof0.copy()
            preds = set(int(y) for y in g.in_idx[g.in_ptr[u]:g.in_ptr[u + 1]])
            for c in np.flatnonzero(e2 != e):
                if c == j:
                    continue
                if c // C == u:                                      # the copy that was cut
                    assert e2[c] < e[c]
                    want[e2[c] + 1:p] -= g.size[u]
                else:                                                # an input kept until p
                    assert c // C in preds and e2[c] == p and e[c] < p and a[c]
                    want[e[c] + 1:p + 1] += g.size[c // C]
                    kept_something += 1
            assert (prof1 == want).all()
            assert res[F["v_prec"]] <= base[F["v_prec"]] and res[F["v_start"]] == base[F["v_start"]]
            assert res[F["v_form"]] == base[F["v_form"]]
            applicable += 1
            if base[F["violations"]] == 0:
                assert res[F["violations"]] == 0
                d0, seq0 = oracle.decode(g, C, s, a)
                d1, seq1 = oracle.decode(g, C, s2, a2)
                assert d1[0][0] == 1 and d1[0][1] == d0[0][1] + 1 and d1[0][2] <= res[F["peak"]]
                step = int((np.sort(s[a != 0]) < p).sum())
                assert list(seq1[0][:step]) == list(seq0[0][:step]) and seq1[0][step] == u
                assert list(seq1[0][step + 1:d1[0][1]]) == list(seq0[0][step:d0[0][1]])
    assert applicable > 100 and kept_something > 10 and differs > 0


def test_merge_by_hand():
    """Node 0 feeds node 1 (position 1) and node 2 (position 5); it is computed at 0 and again at
    4.  Merging the second computation into the first: [0,1] and [4,5] become [0,5]."""
    g = graph_from_edges(3, [(0, 1), (0, 2), (1, 2)], [7, 2, 3], [11, 1, 1])
    C, T = 2, 6
    s = np.array([0, 4, 1, 0, 5, 0], np.int32)
    e = np.array([1, 5, 5, 0, 5, 0], np.int32)
    a = np.array([1, 1, 1, 0, 1, 0], np.uint8)
    base, prof = oracle.profile(g, 100, C, s, e, a)
    assert (base[F["violations"]], base[F["peak"]], base[F["duration"]]) == (0, 12, 24) and list(prof) == [7, 9, 2, 2, 9, 12]
    picks, S, E, A = oracle.merge_candidates(C, s, e, a, T, 8)
    assert list(picks) == [1]                       # the only copy with an earlier live copy of its node
    assert list(S[0]) == list(s) and list(E[0]) == [5, 5, 5, 0, 5, 0] and list(A[0]) == [1, 0, 1, 0, 1, 0]
    r, prof2 = oracle.profile(g, 100, C, S[0], E[0], A[0])
    assert (r[F["violations"]], r[F["peak"]], r[F["duration"]]) == (0, 12, 13) and list(prof2) == [7, 9, 9, 9, 9, 12]
    # within a budget of 12 the merge is taken; a second step finds nothing to merge
    k, s2, e2, a2 = oracle.search_merges(g, 12, C, s, e, a, 5, 8)
    assert k == 1 and list(e2) == [5, 5, 5, 0, 5, 0] and list(a2) == [1, 0, 1, 0, 1, 0]
    # if the gap holds a position that the held output lifts over the budget, the merge is not taken
    g2 = graph_from_edges(4, [(0, 1), (0, 2), (1, 2), (1, 3)], [7, 2, 3, 4], [11, 1, 1, 1])
    s = np.array([0, 4, 1, 0, 5, 0, 3, 0], np.int32)
    e = np.array([1, 5, 5, 0, 5, 0, 3, 0], np.int32)
    a = np.array([1, 1, 1, 0, 1, 0, 1, 0], np.uint8)
    base, prof = oracle.profile(g2, 12, C, s, e, a, T=8)
    assert list(prof[:6]) == [7, 9, 2, 6, 9, 12] and base[F["feasible"]] == 1
    k, s2, e2, a2 = oracle.search_merges(g2, 12, C, s, e, a, 5, 8)     # merged: 7, 9, 9, 13, 9, 12
    assert k == 0 and list(a2) == list(a)
    assert oracle.search_merges(g2, 13, C, s, e, a, 5, 8)[0] == 1
    # the earlier copy may already reach further than the later one: its end stays
    picks, S, E, A = oracle.merge_candidates(2, [0, 2, 1, 0], [5, 3, 1, 0], [1, 1, 1, 0], 4 * 2, 8)
    assert list(picks) == [1] and list(E[0]) == [5, 3, 1, 0] and list(A[0]) == [1, 0, 1, 0]
    # three copies: the third merges into the second, the second into the first; K caps the list
    picks, S, E, A = oracle.merge_candidates(3, [0, 2, 4], [1, 3, 5], [1, 1, 1], 6, 8)
    assert list(picks) == [1, 2] and list(E[0]) == [3, 3, 5] and list(E[1]) == [1, 5, 5]
    assert list(A[0]) == [1, 0, 1] and list(A[1]) == [1, 1, 0]
    assert list(oracle.merge_candidates(3, [0, 2, 4], [1, 3, 5], [1, 1, 1], 6, 1)[0]) == [1]


@pytest.mark.parametrize("cfg", [0, 1])
def test_two_phase_descent_properties(workloads, cfg):
    """From the plain schedule: Phase 1 ends within the budget on the n = 442 workload; every
    merge of Phase 2 keeps the candidate feasible and saves exactly one node's duration; where
    it stops no merge is feasible; the result decodes to a valid sequence of the same duration."""
    w = workloads(cfg)
    g, C = w.graph, w.C
    s, e, a = (x.copy() for x in w.base())
    k1, s1, e1, a1 = oracle.search_cuts(g, w.budget, C, s, e, a, 300, mode=1)
    r1 = oracle.evaluate(g, w.budget, C, s1, e1, a1)[0]
    assert r1[F["violations"]] == 0 and 0 < k1 < 300
    if cfg == 1:
        assert r1[F["feasible"]] == 1                         # the plain cut stops at 12424 > 11200 here
        assert oracle.evaluate(g, w.budget, C, *oracle.search_cuts(g, w.budget, C, s, e, a, 300, mode=0)[1:])[0][F["feasible"]] == 0
    budget = w.budget if r1[F["feasible"]] else int(r1[F["peak"]])     # cfg 0 stops above its budget: use what it reached
    k1, s1, e1, a1 = oracle.search_cuts(g, budget, C, s, e, a, 300, mode=1)
    k1b, k2, s2, e2, a2 = oracle.search_two_phase(g, budget, C, s, e, a, 300, 300, 64)
    assert k1b == k1
    prev = oracle.evaluate(g, budget, C, s1, e1, a1)[0]
    assert prev[F["feasible"]] == 1
    for step in range(1, k2 + 1):
        k, ts, te, ta = oracle.search_merges(g, budget, C, s1, e1, a1, step, 64)
        now = oracle.evaluate(g, budget, C, ts, te, ta)[0]
        assert k == step and now[F["feasible"]] == 1
        saved = prev[F["duration"]] - now[F["duration"]]
        assert saved > 0 and saved in set(int(x) for x in g.dur)
        prev = now
    assert k2 > 0 or cfg == 0
    picks, S, E, A = oracle.merge_candidates(C, s2, e2, a2, w.T, 64)
    if len(picks):
        assert (oracle.evaluate(g, budget, C, S, E, A)[:, F["feasible"]] == 0).all()
    final = oracle.evaluate(g, budget, C, s2, e2, a2)[0]
    d, _ = oracle.decode(g, C, s2, a2)
    assert d[0][0] == 1 and d[0][3] == final[F["duration"]] and d[0][2] <= final[F["peak"]]
    assert final[F["duration"]] == int(g.dur.sum()) + sum(int(g.dur[k // C]) for k in np.flatnonzero(a2) if k % C)
