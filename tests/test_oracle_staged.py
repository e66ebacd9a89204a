"""Pins of the oracle's evaluator in the stage-restricted domain (Section 2.3 of arXiv
2304.14463: n(n+1)/2 events in n stages, node with place k in the topological order only at
event k of a stage, its first interval at event k of stage k).

What fixes it from outside: the worked example of Section 2, whose printed events (1, 3, 7, 10)
are events of this layout; the plain evaluator (pinned on its own) after the live start events
have been renumbered by rank, which changes nothing by the argument of Section 2.2 (memory
cannot rise at an event where nothing starts); the liveness peak of a plain schedule; the
enumerator of rematerialisation sequences with its own simulation; hand-counted cases for what
the restriction adds.
"""
import numpy as np
import pytest

import oracle
from paper_2304_14463_amd.inputs import graph_from_edges
from paper_2304_14463_amd.inputs.staged import gen_staged_candidates, slot_position, staged_base, staged_tables
from test_oracle_pins import read_golden, worked_example
from test_oracle_bruteforce import tiny_dag

F = {name: i for i, name in enumerate(oracle.FIELDS)}
COUNTS = ("v_form", "v_first", "v_order", "v_start", "v_prec")


def counts(r):
    return tuple(int(r[F[k]]) for k in COUNTS)


# ---------------------------------------------------------------- worked example, as printed
def test_worked_example_is_a_staged_schedule():
    """Events 1, 3, 6, 10 are the last events of stages 1..4 (k(k+1)/2): the fixed first starts
    of nodes 1..4; event 7 is the first event of stage 4: node 1's slot.  Evaluated verbatim on
    the 10 events of the drawing."""
    kv, g, C, T, s, e, a = worked_example([1, 1, 1, 1], [3, 5, 7, 11])
    assert T == 4 * 5 // 2
    index = np.arange(4)
    r = oracle.evaluate_staged(g, 3, C, index, s, e, a)[0]
    assert counts(r) == (0, 0, 0, 0, 0)
    assert r[F["peak"]] == int(kv["peak.unit_sizes"]) and r[F["feasible"]] == 1
    assert r[F["duration"]] == 2 * 3 + 5 + 7 + 11
    assert list(r) == list(oracle.evaluate(g, 3, C, s, e, a, T=T)[0])     # the restriction is met: nothing added
    # the first starts are where Section 2.3 fixes them: j(j+1)/2 for the j-th node, 1-based
    assert [int(s[v * C]) + 1 for v in range(4)] == [j * (j + 1) // 2 for j in (1, 2, 3, 4)]
    # node 1 recomputed at event 8 instead of 7: event 8 is node 2's slot of stage 4, not node 1's.
    # The copy is outside its domain: one violation for it, and node 4 loses its input
    s2 = s.copy(); s2[1] = 7
    r = oracle.evaluate_staged(g, 3, C, index, s2, e, a)[0]
    assert counts(r) == (1, 0, 0, 0, 1) and r[F["duration"]] == 2 * 3 + 5 + 7 + 11
    assert r[F["peak"]] == 2                                     # profile without that copy: never more than two outputs
    # the plain evaluator has no such restriction
    assert oracle.evaluate(g, 3, C, s2, e, a, T=T)[0][F["violations"]] == 0
    # node 1 recomputed in stage 3 (event 4 = its slot there): allowed, but then it must be kept to event 10
    s3 = s.copy(); s3[1] = 3
    r = oracle.evaluate_staged(g, 3, C, index, s3, e, a)[0]
    assert counts(r) == (0, 0, 0, 0, 0) and r[F["peak"]] == 3
    # node 2's first interval moved to its slot of stage 3 (event 5): on a slot, but the first start is fixed
    s4, e4 = s.copy(), e.copy(); s4[2] = 4
    r = oracle.evaluate_staged(g, 3, C, index, s4, e4, a)[0]
    assert r[F["v_form"]] == 1 and r[F["v_prec"]] == 1 and r[F["v_first"]] == 0   # node 3 loses node 2


def test_hand_counted_cases():
    """Chain 0 -> 1 -> 2 in the order 0, 1, 2.  Stages: {0}, {1, 2}, {3, 4, 5}; fixed first starts
    0, 2, 5; node 0 may be recomputed at 1 or 3, node 1 at 4."""
    g = graph_from_edges(3, [(0, 1), (1, 2)], [10, 20, 40], [1, 2, 4])
    C = 2
    index = np.array([0, 1, 2])
    s = np.array([0, 0, 2, 0, 5, 0], np.int32)
    e = np.array([2, 0, 5, 0, 5, 0], np.int32)
    a = np.array([1, 0, 1, 0, 1, 0], np.uint8)
    r = oracle.evaluate_staged(g, 100, C, index, s, e, a)[0]
    # memory by position: 10, 10, 30, 20, 20, 60
    assert counts(r) == (0, 0, 0, 0, 0) and r[F["peak"]] == 60 and r[F["duration"]] == 7 and r[F["feasible"]] == 1
    assert oracle.evaluate_staged(g, 59, C, index, s, e, a)[0][F["feasible"]] == 0
    # a second copy of node 1 on its slot of stage 2 (position 4), first copy cut to [2,2]:
    # at position 4 node 0 (kept on [0,2]) is gone -> one uncovered input; memory 10, 10, 30, 0, 20, 60
    s2, e2, a2 = s.copy(), e.copy(), a.copy()
    e2[2] = 2; s2[3], e2[3], a2[3] = 4, 5, 1
    r = oracle.evaluate_staged(g, 100, C, index, s2, e2, a2)[0]
    assert counts(r) == (0, 0, 0, 0, 1) and r[F["peak"]] == 60 and r[F["duration"]] == 9
    # with node 0 kept through position 4 it is clean: memory 10, 10, 30, 10, 30, 60
    e3 = e2.copy(); e3[0] = 4
    r = oracle.evaluate_staged(g, 100, C, index, s2, e3, a2)[0]
    assert counts(r) == (0, 0, 0, 0, 0) and r[F["peak"]] == 60
    # the same second copy one position earlier: 3 is node 0's slot of stage 2, not node 1's.  It is
    # outside its domain (one violation, still paid for) and serves nobody: node 2 at 5 finds node 1
    # kept on [2,2] only.  Memory 10, 10, 30, 10, 10, 40
    s4 = s2.copy(); s4[3] = 3
    r = oracle.evaluate_staged(g, 100, C, index, s4, e3, a2)[0]
    assert counts(r) == (1, 0, 0, 0, 1) and r[F["peak"]] == 40 and r[F["duration"]] == 9
    # a first interval anywhere but its fixed start is outside its domain, also on the node's own slot
    # of a later stage (node 1 at 4): Eq. (7) is about the flag and stays satisfied
    s5 = s.copy(); s5[2] = 4
    r = oracle.evaluate_staged(g, 100, C, index, s5, e, a)[0]
    assert counts(r) == (1, 0, 0, 0, 1) and r[F["peak"]] == 40   # node 2 unserved; memory 10, 10, 10, 0, 0, 40
    # two copies of one node on one event: [2,2] and [2,5] satisfy Eq. (2) and Eq. (3), not Eq. (6)
    s6, e6, a6 = s.copy(), e.copy(), a.copy()
    e6[2] = 2; s6[3], e6[3], a6[3] = 2, 5, 1
    r = oracle.evaluate_staged(g, 100, C, index, s6, e6, a6)[0]
    assert counts(r) == (0, 0, 0, 1, 0) and r[F["peak"]] == 60 and r[F["duration"]] == 9   # 10, 10, 50, 20, 20, 60
    # ends are not restricted to slots, only to the domain
    e7 = e.copy(); e7[4] = 6
    assert counts(oracle.evaluate_staged(g, 100, C, index, s, e7, a)[0]) == (1, 0, 0, 0, 0)
    # another order of the same graph is another restriction: with places 0, 1, 2 -> the nodes are
    # their own places; give node 2 the place of node 1 and the schedule above is outside the domain
    # everywhere except at node 0
    r = oracle.evaluate_staged(g, 100, C, np.array([0, 2, 1]), s, e, a)[0]
    assert r[F["v_form"]] == 2


# ---------------------------------------------------------------- plain schedules
@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_plain_schedule_in_the_stage_layout(workloads, cfg):
    """Section 2.4: a topological order is a violation-free solution; in the stage layout every
    node sits at its fixed start.  Its peak is the liveness peak of the order (the generator's own
    simulation), its duration the sum of all durations."""
    w = workloads(cfg)
    index, out_ptr, cons_idx, _, _ = staged_tables(w.graph, w.order)
    s, e, a = staged_base(w.n, w.C, index, out_ptr, cons_idx)
    r = oracle.evaluate_staged(w.graph, w.budget, w.C, index, s, e, a)[0]
    assert counts(r) == (0, 0, 0, 0, 0)
    assert r[F["peak"]] == w.no_remat_peak and r[F["duration"]] == int(w.graph.dur.sum())
    # the first starts are k(k+1)/2 + k for place k
    for v in range(0, w.n, max(1, w.n // 40)):
        k = int(index[v])
        assert s[v * w.C] == k * (k + 1) // 2 + k == slot_position(k, k)


# ---------------------------------------------------------------- against the plain evaluator
def compress(n, C, D, index, s, e, a):
    """Renumber positions by the rank of the live start events, written here from scratch: a start
    at the r-th distinct live start position becomes 2r, an end becomes 2r for r = the last start
    position not after it, plus 1 if it lies strictly after that start.  Every comparison between a
    start and a start or an end keeps its outcome, and so does the memory at every start event.
    Copies that are active but not usable (ill formed or outside their domain) are made ill
    formed, which the plain evaluator counts the same way."""
    K = n * C
    usable = np.zeros(K, bool)
    for v in range(n):
        for i in range(C):
            k = v * C + i
            if a[k] == 0 or not (0 <= s[k] <= e[k] <= D - 1):
                continue
            j = int((np.sqrt(8.0 * s[k] + 1) - 1) // 2)
            while j * (j + 1) // 2 > s[k]:
                j -= 1
            while (j + 1) * (j + 2) // 2 <= s[k]:
                j += 1
            slot = s[k] - j * (j + 1) // 2
            usable[k] = slot == index[v] and (i > 0 or j == index[v])
    events = np.unique(s[usable])
    s2, e2 = np.zeros(K, np.int32), np.zeros(K, np.int32)
    for k in range(K):
        if usable[k]:
            s2[k] = 2 * np.searchsorted(events, s[k])
            r = np.searchsorted(events, e[k], side="right") - 1
            e2[k] = 2 * r + (1 if e[k] > events[r] else 0)
        elif a[k]:
            s2[k], e2[k] = 1, 0
    return s2, e2, max(2 * len(events), 1)


@pytest.mark.parametrize("cfg", [0, 1])
def test_equals_the_plain_evaluator_on_rank_compressed_events(workloads, cfg):
    w = workloads(cfg)
    tables = staged_tables(w.graph, w.order)
    index = tables[0]
    D = w.n * (w.n + 1) // 2
    B = 96 if cfg == 0 else 40
    S, E, A = gen_staged_candidates(w.seed, w.graph, w.order, w.C, B, 0, B, tables)
    got = oracle.evaluate_staged(w.graph, w.budget, w.C, index, S, E, A)
    kinds = set()
    for b in range(B):
        s2, e2, T2 = compress(w.n, w.C, D, index, S[b], E[b], A[b])
        want = oracle.evaluate(w.graph, w.budget, w.C, s2, e2, A[b], T=T2)[0]
        assert list(got[b]) == list(want), b
        kinds.add(tuple(x > 0 for x in counts(got[b])))
    assert (got[: B // 2, F["violations"]] == 0).all()              # type A: clean by construction
    assert len(kinds) >= 3                                          # the perturbed half breaks several kinds of constraint
    assert (got[B // 2:, F["v_form"]] > 0).any() and (got[B // 2:, F["v_prec"]] > 0).any()


def test_random_garbage_against_the_plain_evaluator():
    """Arbitrary values (starts on and off slots, ends anywhere, flags at random), small graph."""
    rng = np.random.default_rng(8)
    n, C = 7, 3
    g = tiny_dag(n, 31)
    D = n * (n + 1) // 2
    order = rng.permutation(n)          # need not even be topological for the arithmetic to be defined
    index = np.argsort(order)
    for trial in range(200):
        s = rng.integers(-2, D + 2, n * C).astype(np.int32)
        on_slot = rng.random(n * C) < 0.7
        for v in range(n):
            for i in range(C):
                if on_slot[v * C + i]:
                    j = int(rng.integers(index[v], n))
                    s[v * C + i] = slot_position(j if i else int(index[v]), int(index[v]))
        e = (s + rng.integers(-1, D // 2, n * C)).astype(np.int32)
        a = (rng.random(n * C) < 0.7).astype(np.uint8)
        got = oracle.evaluate_staged(g, 20, C, index, s, e, a)[0]
        s2, e2, T2 = compress(n, C, D, index, s, e, a)
        want = oracle.evaluate(g, 20, C, s2, e2, a, T=T2)[0]
        assert list(got) == list(want), trial


# ---------------------------------------------------------------- against enumerated sequences
def staged_form(seq, n, C, ends_in_seq):
    """A rematerialisation sequence over nodes 0..n-1 (ids = places) that fits the stages -- first
    computations in the order 0, 1, .., and between the first computations of j-1 and j only
    recomputations of earlier nodes in increasing order -- as a candidate of the stage layout:
    position of every step, and each end moved to the position of the step it pointed at."""
    pos, stage, last = [], 0, -1
    seen = set()
    for v in seq:
        if v not in seen:
            if v != stage:
                return None
            pos.append(slot_position(stage, v))
            seen.add(v)
            stage, last = stage + 1, -1
        else:
            if stage >= n or v <= last:
                return None
            pos.append(slot_position(stage, v))
            last = v
    s = np.zeros(n * C, np.int32)
    e = np.zeros(n * C, np.int32)
    a = np.zeros(n * C, np.uint8)
    copy = [0] * n
    for step, v in enumerate(seq):
        k = v * C + copy[v]
        copy[v] += 1
        s[k], e[k], a[k] = pos[step], pos[ends_in_seq[step]], 1
    return s, e, a


@pytest.mark.parametrize("n,C,max_extra,seed", [(4, 2, 4, 0), (5, 2, 4, 77), (6, 2, 3, 78), (5, 3, 4, 79)])
def test_stage_compatible_sequences_evaluate_to_their_simulation(n, C, max_extra, seed):
    """Every enumerated sequence that fits the stages, placed on its events, has no violation,
    the peak of the enumerator's liveness simulation and its duration."""
    g = graph_from_edges(4, [(0, 1), (1, 2), (2, 3), (0, 3)], [3, 5, 2, 7], [2, 3, 5, 7]) if seed == 0 else tiny_dag(n, seed)
    en = oracle.enumerate_sequences(g, C, max_extra)
    index = np.arange(n)
    fitted = 0
    for q in range(en["count"]):
        L = int(en["seq_len"][q])
        seq = [int(x) for x in en["seqs"][q][:L]]
        # the canonical candidate's ends are indices into the sequence: copy order = order of occurrence
        copy, ends = [0] * n, []
        for v in seq:
            ends.append(int(en["ends"][q][v * C + copy[v]]))
            copy[v] += 1
        cand = staged_form(seq, n, C, ends)
        if cand is None:
            continue
        fitted += 1
        r = oracle.evaluate_staged(g, 10**9, C, index, *cand)[0]
        assert counts(r) == (0, 0, 0, 0, 0), seq
        assert r[F["peak"]] == en["peak"][q] and r[F["duration"]] == en["duration"][q], seq
    assert fitted > 20
