"""Pins of the oracle's neighbourhood scorer (orc_neighbours) and of its descent by
single-field moves (oracle.search_moves), without a GPU.

The move set is this library's, not the paper's (arXiv 2304.14463 defines the variables a
local search would edit, Section 2.1, and the quantity Phase 1 minimises, Section 2.4); what
has to be pinned is the numbering of the moves, the rule for moves that do not apply, and the
order by which the best one is chosen.  Every expected value below is either written out by
hand or obtained by editing the candidate *in the test* and evaluating it; none goes through
the oracle's own decoding of a move index.
"""
import numpy as np

import oracle
from paper_2304_14463_amd.inputs import graph_from_edges

F = {name: i for i, name in enumerate(oracle.FIELDS)}


def vp(g, budget, C, s, e, a):
    r = oracle.evaluate(g, budget, C, s, e, a)[0]
    return int(r[F["violations"]]), int(r[F["peak"]])


def chain3():
    """0 -> 1 -> 2, sizes 1, 2, 4, two copies per node (T = 6).
    copy:      k=0      k=1         k=2      k=3         k=4      k=5
    node 0: [0,1]   inactive    node 1: [1,2]  inactive  node 2: [2,2]  active, [4,3] (ill formed)"""
    g = graph_from_edges(3, [(0, 1), (1, 2)], [1, 2, 4], [3, 5, 7])
    s = np.array([0, 5, 1, 0, 2, 4], np.int32)
    e = np.array([1, 5, 2, 0, 2, 3], np.int32)
    a = np.array([1, 0, 1, 0, 1, 1], np.uint8)
    return g, 2, s, e, a


def test_base_of_the_hand_case():
    g, C, s, e, a = chain3()
    # profile: t0 = 1, t1 = 1 + 2, t2 = 2 + 4; the only violation is the ill-formed copy 5
    assert vp(g, 100, C, s, e, a) == (1, 6)


def test_move_indices_written_out_by_hand():
    """R = 2: a copy has 8 moves, start by -2, -1, +1, +2 and then end by -2, -1, +1, +2.
    (q, copy, field, displacement) below are counted by hand from that order."""
    g, C, s, e, a = chain3()
    R = 2
    scores, _ = oracle.neighbours(g, 100, C, s, e, a, R)
    assert scores.shape == (6 * 4 * R, 2)
    by_hand = [(2, 0, "s", +1), (5, 0, "e", -1), (6, 0, "e", +1), (7, 0, "e", +2),
               (17, 2, "s", -1), (19, 2, "s", +2), (18, 2, "s", +1), (21, 2, "e", -1), (22, 2, "e", +1),
               (32, 4, "s", -2), (33, 4, "s", -1), (34, 4, "s", +1), (35, 4, "s", +2), (36, 4, "e", -2),
               (38, 4, "e", +1), (40, 5, "s", -2), (41, 5, "s", -1), (46, 5, "e", +1), (47, 5, "e", +2)]
    for q, k, field, delta in by_hand:
        s2, e2 = s.copy(), e.copy()
        (s2 if field == "s" else e2)[k] += delta
        assert tuple(scores[q]) == vp(g, 100, C, s2, e2, a), (q, k, field, delta)
    # and their values, counted by hand
    # q=17: node 1 starts at 0: shares node 0's start (Eq. 6) and s_0 + 1 <= s_1 fails (Eq. 5);
    #       profile t0 = 1+2, t1 = 1+2, t2 = 2+4
    assert tuple(scores[17]) == (1 + 2, 6)
    # q=5: node 0 kept on [0,0] only: node 1 at 1 is not covered; profile 1, 2, 6
    assert tuple(scores[5]) == (1 + 1, 6)
    # q=6: node 0 kept on [0,2]: profile 1, 3, 7
    assert tuple(scores[6]) == (1, 7)
    # q=34: node 2 would be [3,2]: ill formed, so it drops out of everything: profile 1, 3, 2
    assert tuple(scores[34]) == (1 + 1, 3)
    # q=33: node 2 at 1 shares node 1's start and is not covered by it; profile 1, 1+2+4, 2+4
    assert tuple(scores[33]) == (1 + 2, 7)
    # q=46: copy 5 becomes [4,4]: well formed, a second live copy of node 2 after [2,2]: no order
    #       violation (2 <= 4), its input node 1 is kept on [1,2] only: not covered
    assert tuple(scores[46]) == (1, 6)
    # q=41: copy 5 becomes [3,3]: same, profile t3 = 4
    assert tuple(scores[41]) == (1, 6)
    # q=21: node 1 kept on [1,1]: node 2 at 2 not covered; profile 1, 3, 4
    assert tuple(scores[21]) == (1 + 1, 4)


def test_every_move_against_an_enumeration_in_the_documented_order():
    """The whole table against candidates edited here.  The test walks the moves in the
    documented order (copy, then field, then displacement -R..-1, +1..+R) and counts q up,
    instead of taking an index apart."""
    rng = np.random.default_rng(23)
    n, C = 5, 2
    g = graph_from_edges(n, [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (1, 4)], [3, 1, 4, 1, 5], [2, 7, 1, 8, 2])
    T = n * C
    for R in (1, 3):
        for trial in range(4):
            s = rng.integers(0, T, T).astype(np.int32)
            e = np.minimum(T - 1, s + rng.integers(-1, 5, T)).astype(np.int32)
            a = (rng.random(T) < 0.7).astype(np.uint8)
            scores, best = oracle.neighbours(g, 12, C, s, e, a, R)
            q = 0
            keys = []
            for k in range(T):
                for arr_name in ("s", "e"):
                    for delta in list(range(-R, 0)) + list(range(1, R + 1)):
                        s2, e2 = s.copy(), e.copy()
                        arr = s2 if arr_name == "s" else e2
                        arr[k] += delta
                        if a[k] == 0 or arr[k] < 0 or arr[k] > T - 1:
                            assert tuple(scores[q]) == (-1, -1), (R, trial, q)
                        else:
                            want = vp(g, 12, C, s2, e2, a)
                            assert tuple(scores[q]) == want, (R, trial, q)
                            keys.append((want[0], max(want[1], 12), want[1], q))
                        q += 1
            assert q == scores.shape[0]
            if keys:
                v, _, p, qb = min(keys)
                assert best == (qb, v, p)
            else:
                assert best == (-1, 0, 0)


def test_moves_that_do_not_apply():
    g, C, s, e, a = chain3()
    R = 2
    T = 6
    scores, _ = oracle.neighbours(g, 100, C, s, e, a, R)
    # inactive copies 1 and 3: all 4R moves, whatever their start and end are
    for k in (1, 3):
        assert (scores[k * 4 * R:(k + 1) * 4 * R] == -1).all()
    # copy 0 starts at 0: start by -2 and by -1 leave [0, T)
    assert tuple(scores[0]) == (-1, -1) and tuple(scores[1]) == (-1, -1)
    # copy 0 ends at 1: end by -2 leaves, by -1 stays
    assert tuple(scores[4]) == (-1, -1) and scores[5, 0] >= 0
    # the ill-formed but active copy 5 = [4,3]: its moves apply as long as the field stays inside
    assert scores[40, 0] >= 0 and scores[43, 0] < 0     # start 4 -> 2 stays, 4 -> 6 = T leaves
    assert scores[44, 0] >= 0 and scores[47, 0] >= 0    # end 3 -> 1, 3 -> 5 = T - 1
    # an end at T - 1 cannot move up
    s2, e2 = s.copy(), e.copy()
    e2[4] = T - 1
    sc2, _ = oracle.neighbours(g, 100, C, s2, e2, a, R)
    assert tuple(sc2[38]) == (-1, -1) and tuple(sc2[39]) == (-1, -1) and sc2[37, 0] >= 0
    # nothing active at all: no best move
    _, best = oracle.neighbours(g, 100, C, s, e, np.zeros(6, np.uint8), R)
    assert best == (-1, 0, 0)


def test_move_that_turns_a_copy_ill_formed_costs_one_violation_of_eq2():
    """Start past the end: the copy stays active, is one violation of Eq. (2), and no longer
    takes part in anything else."""
    g = graph_from_edges(2, [], [3, 5], [1, 1])
    s = np.array([0, 1], np.int32)
    e = np.array([0, 1], np.int32)
    a = np.ones(2, np.uint8)
    assert vp(g, 100, 1, s, e, a) == (0, 5)
    scores, best = oracle.neighbours(g, 100, 1, s, e, a, 1)
    # copy 0: start -1 leaves; start +1 -> [1,0]: V_form = 1, only node 1 left in the profile
    assert [tuple(x) for x in scores[0:4]] == [(-1, -1), (1, 5), (-1, -1), (0, 5 + 3)]
    # copy 1: start -1 -> [0,1] shares node 0's start; start +1 leaves; end -1 -> [1,0]; end +1 leaves
    assert [tuple(x) for x in scores[4:8]] == [(1, 8), (-1, -1), (1, 3), (-1, -1)]
    # best: no violation, lowest peak -- only q = 3 has none
    assert best == (3, 0, 8)


def test_subset_of_moves_and_its_best():
    """With a list of move indices the scores are those of the listed moves, in the list's
    order, and the best move is taken among them."""
    g, C, s, e, a = chain3()
    full, _ = oracle.neighbours(g, 100, C, s, e, a, 2)
    pick = np.array([34, 6, 0, 21, 17], np.int64)
    sub, best = oracle.neighbours(g, 100, C, s, e, a, 2, moves=pick)
    assert (sub == full[pick]).all()
    # (1,7) for q=6 against (2,3), (2,4), (3,6): fewest violations first
    assert best == (6, 1, 7)


def test_best_move_keys_in_order():
    """(violations, max(peak, M), peak, q): built so that each key decides once."""
    g = graph_from_edges(3, [(0, 1), (1, 2)], [5, 1, 1], [1, 1, 1])
    s = np.array([0, 1, 2], np.int32)
    e = np.array([0, 1, 2], np.int32)
    a = np.ones(3, np.uint8)
    # both edges uncovered.  end of node 0 +1 (q=3): one left, profile 5, 6, 1;
    # end of node 1 +1 (q=7): one left, profile 5, 1, 2.  Fewer violations than any other move.
    scores, best = oracle.neighbours(g, 100, 1, s, e, a, 1)
    assert tuple(scores[3]) == (1, 6) and tuple(scores[7]) == (1, 5)
    assert sorted(int(x) for x in np.flatnonzero((scores[:, 0] >= 0) & (scores[:, 0] < 2))) == [3, 7]
    assert best == (7, 1, 5)                      # peak decides although q is larger ...
    _, best = oracle.neighbours(g, 5, 1, s, e, a, 1)
    assert best == (7, 1, 5)                      # ... also where max(peak, M) already differs (6 > 5 = M)
    # equal peaks: the lower index
    g2 = graph_from_edges(3, [(0, 1), (1, 2)], [1, 1, 1], [1, 1, 1])
    scores, best = oracle.neighbours(g2, 100, 1, s, e, a, 1)
    assert tuple(scores[3]) == (1, 2) == tuple(scores[7])
    assert best == (3, 1, 2)


# ---------------------------------------------------------------- descent by single-field moves
def test_search_moves_followed_by_hand():
    """Chain 0 -> 1 -> 2, sizes 5, 1, 1, one copy per node, every output dropped at once:
    [0,0], [1,1], [2,2], two uncovered inputs.  R = 1.
    Step 1: keeping node 1 one position longer (profile 5, 1, 2) or node 0 (5, 6, 1) each mend
            one input; the lower peak wins: e_1 = 2.
    Step 2: keeping node 0 to position 1 mends the other: profile 5, 6, 2, no violation left.
    Step 3: every move from there adds a violation: stop."""
    g = graph_from_edges(3, [(0, 1), (1, 2)], [5, 1, 1], [1, 1, 1])
    s = np.array([0, 1, 2], np.int32)
    e = np.array([0, 1, 2], np.int32)
    a = np.ones(3, np.uint8)
    for budget in (3, 100):
        k, s1, e1 = oracle.search_moves(g, budget, 1, s, e, a, 1, 1)
        assert (k, list(s1), list(e1)) == (1, [0, 1, 2], [0, 2, 2])
        k, s2, e2 = oracle.search_moves(g, budget, 1, s, e, a, 1, 2)
        assert (k, list(s2), list(e2)) == (2, [0, 1, 2], [1, 2, 2])
        k, s3, e3 = oracle.search_moves(g, budget, 1, s, e, a, 1, 10)
        assert (k, list(s3), list(e3)) == (2, [0, 1, 2], [1, 2, 2])
        assert vp(g, budget, 1, s3, e3, a) == (0, 6)
    # the inputs are left as they were
    assert list(e) == [0, 1, 2]


def test_search_moves_lowers_the_peak_only_above_nothing_else():
    """Without violations a move is taken when it lowers (max(peak, M), peak): an output kept
    past its last use is released earlier, step by step, also below the budget (third key)."""
    g = graph_from_edges(3, [(0, 1), (1, 2)], [4, 1, 1], [1, 1, 1])
    s = np.array([0, 1, 2], np.int32)
    e = np.array([2, 2, 2], np.int32)      # node 0 kept through position 2 although used at 1 only
    a = np.ones(3, np.uint8)
    assert vp(g, 100, 1, s, e, a) == (0, 6)        # profile 4, 5, 6
    k, s1, e1 = oracle.search_moves(g, 100, 1, s, e, a, 2, 10)
    # one move: e_0 = 2 -> 1 (profile 4, 5, 2: peak 5); e_0 -> 0 would uncover node 1;
    # a radius of 2 offers that move directly, it is refused by the violation it adds
    assert (k, list(s1), list(e1)) == (1, [0, 1, 2], [1, 2, 2])
    assert vp(g, 100, 1, s1, e1, a) == (0, 5)
    # a move that leaves all three keys as they are is not taken
    k, s2, e2 = oracle.search_moves(g, 100, 1, s1, e1, a, 2, 10)
    assert k == 0 and list(e2) == [1, 2, 2]


def test_search_moves_is_a_descent_on_random_candidates():
    """Each step applies the first minimum of the table of the candidate it starts from, and
    the key (violations, max(peak, M), peak) falls strictly."""
    rng = np.random.default_rng(3)
    n, C, R = 8, 2, 2
    edges = sorted({(int(u), v) for v in range(1, n) for u in rng.integers(0, v, size=2)})
    g = graph_from_edges(n, edges, rng.integers(1, 20, n), rng.integers(1, 9, n))
    T = n * C
    M = 30
    for trial in range(4):
        s = np.sort(rng.permutation(T)[:T]).astype(np.int32)
        e = np.minimum(T - 1, s + rng.integers(0, 6, T)).astype(np.int32)
        a = (rng.random(T) < 0.6).astype(np.uint8)
        a[::C] = 1
        total, fs, fe = oracle.search_moves(g, M, C, s, e, a, R, 50)
        assert total < 50
        cs, ce = s.copy(), e.copy()
        prev = vp(g, M, C, cs, ce, a)
        for step in range(total):
            scores, _ = oracle.neighbours(g, M, C, cs, ce, a, R)
            best_key, best_edit = None, None
            q = 0
            for k in range(T):
                for arr_name in ("s", "e"):
                    for delta in list(range(-R, 0)) + list(range(1, R + 1)):
                        if scores[q, 0] >= 0:
                            key = (int(scores[q, 0]), max(int(scores[q, 1]), M), int(scores[q, 1]), q)
                            if best_key is None or key < best_key:
                                best_key, best_edit = key, (arr_name, k, delta)
                        q += 1
            assert best_key[:3] < (prev[0], max(prev[1], M), prev[1])
            (cs if best_edit[0] == "s" else ce)[best_edit[1]] += best_edit[2]
            prev = vp(g, M, C, cs, ce, a)
            assert prev == (best_key[0], best_key[2])
            k2, ps, pe = oracle.search_moves(g, M, C, s, e, a, R, step + 1)
            assert k2 == step + 1 and (ps == cs).all() and (pe == ce).all()
        assert (fs == cs).all() and (fe == ce).all()
