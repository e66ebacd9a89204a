"""GPU parity of the two-phase local search (Section 2.4 of arXiv 2304.14463): the cuts that keep
the producer's inputs (moc_eval_cuts_keep) scored as the oracle scores them, and
moc_search_two_phase followed by the oracle's descent, candidate by candidate, field by field."""
import numpy as np
import pytest

import oracle
from helpers import upload
from test_gpu_cuts import assert_best, assert_same, schedules, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moc():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2304_14463_amd import moccasin
    moccasin.lib()
    return moccasin


def gpu_keep_cuts(moc, gh, ds, de, da):
    moves, best = moc.moc_eval_cuts(gh, ds, de, da, want_moves=True, want_best=True, keep_inputs=True)
    _, alone = moc.moc_eval_cuts(gh, ds, de, da, want_moves=False, want_best=True, keep_inputs=True)
    best = moc.results_to_numpy(best, moc.BEST_MOVE_DTYPE)
    assert (moc.results_to_numpy(alone, moc.BEST_MOVE_DTYPE) == best).all()
    return moc.results_to_numpy(moves, moc.TOGGLE_SCORE_DTYPE), best


@pytest.mark.parametrize("n,C", [(2, 2), (5, 1), (9, 2), (17, 3), (40, 2), (64, 4), (130, 2), (257, 3), (600, 2)])
def test_keep_cuts_small_graphs(moc, n, C):
    """Random DAGs with duplicate edges; orderly schedules, schedules with stray copies, and
    random intervals (also outside the domain): tables and best moves against the oracle."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(59 * n + C)
    edges = []
    for v in range(1, n):
        for u in rng.integers(0, v, size=rng.integers(1, 4)):
            edges.append((int(u), v))
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(1, 9, n))
    B = 12
    s, e, a = schedules(rng, g, C, B, wild=True)
    # in the orderly rows, drop some outputs early so that inputs are missing where cuts want to go
    for b in range(0, B, 3):
        early = rng.random(n) < 0.4
        e[b, ::C] = np.where(early, np.minimum(e[b, ::C], s[b, ::C] + rng.integers(0, 4, n)), e[b, ::C])
    budget = int(g.size.sum()) // 2
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    ds, de, da = to_dev(s, e, a)
    got, best = gpu_keep_cuts(moc, gh, ds, de, da)
    applicable = differs = 0
    for b in range(B):
        want = oracle.cuts(g, budget, C, s[b], e[b], a[b], with_at_peak=True, mode=1)
        assert_same(got[b], want, f"n={n} C={C} row {b}")
        assert_best(best[b], want, f"n={n} C={C} row {b}")
        applicable += int((want[:, 0] >= 0).sum())
        differs += int((want[:, :3] != oracle.cuts(g, budget, C, s[b], e[b], a[b])).any())
    assert applicable > 0 or C == 1
    assert differs > 0 or n < 9 or C == 1
    gh.free()


def test_keep_cuts_hub_and_long_inputs(moc):
    """One node feeds all others, another is fed by many: long walks over kept inputs."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    n, C = 200, 2
    rng = np.random.default_rng(9)
    edges = [(0, v) for v in range(1, n)] + [(v - 1, v) for v in range(2, n)] + [(u, 150) for u in range(5, 140, 3)] + \
            [(150, v) for v in range(160, 200, 7)]
    g = graph_from_edges(n, sorted(set(edges)), rng.integers(1, 50, n), rng.integers(1, 9, n))
    s, e, a = schedules(rng, g, C, 6, wild=False)
    for b in (0, 3):
        early = rng.random(n) < 0.5
        e[b, ::C] = np.where(early, np.minimum(e[b, ::C], s[b, ::C] + rng.integers(0, 6, n)), e[b, ::C])
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 1000, C)
    ds, de, da = to_dev(s, e, a)
    got, best = gpu_keep_cuts(moc, gh, ds, de, da)
    for b in range(6):
        want = oracle.cuts(g, 1000, C, s[b], e[b], a[b], with_at_peak=True, mode=1)
        assert_same(got[b], want, f"hub row {b}")
        assert_best(best[b], want, f"hub row {b}")
    gh.free()


@pytest.mark.parametrize("cfg,rows", [(0, 12), (1, 4), (3, 2)])
def test_keep_cuts_workloads(moc, workloads, cfg, rows):
    w = workloads(cfg)
    gh = upload(moc, w)
    s1, e1, a1 = w.candidates(0, rows)
    s2, e2, a2 = w.candidates(w.B - rows, rows)
    s, e, a = np.vstack([s1, s2]), np.vstack([e1, e2]), np.vstack([a1, a2])
    s[0], e[0], a[0] = w.base()
    ds, de, da = to_dev(s, e, a)
    got, best = gpu_keep_cuts(moc, gh, ds, de, da)
    for b in range(2 * rows):
        want = oracle.cuts(w.graph, w.budget, w.C, s[b], e[b], a[b], with_at_peak=True, mode=1)
        assert_same(got[b], want, f"cfg {cfg} row {b}")
        assert_best(best[b], want, f"cfg {cfg} row {b}")
    gh.free()


@pytest.mark.parametrize("cfg,count,cuts,merges,K", [(0, 40, 8, 4, 16), (1, 6, 40, 8, 64), (1, 6, 12, 3, 2)])
def test_two_phase_follows_the_oracle(moc, workloads, cfg, count, cuts, merges, K):
    """After the same numbers of steps the candidates are, field by field, what the oracle's
    two-phase descent leaves.  Budgets are set so that the first phase ends within them for some
    walkers (the second phase only moves feasible ones)."""
    w = workloads(cfg)
    s, e, a = w.candidates(0, count)
    s[0], e[0], a[0] = w.base()
    budget = w.budget if cfg == 1 and cuts >= 40 else int(0.93 * w.no_remat_peak)
    gh = upload(moc, w, budget=budget)
    ds, de, da = to_dev(s, e, a)
    n_cuts, n_merges = moc.moc_search_two_phase(gh, ds, de, da, cuts, merges, K)
    n_cuts, n_merges = n_cuts.cpu().numpy(), n_merges.cpu().numpy()
    gs, ge, ga = ds.cpu().numpy(), de.cpu().numpy(), da.cpu().numpy()
    for b in range(count):
        k1, k2, ws, we, wa = oracle.search_two_phase(w.graph, budget, w.C, s[b], e[b], a[b], cuts, merges, K)
        assert (n_cuts[b], n_merges[b]) == (k1, k2), b
        live = wa != 0
        assert (ga[b] == wa).all() and (gs[b][live] == ws[live]).all() and (ge[b][live] == we[live]).all(), b
    assert n_cuts.max() > 0 and n_merges.max() > 0
    # what comes out is still a schedule wherever it went in as one
    res = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    before = oracle.evaluate(w.graph, budget, w.C, s, e, a)
    clean = before[:, 2] == 0
    dec = moc.results_to_numpy(moc.moc_decode_batch(gh, ds, da, want_seq=False)[0], moc.DECODE_RESULT_DTYPE)
    assert (res["violations"][clean] == 0).all() and (dec["status"][clean] == 1).all()
    assert (dec["duration"][clean] == res["duration"][clean]).all() and (dec["peak"][clean] <= res["peak"][clean]).all()
    gh.free()


def test_two_phase_rejects_bad_arguments(moc):
    import ctypes
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(3, [(0, 1), (1, 2)], [1, 1, 1], [1, 1, 1])
    gh = moc.moc_graph_upload(3, g.in_ptr, g.in_idx, g.size, g.dur, 1, 2)
    B, K, T = 2, 4, 6
    s = torch.zeros((B, T), dtype=torch.int32, device="cuda")
    a = torch.zeros((B, T), dtype=torch.uint8, device="cuda")
    best = torch.zeros((B, 16), dtype=torch.uint8, device="cuda")
    ws = torch.zeros((B * K, T), dtype=torch.int32, device="cuda")
    wa = torch.zeros((B * K, T), dtype=torch.uint8, device="cuda")
    wl = torch.zeros((B * K,), dtype=torch.int32, device="cuda")
    wr = torch.zeros((B * K, 24), dtype=torch.uint8, device="cuda")
    c1 = torch.full((B,), 9, dtype=torch.int32, device="cuda")
    c2 = torch.full((B,), 9, dtype=torch.int32, device="cuda")
    L = moc.lib()
    vp = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    call = lambda *x: L.moc_search_two_phase(gh._h, *x)
    ok = (B, vp(s), vp(s), vp(a), 1, 1, K, vp(best), vp(ws), vp(ws), vp(wa), vp(wl), vp(wr), vp(c1), vp(c2), None)
    bad = lambda i, v: ok[:i] + (v,) + ok[i + 1:]
    assert call(*bad(4, -1)) == -1 and call(*bad(5, -1)) == -1 and call(*bad(6, 0)) == -1
    assert call(*bad(7, None)) == -1 and call(*bad(8, None)) == -1 and call(*bad(12, None)) == -1
    assert call(*bad(13, None)) == -1 and call(*bad(12, vp(wr, 4))) == -1
    assert (c1.cpu().numpy() == 9).all()                       # nothing was queued by the calls above
    assert call(*bad(5, 0)[:8], None, None, None, None, None, vp(c1), vp(c2), None) == 0   # no second phase: no workspace
    assert call(0, None, None, None, 1, 1, K, None, None, None, None, None, None, None, None, None) == 0
    e = s.clone()
    assert call(B, vp(s), vp(e), vp(a), 1, 1, K, vp(best), vp(ws), vp(ws.clone()), vp(wa), vp(wl), vp(wr), vp(c1), vp(c2), None) == 0
    torch.cuda.synchronize()
    assert (c1.cpu().numpy() == 0).all() and (c2.cpu().numpy() == 0).all()
    gh.free()
