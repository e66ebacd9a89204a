"""GPU parity of moc_eval_cuts: every cut-and-recompute move scored as the
oracle scores it (edit the candidate, evaluate it in full), bit-exact."""
import numpy as np
import pytest

import oracle
from helpers import upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moc():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2304_14463_amd import moccasin
    moccasin.lib()
    return moccasin


def to_dev(*arrs):
    import torch
    return [torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in arrs]


def gpu_cuts(moc, gh, ds, de, da):
    """Table and best move of every base, and the best move from a launch that writes no table."""
    moves, best = moc.moc_eval_cuts(gh, ds, de, da, want_moves=True, want_best=True)
    _, alone = moc.moc_eval_cuts(gh, ds, de, da, want_moves=False, want_best=True)
    best = moc.results_to_numpy(best, moc.BEST_MOVE_DTYPE)
    assert (moc.results_to_numpy(alone, moc.BEST_MOVE_DTYPE) == best).all()
    return moc.results_to_numpy(moves, moc.TOGGLE_SCORE_DTYPE), best


def assert_best(best, want, what=""):
    """want: the oracle's table of one base with its fourth column; the best move is the first
    minimum of (violations, peak, positions left at the base's peak)."""
    ok = np.flatnonzero(want[:, 0] >= 0)
    if ok.size == 0:
        assert (int(best["move"]), int(best["violations"]), int(best["peak"])) == (-1, 0, 0), what
        return
    q = min(ok, key=lambda q: (want[q, 0], want[q, 1], want[q, 3], q))
    assert (int(best["move"]), int(best["violations"]), int(best["peak"])) == (q, want[q, 0], want[q, 1]), what


def assert_same(got, want, what=""):
    for i, name in enumerate(("violations", "peak", "duration")):
        bad = np.flatnonzero(got[name].astype(np.int64) != want[:, i])
        assert bad.size == 0, f"{what}: {name} differs at {bad[:8]}: gpu {got[name][bad[:8]]} oracle {want[bad[:8], i]}"


def schedules(rng, g, C, B, wild):
    """Rows in turn: a topological order spread over the positions with every output kept to
    its last use (violation-free, plenty of cuts); the same with some copies of other nodes
    active at random places; random intervals (wild: also outside [0, T))."""
    n, T = g.n, g.n * C
    out_last = np.zeros(n, int)
    s = np.zeros((B, T), np.int32); e = np.zeros((B, T), np.int32); a = np.zeros((B, T), np.uint8)
    for b in range(B):
        kind = b % 3
        if kind == 2:
            lo, hi = (-3, T + 3) if wild else (0, T)
            s[b] = rng.integers(lo, hi, T); e[b] = rng.integers(lo, hi, T)
            swap = (s[b] > e[b]) & (rng.random(T) < 0.8)
            s[b], e[b] = np.where(swap, e[b], s[b]), np.where(swap, s[b], e[b])
            a[b] = rng.random(T) < 0.6
            continue
        pos = np.sort(rng.choice(T, size=n, replace=False))
        out_last[:] = pos
        for v in range(n):
            for u in g.in_idx[g.in_ptr[v]:g.in_ptr[v + 1]]:
                out_last[u] = max(out_last[u], pos[v])
        s[b] = rng.integers(0, T, T); e[b] = rng.integers(0, T, T)    # fields of inactive copies: anything
        s[b, ::C], e[b, ::C], a[b, ::C] = pos, out_last, 1
        if kind == 1 and C > 1:
            extra = rng.random(T) < 0.15
            extra[::C] = False
            a[b][extra] = 1
            hi = np.maximum(s[b], e[b]); lo = np.minimum(s[b], e[b])
            s[b][extra], e[b][extra] = lo[extra], hi[extra]
    return s, e, a


@pytest.mark.parametrize("n,C", [(2, 2), (5, 1), (9, 2), (17, 3), (40, 2), (64, 4), (130, 2), (257, 3), (600, 2)])
def test_cuts_small_graphs(moc, n, C):
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(53 * n + C)
    edges = []
    for v in range(1, n):
        for u in rng.integers(0, v, size=rng.integers(1, 4)):
            edges.append((int(u), v))         # duplicates stay: separate instances
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(1, 9, n))
    B = 9
    s, e, a = schedules(rng, g, C, B, wild=True)
    budget = int(g.size.sum()) // 2
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    ds, de, da = to_dev(s, e, a)
    got, best = gpu_cuts(moc, gh, ds, de, da)
    applicable = 0
    for b in range(B):
        want = oracle.cuts(g, budget, C, s[b], e[b], a[b], with_at_peak=True)
        assert_same(got[b], want, f"n={n} C={C} row {b}")
        assert_best(best[b], want, f"n={n} C={C} row {b}")
        applicable += int((want[:, 0] >= 0).sum())
    assert applicable > 0 or C == 1
    gh.free()


def test_cuts_hub_node(moc):
    """One node feeds all others: long adjacency walks, uses on both sides of every cut."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    n, C = 300, 2
    rng = np.random.default_rng(8)
    edges = [(0, v) for v in range(1, n)] + [(v - 1, v) for v in range(2, n)]
    g = graph_from_edges(n, sorted(edges), rng.integers(1, 50, n), rng.integers(1, 9, n))
    s, e, a = schedules(rng, g, C, 6, wild=False)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 1000, C)
    ds, de, da = to_dev(s, e, a)
    got, best = gpu_cuts(moc, gh, ds, de, da)
    for b in range(6):
        want = oracle.cuts(g, 1000, C, s[b], e[b], a[b], with_at_peak=True)
        assert_same(got[b], want, f"hub row {b}")
        assert_best(best[b], want, f"hub row {b}")
    assert (got["violations"][0] >= 0).sum() > n // 2
    gh.free()


def test_cuts_workload(moc, workloads):
    """n=2000, C=2 at the full batch: sampled bases against the oracle; sampled moves applied by
    the oracle and evaluated with moc_eval_batch; a cut never raises the peak."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(3)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    out, best = moc.moc_eval_cuts(gh, ds, de, da, want_best=True)
    _, alone = moc.moc_eval_cuts(gh, ds, de, da, want_moves=False, want_best=True)
    base = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    torch.cuda.synchronize()
    best = moc.results_to_numpy(best, moc.BEST_MOVE_DTYPE)
    assert (moc.results_to_numpy(alone, moc.BEST_MOVE_DTYPE) == best).all()
    for b in (0, w.B // 2 + 1, w.B - 1):
        s, e, a = ds[b].cpu().numpy(), de[b].cpu().numpy(), da[b].cpu().numpy()
        got = moc.results_to_numpy(out[b], moc.TOGGLE_SCORE_DTYPE)
        want = oracle.cuts(w.graph, w.budget, w.C, s, e, a, with_at_peak=True)
        assert_same(got, want, f"base {b}")
        assert_best(best[b], want, f"base {b}")
    # every base: the best move carries the least (violations, peak) of its own table
    for b in range(0, w.B, 97):
        got = moc.results_to_numpy(out[b], moc.TOGGLE_SCORE_DTYPE)
        ok = np.flatnonzero(got["violations"] >= 0)
        least = min((int(got["violations"][q]), int(got["peak"][q])) for q in ok)
        q = int(best[b]["move"])
        assert (int(best[b]["violations"]), int(best[b]["peak"])) == least == (int(got["violations"][q]), int(got["peak"][q]))
    rng = np.random.default_rng(5)
    rows, es, ee, ea, want = [], [], [], [], []
    for b in rng.integers(0, w.B, 48):
        got = moc.results_to_numpy(out[b], moc.TOGGLE_SCORE_DTYPE)
        ok = np.flatnonzero(got["violations"] >= 0)
        assert ok.size > 0
        assert (got["peak"][ok] <= base["peak"][b]).all()
        for q in rng.choice(ok, 4):
            x, i = divmod(int(q), w.C)
            s, e, a = ds[b].cpu().numpy(), de[b].cpu().numpy(), da[b].cpu().numpy()
            applied, s2, e2, a2 = oracle.cut_apply(w.graph, w.C, s, e, a, x, i)
            assert applied
            es.append(s2); ee.append(e2); ea.append(a2); want.append(got[q])
    d2 = to_dev(np.stack(es), np.stack(ee), np.stack(ea))
    res = moc.results_to_numpy(moc.moc_eval_batch(gh, *d2))
    want = np.array(want)
    assert (res["violations"] == want["violations"]).all()
    assert (res["peak"] == want["peak"]).all() and (res["duration"] == want["duration"]).all()
    gh.free()


def test_cuts_adjacency_from_global_memory(moc):
    """A graph whose adjacency lists do not fit in LDS beside the working set."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    n, C = 4300, 2
    rng = np.random.default_rng(12)
    edges = []
    for v in range(1, n):
        for u in rng.integers(max(0, v - 40), v, size=rng.integers(1, 4)):
            edges.append((int(u), v))
    g = graph_from_edges(n, sorted(set(edges)), rng.integers(1, 50, n), rng.integers(1, 9, n))
    s, e, a = schedules(rng, g, C, 3, wild=False)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 5000, C)
    ds, de, da = to_dev(s, e, a)
    got, best = gpu_cuts(moc, gh, ds, de, da)
    for b in range(3):
        want = oracle.cuts(g, 5000, C, s[b], e[b], a[b], with_at_peak=True)
        assert_same(got[b], want, f"row {b}")
        assert_best(best[b], want, f"row {b}")
    gh.free()


def test_cuts_rejects_bad_arguments(moc):
    import ctypes
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(3, [(0, 1), (1, 2)], [1, 1, 1], [1, 1, 1])
    gh = moc.moc_graph_upload(3, g.in_ptr, g.in_idx, g.size, g.dur, 1, 2)
    s = torch.zeros((2, 6), dtype=torch.int32, device="cuda")
    a = torch.zeros((2, 6), dtype=torch.uint8, device="cuda")
    out = torch.zeros((2, 4, 16), dtype=torch.uint8, device="cuda")
    L = moc.lib()
    vp = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    assert L.moc_eval_cuts(gh._h, 2, vp(s), vp(s), vp(a), None, None, None) == -1
    assert L.moc_eval_cuts(gh._h, 2, None, vp(s), vp(a), vp(out), None, None) == -1
    assert L.moc_eval_cuts(gh._h, 1, vp(s), vp(s), vp(a), vp(out, 4), None, None) == -1
    assert L.moc_eval_cuts(gh._h, 0, None, None, None, vp(out), None, None) == 0
    gh.free()
    gl = graph_from_edges(2, [(0, 0), (0, 1)], [1, 1], [1, 1])
    gh = moc.moc_graph_upload(2, gl.in_ptr, gl.in_idx, gl.size, gl.dur, 1, 2)
    assert L.moc_eval_cuts(gh._h, 1, vp(s), vp(s), vp(a), vp(out), None, None) == -1      # an edge (v, v)
    gh.free()
    g0 = graph_from_edges(2, [], [1, 1], [1, 1])                                    # no edges: nothing to do
    gh = moc.moc_graph_upload(2, g0.in_ptr, g0.in_idx, g0.size, g0.dur, 1, 2)
    best = torch.full((1, 16), 7, dtype=torch.uint8, device="cuda")
    assert L.moc_eval_cuts(gh._h, 1, vp(s), vp(s), vp(a), vp(out), vp(best), None) == 0
    bm = moc.results_to_numpy(best, moc.BEST_MOVE_DTYPE)
    assert (int(bm["move"][0]), int(bm["violations"][0]), int(bm["peak"][0])) == (-1, 0, 0)
    gh.free()


@pytest.mark.parametrize("cfg,count,steps", [(0, 48, 6), (1, 12, 20)])
def test_search_cuts_follows_the_oracle(moc, workloads, cfg, count, steps):
    """Greedy descent by cuts: after the same number of steps the candidates are, field by
    field, what the oracle's descent leaves (active copies compared on all three arrays,
    inactive ones on the flag: their starts and ends are never touched)."""
    import torch
    w = workloads(cfg)
    s, e, a = w.candidates(0, count)
    s0, e0, a0 = w.base()
    s[0], e[0], a[0] = s0, e0, a0          # the plain schedule: violation-free, above the budget
    gh = upload(moc, w)
    ds, de, da = to_dev(s, e, a)
    n_steps = moc.moc_search_cuts(gh, ds, de, da, steps).cpu().numpy()
    gs, ge, ga = ds.cpu().numpy(), de.cpu().numpy(), da.cpu().numpy()
    moved = 0
    for b in range(count):
        want_steps, ws, we, wa = oracle.search_cuts(w.graph, w.budget, w.C, s[b], e[b], a[b], steps)
        assert n_steps[b] == want_steps, b
        assert (ga[b] == wa).all() and (gs[b] == ws).all() and (ge[b] == we).all(), b
        moved += want_steps
    assert n_steps[0] > 0 and moved > count // 4
    gh.free()


def test_search_cuts_full_batch(moc, workloads):
    """n=2000, C=2, all 8192 bases, 3 steps: no candidate gets worse, every applied cut adds one
    active copy, and one candidate is followed step by step by the oracle."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(3)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    before = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    s0, e0, a0 = ds[5].cpu().numpy(), de[5].cpu().numpy(), da[5].cpu().numpy()
    n_active = (da != 0).sum(1)
    n_steps = moc.moc_search_cuts(gh, ds, de, da, 3)
    after = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    torch.cuda.synchronize()
    steps = n_steps.cpu().numpy()
    assert ((da != 0).sum(1) - n_active).cpu().numpy().tolist() == steps.tolist()
    assert steps.max() == 3 and (steps > 0).mean() > 0.5
    key0 = np.stack([before["violations"], np.maximum(before["peak"], w.budget)], 1)
    key1 = np.stack([after["violations"], np.maximum(after["peak"], w.budget)], 1)
    worse = (key1[:, 0] > key0[:, 0]) | ((key1[:, 0] == key0[:, 0]) & (key1[:, 1] > key0[:, 1]))
    assert not worse.any()
    better = (key1[:, 0] < key0[:, 0]) | ((key1[:, 0] == key0[:, 0]) & (key1[:, 1] < key0[:, 1]))
    assert (better == (steps > 0)).all()
    assert (after["duration"] > before["duration"])[steps > 0].all()
    # walkers that started without violations still stand for valid sequences, one step longer
    # per cut, costed by the decoder at the evaluator's duration and at most its peak
    dec = moc.results_to_numpy(moc.moc_decode_batch(gh, ds, da, want_seq=False)[0], moc.DECODE_RESULT_DTYPE)
    clean = before["violations"] == 0
    assert clean.sum() > 100 and (dec["status"][clean] == 1).all()
    assert (dec["length"][clean] == (n_active.cpu().numpy() + steps)[clean]).all()
    assert (dec["duration"][clean] == after["duration"][clean]).all()
    assert (dec["peak"][clean] <= after["peak"][clean]).all()
    want_steps, ws, we, wa = oracle.search_cuts(w.graph, w.budget, w.C, s0, e0, a0, 3)
    assert steps[5] == want_steps
    assert (da[5].cpu().numpy() == wa).all() and (ds[5].cpu().numpy() == ws).all() and (de[5].cpu().numpy() == we).all()
    gh.free()


def test_search_cuts_rejects_bad_arguments(moc):
    import ctypes
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(3, [(0, 1), (1, 2)], [1, 1, 1], [1, 1, 1])
    gh = moc.moc_graph_upload(3, g.in_ptr, g.in_idx, g.size, g.dur, 1, 2)
    s = torch.zeros((2, 6), dtype=torch.int32, device="cuda")
    a = torch.zeros((2, 6), dtype=torch.uint8, device="cuda")
    best = torch.zeros((2, 16), dtype=torch.uint8, device="cuda")
    steps = torch.full((2,), 9, dtype=torch.int32, device="cuda")
    L = moc.lib()
    vp = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    assert L.moc_search_cuts(gh._h, 2, vp(s), vp(s), vp(a), 1, None, vp(steps), None) == -1
    assert L.moc_search_cuts(gh._h, 2, vp(s), vp(s), vp(a), 1, vp(best), None, None) == -1
    assert L.moc_search_cuts(gh._h, 2, vp(s), vp(s), vp(a), -1, vp(best), vp(steps), None) == -1
    assert L.moc_search_cuts(gh._h, 2, vp(s), vp(s), vp(a), 1, vp(best, 4), vp(steps), None) == -1
    assert L.moc_search_cuts(gh._h, 0, None, None, None, 1, None, None, None) == 0
    assert (steps.cpu().numpy() == 9).all()                       # nothing was queued by the calls above
    e = s.clone()
    assert L.moc_search_cuts(gh._h, 2, vp(s), vp(e), vp(a), 0, vp(best), vp(steps), None) == 0
    assert (steps.cpu().numpy() == 0).all()                       # no steps: the counters are cleared, nothing else
    gh.free()
