"""GPU parity of moc_eval_neighbours: every move score equals the oracle's full
re-evaluation of the moved candidate, bit-exact; the best move follows the
documented ordering."""
import numpy as np
import pytest

import oracle
from helpers import F, upload

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


def gpu_neighbours(moc, gh, s, e, a, R, moves=True, best=True):
    ds, de, da = to_dev(s, e, a)
    om, ob = moc.moc_eval_neighbours(gh, ds, de, da, R, want_moves=moves, want_best=best)
    om = moc.results_to_numpy(om, moc.MOVE_SCORE_DTYPE) if om is not None else None
    ob = moc.results_to_numpy(ob, moc.BEST_MOVE_DTYPE) if ob is not None else None
    return om, ob


def random_candidates(rng, B, K, T, wild):
    lo, hi = (-3, T + 3) if wild else (0, T)
    s = rng.integers(lo, hi, size=(B, K)).astype(np.int32)
    e = rng.integers(lo, hi, size=(B, K)).astype(np.int32)
    swap = (rng.random((B, K)) < 0.8) & (s > e)
    s, e = np.where(swap, e, s).astype(np.int32), np.where(swap, s, e).astype(np.int32)
    a = (rng.random((B, K)) < 0.7).astype(np.uint8)
    return s, e, a


@pytest.mark.parametrize("n,C,R", [(1, 1, 1), (2, 2, 2), (5, 1, 3), (9, 2, 8), (12, 3, 4), (17, 2, 8), (30, 4, 2),
                                   (40, 3, 8), (64, 2, 5), (20, 2, 17), (10, 1, 32), (24, 5, 8), (70, 1, 16),
                                   (33, 4, 9)])
def test_neighbours_full_table_small_graphs(moc, n, C, R):
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(1000 * n + 10 * C + R)
    edges = set()
    for v in range(1, n):
        for u in rng.integers(0, v, size=rng.integers(0, 4)):
            edges.add((int(u), v))
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(1, 9, n))
    T = n * C
    budget = int(g.size.sum()) // 2
    B = 6
    s, e, a = random_candidates(rng, B, T, T, wild=True)
    # one orderly candidate: a topological order with every copy 0 kept to the end
    s[0] = 0; e[0] = 0; a[0] = 0
    for v in range(n):
        s[0, v * C], e[0, v * C], a[0, v * C] = v, T - 1, 1
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    om, ob = gpu_neighbours(moc, gh, s, e, a, R)
    for b in range(B):
        scores, best = oracle.neighbours(g, budget, C, s[b], e[b], a[b], R)
        assert (om[b]["violations"].astype(np.int64) == scores[:, 0]).all(), (n, C, R, b)
        assert (om[b]["peak"].astype(np.int64) == scores[:, 1]).all(), (n, C, R, b)
        assert (int(ob[b]["move"]), int(ob[b]["violations"]), int(ob[b]["peak"])) == best, (n, C, R, b)
    # each output alone
    om2, _ = gpu_neighbours(moc, gh, s, e, a, R, best=False)
    _, ob2 = gpu_neighbours(moc, gh, s, e, a, R, moves=False)
    assert om2.tobytes() == om.tobytes() and ob2.tobytes() == ob.tobytes()
    gh.free()


@pytest.mark.parametrize("consumers,C,R", [(10, 1, 4), (70, 1, 4), (40, 2, 8), (70, 2, 16)])
def test_neighbours_hub_node(moc, consumers, C, R):
    """One provider with many consumers: moving its copy uncovers up to `consumers` * C
    consumer copies at once, more than the per-move counters of the fast path hold (63) in
    the larger cases, and more than fit three bit planes in the smaller ones.  Also a base
    with no active copy at all, and one with every copy active."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(7 * consumers + C + R)
    n = consumers + 2
    edges = [(0, v) for v in range(1, consumers + 1)] + [(1, n - 1)]
    g = graph_from_edges(n, edges, rng.integers(1, 20, n), rng.integers(1, 5, n))
    T = n * C
    budget = int(g.size.sum()) // 3
    B = 4
    s = np.zeros((B, T), np.int32); e = np.zeros((B, T), np.int32); a = np.zeros((B, T), np.uint8)
    for b in range(2):   # node v computed at position v*C, kept to the end; b = 1: the hub is dropped early
        for v in range(n):
            s[b, v * C], e[b, v * C], a[b, v * C] = v * C, T - 1, 1
    e[1, 0] = min(T - 1, 3 * C)
    a[3, :] = 1   # every copy active, all intervals [0, 0]; b = 2: nothing active
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    om, ob = gpu_neighbours(moc, gh, s, e, a, R)
    _, ob2 = gpu_neighbours(moc, gh, s, e, a, R, moves=False)
    for b in range(B):
        scores, best = oracle.neighbours(g, budget, C, s[b], e[b], a[b], R)
        assert (om[b]["violations"].astype(np.int64) == scores[:, 0]).all(), b
        assert (om[b]["peak"].astype(np.int64) == scores[:, 1]).all(), b
        assert (int(ob[b]["move"]), int(ob[b]["violations"]), int(ob[b]["peak"])) == best, b
    assert ob2.tobytes() == ob.tobytes()
    gh.free()


def test_neighbours_smallest_workload_all_moves(moc, workloads):
    w = workloads(0)
    gh = upload(moc, w)
    s1, e1, a1 = w.candidates(0, 4)
    s2, e2, a2 = w.candidates(w.B - 4, 4)
    s, e, a = np.vstack([s1, s2]), np.vstack([e1, e2]), np.vstack([a1, a2])
    om, ob = gpu_neighbours(moc, gh, s, e, a, 8)
    for b in range(8):
        scores, best = oracle.neighbours(w.graph, w.budget, w.C, s[b], e[b], a[b], 8)
        assert (om[b]["violations"].astype(np.int64) == scores[:, 0]).all()
        assert (om[b]["peak"].astype(np.int64) == scores[:, 1]).all()
        assert (int(ob[b]["move"]), int(ob[b]["violations"]), int(ob[b]["peak"])) == best
    gh.free()


@pytest.mark.timeout(900)
def test_neighbours_workload_eight_bases_all_moves(moc, workloads):
    """n=2000, C=2, R=8 at the full batch of 8192 bases (1.05e9 moves): the oracle
    re-evaluates sampled moves; the best move is checked against the GPU's own
    table for every base, and a sample of moves is applied and re-evaluated with
    moc_eval_batch."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(3)
    R = w.R
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    om_t, ob_t = moc.moc_eval_neighbours(gh, ds, de, da, R)
    torch.cuda.synchronize()
    n_moves = w.T * 4 * R
    rng = np.random.default_rng(3)
    # eight bases (both kinds of candidate), all 128000 moves of each, against the oracle's
    # full re-evaluation of every move (about a minute on 16 host threads: the moves of a base
    # go to the oracle in slices, so that the run reports as it goes)
    import os
    from concurrent.futures import ThreadPoolExecutor
    bases = (0, 1, 1717, w.B // 2 - 1, w.B // 2, w.B // 2 + 1, 6000, w.B - 1)
    host = {b: (ds[b].cpu().numpy(), de[b].cpu().numpy(), da[b].cpu().numpy()) for b in bases}
    ob_all = moc.results_to_numpy(ob_t, moc.BEST_MOVE_DTYPE)
    slices = 16
    cut = np.linspace(0, n_moves, slices + 1).astype(np.int64)

    def score(job):
        b, j = job
        s, e, a = host[b]
        return b, j, oracle.neighbours(w.graph, w.budget, w.C, s, e, a, R, moves=np.arange(cut[j], cut[j + 1]))[0]

    table = {b: np.zeros((n_moves, 2), np.int64) for b in bases}
    with ThreadPoolExecutor(min(os.cpu_count() or 8, 16)) as ex:
        for done, (b, j, part) in enumerate(ex.map(score, [(b, j) for b in bases for j in range(slices)])):
            table[b][cut[j]:cut[j + 1]] = part
            if done % 8 == 7:
                print(f"cfg 3: {done + 1} of {len(bases) * slices} slices scored by the oracle", flush=True)
    for b in bases:
        scores = table[b]
        row = moc.results_to_numpy(om_t[b], moc.MOVE_SCORE_DTYPE)
        assert (row["violations"].astype(np.int64) == scores[:, 0]).all(), b
        assert (row["peak"].astype(np.int64) == scores[:, 1]).all(), b
        ok = np.flatnonzero(scores[:, 0] >= 0)
        assert ok.size > 30000
        first = ok[np.lexsort((ok, scores[ok, 1], np.maximum(scores[ok, 1], w.budget), scores[ok, 0]))[0]]
        assert (int(ob_all[b]["move"]), int(ob_all[b]["violations"]), int(ob_all[b]["peak"])) == \
            (int(first), int(scores[first, 0]), int(scores[first, 1])), b
    # best = lexicographic minimum of (violations, max(peak, M), peak, move) over the applicable moves
    ob = moc.results_to_numpy(ob_t, moc.BEST_MOVE_DTYPE)
    for b0 in range(0, w.B, 1024):
        rows = moc.results_to_numpy(om_t[b0:b0 + 8], moc.MOVE_SCORE_DTYPE)
        for j in range(8):
            v, p = rows[j]["violations"].astype(np.int64), rows[j]["peak"].astype(np.int64)
            ok = v >= 0
            key = np.lexsort((np.arange(n_moves)[ok], p[ok], np.maximum(p[ok], w.budget), v[ok]))
            q = int(np.arange(n_moves)[ok][key[0]])
            assert (int(ob[b0 + j]["move"]), int(ob[b0 + j]["violations"]), int(ob[b0 + j]["peak"])) == (q, v[q], p[q])
    # the kernel for the best move alone (which leaves out fields that cannot win) agrees with the
    # kernel that writes the table, on every base
    _, ob_alone = moc.moc_eval_neighbours(gh, ds, de, da, R, want_moves=False)
    torch.cuda.synchronize()
    assert moc.results_to_numpy(ob_alone, moc.BEST_MOVE_DTYPE).tobytes() == ob.tobytes()
    # apply sampled moves and evaluate them as candidates
    b = 5
    row = moc.results_to_numpy(om_t[b], moc.MOVE_SCORE_DTYPE)
    pick = np.flatnonzero(row["violations"] >= 0)
    pick = pick[rng.choice(pick.size, 512, replace=False)]
    s = ds[b].cpu().numpy()[None].repeat(512, 0)
    e = de[b].cpu().numpy()[None].repeat(512, 0)
    a = da[b].cpu().numpy()[None].repeat(512, 0)
    for j, q in enumerate(pick):
        d, field, k = q % (2 * R), (q // (2 * R)) % 2, q // (4 * R)
        delta = d - R if d < R else d - R + 1
        (s if field == 0 else e)[j, k] += delta
    ms, me, ma = to_dev(s, e, a)
    res = moc.results_to_numpy(moc.moc_eval_batch(gh, ms, me, ma))
    assert (res["violations"] == row["violations"][pick]).all() and (res["peak"] == row["peak"][pick]).all()
    gh.free()


def test_neighbours_argument_errors(moc, workloads):
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    w = workloads(0)
    gh = upload(moc, w)
    s, e, a = to_dev(*w.candidates(0, 2))
    for R in (0, 33):
        with pytest.raises(moc.MoccasinError) as err:
            moc.moc_eval_neighbours(gh, s, e, a, R)
        assert err.value.code == -1
    with pytest.raises(moc.MoccasinError):
        moc.moc_eval_neighbours(gh, s, e, a, 4, want_moves=False, want_best=False)
    gh.free()
    # 4.5 words per copy do not fit the LDS for T = 9000
    n = 9000
    g = graph_from_edges(n, [(i, i + 1) for i in range(n - 1)], np.ones(n), np.ones(n))
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 10, 1)
    z = torch.zeros((1, n), dtype=torch.int32, device="cuda")
    with pytest.raises(moc.MoccasinError) as err:
        moc.moc_eval_neighbours(gh, z, z, torch.zeros((1, n), dtype=torch.uint8, device="cuda"), 2)
    assert err.value.code == -2
    gh.free()
    # the toggles keep 4.7 words per copy: T = 10200 is too much for them
    n = 10200
    g = graph_from_edges(n, [(i, i + 1) for i in range(n - 1)], np.ones(n), np.ones(n))
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 10, 1)
    z = torch.zeros((1, n), dtype=torch.int32, device="cuda")
    with pytest.raises(moc.MoccasinError) as err:
        moc.moc_eval_toggles(gh, z, z, torch.zeros((1, n), dtype=torch.uint8, device="cuda"))
    assert err.value.code == -2
    gh.free()
    # self loops are refused by this call only
    g = graph_from_edges(3, [(0, 1), (1, 1)], [1, 1, 1], [1, 1, 1])
    gh = moc.moc_graph_upload(3, g.in_ptr, g.in_idx, g.size, g.dur, 10, 1)
    z = torch.zeros((1, 3), dtype=torch.int32, device="cuda")
    with pytest.raises(moc.MoccasinError) as err:
        moc.moc_eval_neighbours(gh, z, z, torch.ones((1, 3), dtype=torch.uint8, device="cuda"), 2)
    assert err.value.code == -1
    with pytest.raises(moc.MoccasinError) as err:
        moc.moc_eval_toggles(gh, z, z, torch.ones((1, 3), dtype=torch.uint8, device="cuda"))
    assert err.value.code == -1
    gh.free()


@pytest.mark.parametrize("n,C", [(1, 1), (2, 2), (9, 2), (12, 3), (30, 4), (40, 3), (64, 2), (150, 1), (24, 5)])
def test_toggles_small_graphs(moc, n, C):
    """Every toggle of random candidates (wild starts and ends included), of a violation-free
    one and of an empty one, against the oracle's full re-evaluation."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(77 * n + C)
    edges = set()
    for v in range(1, n):
        for u in rng.integers(0, v, size=rng.integers(0, 4)):
            edges.add((int(u), v))
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(1, 9, n))
    T = n * C
    budget = int(g.size.sum()) // 2
    B = 6
    s, e, a = random_candidates(rng, B, T, T, wild=True)
    s[0] = 0; e[0] = 0; a[0] = 0
    for v in range(n):   # a topological order with every copy 0 kept to the end
        s[0, v * C], e[0, v * C], a[0, v * C] = v, T - 1, 1
    a[1] = 0             # nothing active
    long = rng.integers(0, max(T // 8, 1), T)   # long intervals: the block maxima are used when T allows
    s[2] = long; e[2] = np.minimum(T - 1, long + T // 2)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    ds, de, da = to_dev(s, e, a)
    got = moc.results_to_numpy(moc.moc_eval_toggles(gh, ds, de, da), moc.TOGGLE_SCORE_DTYPE)
    for b in range(B):
        want = oracle.toggles(g, budget, C, s[b], e[b], a[b])
        assert (got[b]["violations"].astype(np.int64) == want[:, 0]).all(), (n, C, b)
        assert (got[b]["peak"].astype(np.int64) == want[:, 1]).all(), (n, C, b)
        assert (got[b]["duration"] == want[:, 2]).all(), (n, C, b)
    gh.free()


def test_toggles_workload(moc, workloads):
    """n=2000, C=2 at the full batch: sampled bases against the oracle, and sampled toggles
    applied and evaluated with moc_eval_batch."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(3)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    out = moc.moc_eval_toggles(gh, ds, de, da)
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    for b in (0, w.B // 2 + 1, w.B - 1):
        s, e, a = ds[b].cpu().numpy(), de[b].cpu().numpy(), da[b].cpu().numpy()
        got = moc.results_to_numpy(out[b], moc.TOGGLE_SCORE_DTYPE)
        want = oracle.toggles(w.graph, w.budget, w.C, s, e, a)
        assert (got["violations"].astype(np.int64) == want[:, 0]).all(), b
        assert (got["peak"].astype(np.int64) == want[:, 1]).all(), b
        assert (got["duration"] == want[:, 2]).all(), b
    pb, pk = rng.integers(0, w.B, 256), rng.integers(0, w.T, 256)
    tb, tk = torch.from_numpy(pb).cuda(), torch.from_numpy(pk).cuda()
    s = ds[tb].contiguous(); e = de[tb].contiguous(); a = da[tb].contiguous()
    a[torch.arange(256, device="cuda"), tk] ^= 1
    res = moc.results_to_numpy(moc.moc_eval_batch(gh, s, e, a))
    got = moc.results_to_numpy(out[tb, tk], moc.TOGGLE_SCORE_DTYPE)
    assert (res["violations"] == got["violations"]).all() and (res["peak"] == got["peak"]).all()
    assert (res["duration"] == got["duration"]).all()
    gh.free()


def test_toggles_adjacency_from_global_memory(moc):
    """A graph whose adjacency lists do not fit the LDS beside the base (n = 6000, m = 12000):
    the kernel then reads them from global memory."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(61)
    n, C = 6000, 1
    edges = sorted({(int(u), v) for v in range(1, n) for u in rng.integers(max(0, v - 50), v, size=2)})
    g = graph_from_edges(n, edges, rng.integers(1, 30, n), rng.integers(1, 9, n))
    T = n * C
    s = np.arange(T, dtype=np.int32)[None].repeat(2, 0)
    last = np.arange(T, dtype=np.int32)
    for u, v in edges:
        last[u] = max(last[u], v)
    e = last[None].repeat(2, 0).astype(np.int32)
    a = np.ones((2, T), np.uint8)
    flip = rng.random(T) < 0.2
    a[1, flip] = 0                                     # some nodes dropped: violations to mend
    e[1] = np.minimum(T - 1, e[1] + rng.integers(-3, 4, T)).astype(np.int32)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, int(g.size.sum()), C)
    ds, de, da = to_dev(s, e, a)
    got = moc.results_to_numpy(moc.moc_eval_toggles(gh, ds, de, da), moc.TOGGLE_SCORE_DTYPE)
    for b in range(2):
        want = oracle.toggles(g, int(g.size.sum()), C, s[b], e[b], a[b])
        assert (got[b]["violations"].astype(np.int64) == want[:, 0]).all(), b
        assert (got[b]["peak"].astype(np.int64) == want[:, 1]).all(), b
        assert (got[b]["duration"] == want[:, 2]).all(), b
    gh.free()


def test_neighbours_workload_wide_radius(moc, workloads):
    """R = 16 (64-bit displacement masks) on 512 bases of the n=2000 workload: sampled moves
    against the oracle, the best move against the table, the two kernels against each other."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(3)
    R, Bs = 16, 512
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    ds, de, da = ds[:Bs].contiguous(), de[:Bs].contiguous(), da[:Bs].contiguous()
    om_t, ob_t = moc.moc_eval_neighbours(gh, ds, de, da, R)
    _, ob_alone = moc.moc_eval_neighbours(gh, ds, de, da, R, want_moves=False)
    torch.cuda.synchronize()
    ob = moc.results_to_numpy(ob_t, moc.BEST_MOVE_DTYPE)
    assert moc.results_to_numpy(ob_alone, moc.BEST_MOVE_DTYPE).tobytes() == ob.tobytes()
    n_moves = w.T * 4 * R
    rng = np.random.default_rng(16)
    for b in (0, Bs - 1):
        s, e, a = ds[b].cpu().numpy(), de[b].cpu().numpy(), da[b].cpu().numpy()
        row = moc.results_to_numpy(om_t[b], moc.MOVE_SCORE_DTYPE)
        pick = np.sort(rng.choice(n_moves, 1500, replace=False))
        scores, _ = oracle.neighbours(w.graph, w.budget, w.C, s, e, a, R, moves=pick)
        assert (row["violations"][pick].astype(np.int64) == scores[:, 0]).all(), b
        assert (row["peak"][pick].astype(np.int64) == scores[:, 1]).all(), b
    for b0 in range(0, Bs, 64):
        rows = moc.results_to_numpy(om_t[b0:b0 + 4], moc.MOVE_SCORE_DTYPE)
        for j in range(4):
            v, p = rows[j]["violations"].astype(np.int64), rows[j]["peak"].astype(np.int64)
            ok = np.flatnonzero(v >= 0)
            q = int(ok[np.lexsort((ok, p[ok], v[ok]))[0]])
            assert (int(ob[b0 + j]["move"]), int(ob[b0 + j]["violations"]), int(ob[b0 + j]["peak"])) == (q, v[q], p[q])
    gh.free()


@pytest.mark.parametrize("cfg,count,R,steps", [(0, 40, 8, 6), (0, 12, 3, 12), (1, 3, 8, 3)])
def test_search_moves_follows_the_oracle(moc, workloads, cfg, count, R, steps):
    """Greedy descent by single-field moves: after the same number of steps the starts and ends
    are what the oracle's descent (evaluate + neighbours + apply, step by step) leaves."""
    w = workloads(cfg)
    s, e, a = w.candidates(0, count)
    s0, e0, a0 = w.base()
    s[0], e[0], a[0] = s0, e0, a0
    gh = upload(moc, w)
    ds, de, da = to_dev(s, e, a)
    n_steps = moc.moc_search_moves(gh, ds, de, da, R, steps).cpu().numpy()
    gs, ge = ds.cpu().numpy(), de.cpu().numpy()
    assert (da.cpu().numpy() == a).all()
    for b in range(count):
        k, ws, we = oracle.search_moves(w.graph, w.budget, w.C, s[b], e[b], a[b], R, steps)
        assert n_steps[b] == k, b
        assert (gs[b] == ws).all() and (ge[b] == we).all(), b
    assert n_steps.sum() > 0
    gh.free()


def test_search_moves_full_batch(moc, workloads):
    """n=2000, C=2, all 8192 bases, 4 steps of radius 8: nobody gets worse, whoever moved got
    better in (violations, max(peak, M), peak), durations stay."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(3)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    before = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    steps = moc.moc_search_moves(gh, ds, de, da, w.R, 4).cpu().numpy()
    after = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    key = lambda r: list(zip(r["violations"].tolist(), np.maximum(r["peak"], w.budget).tolist(), r["peak"].tolist()))
    k0, k1 = key(before), key(after)
    assert all((k1[b] < k0[b]) == (steps[b] > 0) and k1[b] <= k0[b] for b in range(w.B))
    assert (after["duration"] == before["duration"]).all()
    assert steps.max() == 4 and (steps > 0).mean() > 0.5
    gh.free()


def test_search_moves_rejects_bad_arguments(moc):
    import ctypes
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(3, [(0, 1), (1, 2)], [1, 1, 1], [1, 1, 1])
    gh = moc.moc_graph_upload(3, g.in_ptr, g.in_idx, g.size, g.dur, 1, 2)
    s = torch.zeros((2, 6), dtype=torch.int32, device="cuda")
    e = torch.zeros((2, 6), dtype=torch.int32, device="cuda")
    a = torch.zeros((2, 6), dtype=torch.uint8, device="cuda")
    res = torch.zeros((2, 24), dtype=torch.uint8, device="cuda")
    best = torch.zeros((2, 16), dtype=torch.uint8, device="cuda")
    steps = torch.full((2,), 9, dtype=torch.int32, device="cuda")
    L = moc.lib()
    vp = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    call = lambda R, n, r, b, st: L.moc_search_moves(gh._h, 2, vp(s), vp(e), vp(a), R, n, r, b, st, None)
    assert call(0, 1, vp(res), vp(best), vp(steps)) == -1
    assert call(33, 1, vp(res), vp(best), vp(steps)) == -1
    assert call(2, -1, vp(res), vp(best), vp(steps)) == -1
    assert call(2, 1, None, vp(best), vp(steps)) == -1
    assert call(2, 1, vp(res), None, vp(steps)) == -1
    assert call(2, 1, vp(res), vp(best), None) == -1
    assert call(2, 1, vp(res, 4), vp(best), vp(steps)) == -1
    assert (steps.cpu().numpy() == 9).all()
    assert call(2, 0, vp(res), vp(best), vp(steps)) == 0 and (steps.cpu().numpy() == 0).all()
    assert L.moc_search_moves(gh._h, 0, None, None, None, 2, 1, None, None, None, None) == 0
    gh.free()
