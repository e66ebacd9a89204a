"""Randomised parity sweeps: moc_eval_batch, moc_eval_neighbours, moc_eval_cuts
(table and best move), moc_eval_toggles, moc_search_cuts, moc_search_moves and
moc_decode_batch against the oracle on a few hundred small random graphs with
1 to 5 copies per node, orderly and wild candidates."""
import numpy as np
import pytest

import oracle
import test_gpu_cuts as tc
import test_gpu_decode as td

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moc():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2304_14463_amd import moccasin
    moccasin.lib()
    return moccasin


@pytest.mark.parametrize("first", [0, 100, 200])
def test_sweep(moc, first):
    from paper_2304_14463_amd.inputs import graph_from_edges
    for seed in range(first, first + 100):
        rng = np.random.default_rng(seed)
        n = int(rng.integers(2, 70 if seed % 10 else 300))
        C = int(rng.integers(1, 5))
        edges = []
        for v in range(1, n):
            for u in rng.integers(0, v, size=rng.integers(0, 4)):
                edges.append((int(u), v))
        if rng.random() < 0.5:
            edges = sorted(set(edges))           # otherwise duplicate edges stay
        g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(0, 9, n))
        budget = int(g.size.sum() * rng.random())
        B = 6
        s, e, a = tc.schedules(rng, g, C, B, wild=bool(seed % 2))
        gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
        ds, de, da = tc.to_dev(s, e, a)
        if edges:
            got, best = tc.gpu_cuts(moc, gh, ds, de, da)
            for b in range(B):
                want = oracle.cuts(g, budget, C, s[b], e[b], a[b], with_at_peak=True)
                tc.assert_same(got[b], want, f"seed {seed} cuts row {b}")
                tc.assert_best(best[b], want, f"seed {seed} best cut row {b}")
        tg = moc.results_to_numpy(moc.moc_eval_toggles(gh, ds, de, da), moc.TOGGLE_SCORE_DTYPE)
        for b in range(B):
            want = oracle.toggles(g, budget, C, s[b], e[b], a[b])
            for i, name in enumerate(("violations", "peak", "duration")):
                assert (tg[b][name].astype(np.int64) == want[:, i]).all(), (seed, "toggles", b, name)
        ws, we, wa = ds.clone(), de.clone(), da.clone()
        steps = moc.moc_search_cuts(gh, ws, we, wa, 5).cpu().numpy()
        for b in range(B):
            k, s2, e2, a2 = oracle.search_cuts(g, budget, C, s[b], e[b], a[b], 5)
            assert steps[b] == k, (seed, "search", b)
            assert (wa[b].cpu().numpy() == a2).all() and (ws[b].cpu().numpy() == s2).all(), (seed, "search", b)
            assert (we[b].cpu().numpy() == e2).all(), (seed, "search", b)
        if n < 70:
            R = int(rng.integers(1, 6))
            ws, we = ds[:3].clone(), de[:3].clone()
            steps = moc.moc_search_moves(gh, ws, we, da[:3].contiguous(), R, 3).cpu().numpy()
            for b in range(3):
                k, s2, e2 = oracle.search_moves(g, budget, C, s[b], e[b], a[b], R, 3)
                assert steps[b] == k, (seed, "moves", b)
                assert (ws[b].cpu().numpy() == s2).all() and (we[b].cpu().numpy() == e2).all(), (seed, "moves", b)
        for cs, ca in ((td.orderly_candidates(rng, g, C, 8)), (s, a)):
            want, want_seq = oracle.decode(g, C, cs, ca)
            got, seq = td.gpu_decode(moc, gh, cs, ca)
            td.assert_same(got, seq, want, want_seq, f"seed {seed} decode")
        gh.free()


def test_sweep_evaluator_and_neighbourhood(moc):
    """moc_eval_batch and moc_eval_neighbours (table, best move, best move alone) on 150 random
    graphs with 1 to 5 copies per node, random batch sizes, radii up to 32."""
    import test_gpu_eval as te
    import test_gpu_neighbours as tn
    from helpers import assert_results_equal
    from paper_2304_14463_amd.inputs import graph_from_edges
    for seed in range(150):
        rng = np.random.default_rng(10_000_000 + seed)
        n = int(rng.integers(1, 90 if seed % 8 else 700))
        C = int(rng.integers(1, 6))
        edges = set()
        for v in range(1, n):
            for u in rng.integers(0, v, size=rng.integers(0, 4)):
                edges.add((int(u), v))
        g = graph_from_edges(n, sorted(edges), rng.integers(0, 1000, n), rng.integers(0, 50, n))
        T, B = n * C, int(rng.integers(1, 40))
        s, e, a = te.random_candidates(rng, B, n, C, T, wild=bool(seed % 2))
        budget = int(g.size.sum() * rng.random())
        gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
        ref = oracle.evaluate(g, budget, C, s, e, a)
        assert_results_equal(te.run_eval(moc, gh, s, e, a), ref, f"seed {seed} n={n} C={C}")
        if n < 90:
            R = int(rng.integers(1, 33 if seed % 5 == 0 else 9))
            nb = min(B, 3)
            om, ob = tn.gpu_neighbours(moc, gh, s[:nb], e[:nb], a[:nb], R)
            _, alone = tn.gpu_neighbours(moc, gh, s[:nb], e[:nb], a[:nb], R, moves=False)
            for b in range(nb):
                scores, bm = oracle.neighbours(g, budget, C, s[b], e[b], a[b], R)
                assert (om[b]["violations"] == scores[:, 0]).all() and (om[b]["peak"] == scores[:, 1]).all(), (seed, b)
                assert (int(ob[b]["move"]), int(ob[b]["violations"]), int(ob[b]["peak"])) == bm, (seed, b)
                assert (int(alone[b]["move"]), int(alone[b]["violations"]), int(alone[b]["peak"])) == bm, (seed, b)
        gh.free()
