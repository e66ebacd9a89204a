"""GPU parity of moc_eval_batch_staged (stage-restricted domain, Section 2.3 of arXiv
2304.14463) against the oracle's evaluate_staged: bit-exact on every field, through the C ABI."""
import numpy as np
import pytest

import oracle
from helpers import F, assert_results_equal
from paper_2304_14463_amd.inputs.staged import gen_staged_candidates, slot_position, staged_base, staged_tables

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


def oracle_staged_parallel(g, budget, C, index, s, e, a, threads=16):
    from concurrent.futures import ThreadPoolExecutor
    B = s.shape[0]
    cuts = np.linspace(0, B, min(threads, B) + 1).astype(int)
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda i: oracle.evaluate_staged(g, budget, C, index, s[cuts[i]:cuts[i + 1]],
                                                             e[cuts[i]:cuts[i + 1]], a[cuts[i]:cuts[i + 1]]),
                            range(len(cuts) - 1)))
    return np.vstack(parts)


@pytest.mark.parametrize("cfg,B", [(0, 1024), (1, 2048), (2, 512)])
def test_staged_parity_workloads(moc, workloads, cfg, B):
    """The graphs, orders and budgets of the first three workloads with staged candidates: half
    violation-free recomputation schedules, half perturbed."""
    w = workloads(cfg)
    tables = staged_tables(w.graph, w.order)
    index = tables[0]
    s, e, a = gen_staged_candidates(w.seed, w.graph, w.order, w.C, B, 0, B, tables)
    s[0], e[0], a[0] = staged_base(w.n, w.C, *tables[:3])
    g = w.graph
    gh = moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, w.budget, w.C)
    moc.moc_graph_set_order(gh, w.order)
    ds, de, da = to_dev(s, e, a)
    gpu = moc.results_to_numpy(moc.moc_eval_batch_staged(gh, ds, de, da))
    ref = oracle_staged_parallel(g, w.budget, w.C, index, s, e, a)
    assert_results_equal(gpu, ref, f"staged cfg {cfg}")
    assert (gpu["violations"][0], gpu["peak"][0], gpu["duration"][0]) == (0, w.no_remat_peak, int(g.dur.sum()))
    assert (ref[: B // 2, F["violations"]] == 0).all() and (ref[B // 2:, F["violations"]] > 0).mean() > 0.9
    # a budget that splits the violation-free half
    clean = ref[:, F["violations"]] == 0
    mid = int(np.median(ref[clean, F["peak"]]))
    gh2 = moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, mid, w.C)
    moc.moc_graph_set_order(gh2, w.order)
    gpu2 = moc.results_to_numpy(moc.moc_eval_batch_staged(gh2, ds, de, da))
    want = (clean & (ref[:, F["peak"]] <= mid)).astype(np.int64)
    assert (gpu2["feasible"] == want).all() and 0 < want.sum() < clean.sum() + 1
    # determinism
    again = moc.results_to_numpy(moc.moc_eval_batch_staged(gh, ds, de, da))
    assert again.tobytes() == gpu.tobytes()
    gh.free(); gh2.free()


def test_staged_worked_example(moc):
    """The example of Section 2 as printed (events 1, 3, 6, 7, 10 of the 10-event axis)."""
    from test_oracle_pins import worked_example
    kv, g, C, T, s, e, a = worked_example([1, 1, 1, 1], [3, 5, 7, 11])
    gh = moc.moc_graph_upload(4, g.in_ptr, g.in_idx, g.size, g.dur, 3, C)
    moc.moc_graph_set_order(gh, [0, 1, 2, 3])
    s2 = s.copy(); s2[1] = 7          # node 1 recomputed at event 8: not its slot
    ds, de, da = to_dev(np.stack([s, s2]), np.stack([e, e]), np.stack([a, a]))
    got = moc.results_to_numpy(moc.moc_eval_batch_staged(gh, ds, de, da))
    assert (got["violations"][0], got["peak"][0], got["duration"][0], got["feasible"][0]) == (0, 3, 2 * 3 + 5 + 7 + 11, 1)
    assert (got["violations"][1], got["peak"][1], got["duration"][1], got["feasible"][1]) == (2, 2, 2 * 3 + 5 + 7 + 11, 0)
    gh.free()


@pytest.mark.parametrize("n,C", [(1, 1), (2, 2), (3, 3), (7, 1), (13, 3), (40, 4), (64, 2), (65, 3), (130, 5),
                                 (513, 2), (700, 3), (1025, 1), (1500, 2), (4000, 2)])
def test_staged_ragged_shapes_random_values(moc, n, C):
    """Random DAGs, a random topological order, and candidates with starts on and off their
    slots, first copies on and off their fixed start, ends anywhere, values outside the domain,
    flags at random, several copies of a node on one event, ends on the first position of a stage
    and on the position before it (up to 8 million positions at n = 4000)."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(n * 17 + C)
    edges = set()
    for v in range(1, n):
        for u in rng.integers(0, v, size=rng.integers(0, 4)):
            edges.add((int(u), v))
    if n > 40:
        edges |= {(u, n - 1) for u in range(0, n - 1, 2)} | {(0, v) for v in range(1, n, 3)}
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 1000, n), rng.integers(0, 50, n))
    # a random topological order: ids are topological; shuffle within the constraint by random keys
    key = rng.random(n)
    order, placed, indeg = [], set(), [int(g.in_ptr[v + 1] - g.in_ptr[v]) for v in range(n)]
    cons = g.consumers()
    ready = sorted((v for v in range(n) if indeg[v] == 0), key=lambda v: key[v])
    while ready:
        v = ready.pop(0)
        order.append(v)
        for w_ in cons[v]:
            indeg[w_] -= 1
            if indeg[w_] == 0:
                ready.append(w_)
                ready.sort(key=lambda x: key[x])
    index = np.zeros(n, np.int32)
    index[order] = np.arange(n)
    D = n * (n + 1) // 2
    B = 24 if n <= 2000 else 6
    K = n * C
    s = rng.integers(-2, D + 2, size=(B, K)).astype(np.int64)
    on = rng.random((B, K)) < 0.8
    stage = np.maximum(index[None, :, None], rng.integers(0, n, size=(B, n, C)))
    stage[:, :, 0] = np.where(rng.random((B, n)) < 0.9, index[None, :], stage[:, :, 0])
    slot_pos = (stage * (stage + 1) // 2 + index[None, :, None]).reshape(B, K)
    s = np.where(on, slot_pos, s)
    e = s + rng.integers(-1, max(2, D // 3), size=(B, K))
    e = np.where(rng.random((B, K)) < 0.1, rng.integers(-2, D + 2, size=(B, K)), e)
    later = rng.integers(stage.reshape(B, K), n + 1)   # a stage not before the start's (n: one past the last)
    edge_of_stage = later * (later + 1) // 2 - rng.integers(0, 2, size=(B, K))
    e = np.where(rng.random((B, K)) < 0.2, edge_of_stage, e)
    a = ((rng.random((B, K)) < 0.7) * rng.integers(1, 256, size=(B, K))).astype(np.uint8)
    s, e = s.astype(np.int32), e.astype(np.int32)
    # row 0: the plain schedule; row 1: every copy of a node on the node's fixed start
    tables = staged_tables(g, order)
    s[0], e[0], a[0] = staged_base(n, C, *tables[:3])
    fixed = (index * (index + 1) // 2 + index).astype(np.int32)
    s[1] = np.repeat(fixed, C); e[1] = D - 1; a[1] = 1
    budget = int(g.size.sum()) // 2
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    moc.moc_graph_set_order(gh, order)
    ds, de, da = to_dev(s, e, a)
    gpu = moc.results_to_numpy(moc.moc_eval_batch_staged(gh, ds, de, da))
    ref = oracle.evaluate_staged(g, budget, C, index, s, e, a)
    assert_results_equal(gpu, ref, f"staged n={n} C={C}")
    assert ref[0, F["violations"]] == 0
    assert ref[1, F["v_start"]] == n * (C - 1)
    # the same rows at odd addresses: the kernel reads a node's copies in one load per array
    import torch
    pad_s = torch.zeros(B * K + 1, dtype=torch.int32, device="cuda")
    pad_e = torch.zeros(B * K + 3, dtype=torch.int32, device="cuda")
    pad_a = torch.zeros(B * K + 1, dtype=torch.uint8, device="cuda")
    pad_s[1:], pad_e[3:], pad_a[1:] = ds.reshape(-1), de.reshape(-1), da.reshape(-1)
    gpu = moc.results_to_numpy(moc.moc_eval_batch_staged(gh, pad_s[1:], pad_e[3:], pad_a[1:]))
    assert_results_equal(gpu, ref, f"staged n={n} C={C}, arrays at odd addresses")
    gh.free()


def test_staged_argument_errors(moc):
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(4, [(0, 1), (1, 2), (2, 3), (0, 3)], [1, 1, 1, 1], [1, 1, 1, 1])
    gh = moc.moc_graph_upload(4, g.in_ptr, g.in_idx, g.size, g.dur, 3, 2)
    z = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    a = torch.ones((1, 8), dtype=torch.uint8, device="cuda")
    with pytest.raises(moc.MoccasinError) as err:      # no order yet
        moc.moc_eval_batch_staged(gh, z, z, a)
    assert err.value.code == -1
    for bad in ([0, 1, 2, 2], [0, 1, 2, 4], [1, 0, 2, 3], [0, 2, 1, 3]):   # not a permutation / not topological
        with pytest.raises(moc.MoccasinError) as err:
            moc.moc_graph_set_order(gh, bad)
        assert err.value.code == -1
    moc.moc_graph_set_order(gh, [0, 1, 2, 3])
    moc.moc_eval_batch_staged(gh, z, z, a)
    moc.moc_graph_set_order(gh, [0, 1, 2, 3])          # setting it again is allowed
    empty = torch.zeros((0, 8), dtype=torch.int32, device="cuda")
    assert moc.moc_eval_batch_staged(gh, empty, empty, torch.zeros((0, 8), dtype=torch.uint8, device="cuda")).shape[0] == 0
    gh.free()
    # too large for this call's LDS layout
    n = 9000
    g = graph_from_edges(n, [(i, i + 1) for i in range(n - 1)], np.ones(n), np.ones(n))
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 10, 2)
    moc.moc_graph_set_order(gh, np.arange(n))
    z = torch.zeros((1, 2 * n), dtype=torch.int32, device="cuda")
    with pytest.raises(moc.MoccasinError) as err:
        moc.moc_eval_batch_staged(gh, z, z, torch.zeros((1, 2 * n), dtype=torch.uint8, device="cuda"))
    assert err.value.code == -2
    gh.free()
