"""GPU parity of moc_eval_batch against the CPU oracle: bit-exact on every
field, through the C ABI (ctypes binding), on the five synthetic workloads and
on edge-case shapes."""
import numpy as np
import pytest

from helpers import F, assert_results_equal, oracle_eval_parallel, upload

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


def run_eval(moc, gh, s, e, a):
    ds, de, da = to_dev(s, e, a)
    return moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))


# ---------------------------------------------------------------- the device generator emits the host's bits
@pytest.mark.parametrize("cfg,dense", [(0, False), (1, False), (2, False), (3, False), (4, False), (1, True), (4, True)])
def test_device_generator_matches_host(workloads, cfg, dense):
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload, make_workload
    w = make_workload(cfg, dense=True) if dense else workloads(cfg)
    dw = DeviceWorkload(w)
    count = min(w.B, 2048 if cfg < 4 else 256)
    for b0 in (0, w.B // 2 - count // 2, w.B - count):
        s, e, a = w.candidates(b0, count)
        ds, de, da = dw.candidates(b0, count)
        torch.cuda.synchronize()
        assert (ds.cpu().numpy() == s).all() and (de.cpu().numpy() == e).all() and (da.cpu().numpy() == a).all()


# ---------------------------------------------------------------- full workloads
@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_eval_parity_full_batch(moc, workloads, cfg):
    """Configs 0-3 at their full batch size, every candidate compared."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(cfg)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    gpu = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    s, e, a = ds.cpu().numpy(), de.cpu().numpy(), da.cpu().numpy()
    ref = oracle_eval_parallel(w.graph, w.budget, w.C, s, e, a)
    assert_results_equal(gpu, ref, f"cfg {cfg}")
    assert (ref[:, F["violations"]] == 0).any() and (ref[:, F["violations"]] > 0).any()
    # same batch under a budget that splits the violation-free candidates
    clean = ref[:, F["violations"]] == 0
    mid = int(np.median(ref[clean, F["peak"]]))
    gh2 = upload(moc, w, budget=mid)
    gpu2 = moc.results_to_numpy(moc.moc_eval_batch(gh2, ds, de, da))
    want = (clean & (ref[:, F["peak"]] <= mid)).astype(np.int64)
    assert (gpu2["feasible"] == want).all() and 0 < want.sum() < len(want)
    # determinism: a second launch returns the same bytes
    again = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    assert gpu.tobytes() == again.tobytes()
    gh.free(); gh2.free()
    torch.cuda.synchronize()


@pytest.mark.timeout(900)
def test_eval_parity_largest_workload_every_candidate(moc, workloads):
    """Config 4 (n=5000, C=3, T=15000) as the benchmark runs it: all 262144 candidates
    (35.4 GB) resident in HBM, one launch; every one of them is compared with the oracle,
    which takes them from the device in slices of 2.2 GB and splits a slice over the host's
    threads."""
    import os
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(4)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    gpu = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    threads = min(os.cpu_count() or 8, 16)
    step = 16384
    n_clean = 0
    for b0 in range(0, w.B, step):
        s, e, a = ds[b0:b0 + step].cpu().numpy(), de[b0:b0 + step].cpu().numpy(), da[b0:b0 + step].cpu().numpy()
        ref = oracle_eval_parallel(w.graph, w.budget, w.C, s, e, a, threads=threads)
        assert_results_equal(gpu[b0:b0 + step], ref, f"cfg 4, candidates {b0}..")
        n_clean += int((ref[:, F["violations"]] == 0).sum())
        print(f"cfg 4: {b0 + len(ref)} of {w.B} candidates compared", flush=True)
    assert 0 < n_clean < w.B
    assert (gpu["violations"][: w.B // 2] < gpu["violations"][w.B // 2:].mean()).mean() > 0.99   # type A vs type B
    # the same batch under a budget that splits the violation-free candidates: feasible = 1 occurs
    clean = gpu["violations"] == 0
    mid = int(np.median(gpu["peak"][clean]))
    gh2 = upload(moc, w, budget=mid)
    gpu2 = moc.results_to_numpy(moc.moc_eval_batch(gh2, ds, de, da))
    want = (clean & (gpu["peak"] <= mid)).astype(np.int32)   # gpu's peaks and counts equal the oracle's, shown above
    assert (gpu2["feasible"] == want).all() and 0 < want.sum() < clean.sum() + 1
    for name in ("peak", "duration", "violations"):
        assert (gpu2[name] == gpu[name]).all(), name
    gh2.free()
    # the same rows evaluated as a separate, smaller launch give the same bytes
    sub = moc.results_to_numpy(moc.moc_eval_batch(gh, ds[1000:1300], de[1000:1300], da[1000:1300]))
    assert sub.tobytes() == gpu[1000:1300].tobytes()
    del ds, de, da
    gh.free()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg,B", [(1, 4096), (2, 4096), (4, 2048)])
def test_eval_parity_dense_batch(moc, cfg, B):
    """The dense batch (more than 90 % of all copies live, every node computed up to C times):
    the paths for copies beyond the first carry most of the work."""
    from paper_2304_14463_amd.inputs import DeviceWorkload, make_workload
    w = make_workload(cfg, B, dense=True)
    gh = upload(moc, w)
    ds, de, da = DeviceWorkload(w).candidates()
    gpu = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    s, e, a = ds.cpu().numpy(), de.cpu().numpy(), da.cpu().numpy()
    assert (a != 0).mean() > 0.9
    ref = oracle_eval_parallel(w.graph, w.budget, w.C, s, e, a)
    assert_results_equal(gpu, ref, f"cfg {cfg} dense")
    assert (ref[: B // 2, F["violations"]] == 0).all() and (ref[B // 2:, F["violations"]] > 0).mean() > 0.9
    gh.free()


def test_stream_read_runs(moc):
    """The read-only kernel the benchmark times beside the evaluator: it reads three arrays and
    writes one word per thread; the XOR of what it wrote is the XOR of the words it read."""
    import torch
    from paper_2304_14463_amd.inputs import stream_read
    g = torch.Generator(device="cuda").manual_seed(5)
    x = [torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device="cuda", generator=g) for n in (40000, 40004, 8)]
    out = stream_read(x, 7)
    torch.cuda.synchronize()
    want = 0
    for t in x:
        n = t.numel() // 4 * 4
        want ^= int(np.bitwise_xor.reduce(t[:n].cpu().numpy().view(np.uint32)))
    assert int(np.bitwise_xor.reduce(out.cpu().numpy().view(np.uint32))) == want


# ---------------------------------------------------------------- edge cases
def random_candidates(rng, B, n, C, T, wild):
    """Uniformly random (mostly broken) candidates; `wild` adds out-of-domain values."""
    lo, hi = (-3, T + 3) if wild else (0, T)
    s = rng.integers(lo, hi, size=(B, n * C)).astype(np.int32)
    e = rng.integers(lo, hi, size=(B, n * C)).astype(np.int32)
    swap = (rng.random((B, n * C)) < 0.7) & (s > e)
    s, e = np.where(swap, e, s).astype(np.int32), np.where(swap, s, e).astype(np.int32)
    a = (rng.random((B, n * C)) < 0.6).astype(np.uint8) * rng.integers(1, 256, size=(B, n * C)).astype(np.uint8)
    return s, e, a


@pytest.mark.parametrize("n,C", [(1, 1), (1, 3), (2, 2), (7, 1), (13, 3), (21, 5), (64, 2), (65, 3), (100, 7),
                                 (341, 3), (513, 2), (1025, 1), (1031, 2), (1537, 4), (2049, 3), (3000, 6),
                                 (255, 4), (256, 4), (320, 4), (511, 4), (512, 4), (640, 2), (640, 3)])
def test_eval_ragged_shapes_random_candidates(moc, n, C):
    """Shapes around every tile boundary (wave of 64 nodes, 4 copies per lane, workgroup
    sizes, rows whose byte length is not a multiple of 16, the sizes at which small workgroups
    run out of delta chunks of 16 positions) with random DAGs and random,
    mostly infeasible candidates including out-of-domain positions and a > 1."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(n * 131 + C)
    edges = set()
    for v in range(1, n):
        for u in rng.integers(0, v, size=rng.integers(0, 4)):
            edges.add((int(u), v))
    if n > 40:   # one node with a very high in-degree, one with a very high out-degree
        edges |= {(u, n - 1) for u in range(0, n - 1, 2)} | {(0, v) for v in range(1, n, 3)}
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 1000, n), rng.integers(0, 50, n))
    T = n * C
    B = 37
    s, e, a = random_candidates(rng, B, n, C, T, wild=True)
    # a few structured rows: everything active on [0,T-1]; all ends equal; only first copies
    s[0], e[0], a[0] = 0, T - 1, 1
    e[1] = T - 1
    a[2].reshape(n, C)[:, 1:] = 0
    a[2].reshape(n, C)[:, 0] = 1
    budget = int(g.size.sum()) // 2
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    import oracle
    ref = oracle.evaluate(g, budget, C, s, e, a)
    assert_results_equal(run_eval(moc, gh, s, e, a), ref, f"n={n} C={C}")
    # unaligned views of the same rows (element-wise load path)
    import torch
    pad_s = torch.zeros(B * T + 1, dtype=torch.int32, device="cuda")
    pad_e = torch.zeros(B * T + 1, dtype=torch.int32, device="cuda")
    pad_a = torch.zeros(B * T + 1, dtype=torch.uint8, device="cuda")
    pad_s[1:] = torch.from_numpy(s.reshape(-1)).cuda()
    pad_e[1:] = torch.from_numpy(e.reshape(-1)).cuda()
    pad_a[1:] = torch.from_numpy(a.reshape(-1)).cuda()
    out = moc.moc_eval_batch(gh, pad_s[1:], pad_e[1:], pad_a[1:])
    assert_results_equal(moc.results_to_numpy(out), ref, f"n={n} C={C} unaligned")
    gh.free()



@pytest.mark.parametrize("n,m,C", [(64, 100, 2), (64, 250, 2), (64, 300, 1), (64, 380, 2), (128, 700, 2),
                                   (128, 850, 1), (256, 2300, 2), (256, 2700, 2)])
def test_eval_partial_last_slice_of_edges(moc, n, m, C):
    """Graphs whose edge count, not their node count, sets the number of edge slices per lane,
    with a last slice that holds edges in one, two or all three of its entries (C <= 2: the
    kernel has a block of its own for each case)."""
    from paper_2304_14463_amd.inputs import graph_from_edges
    import oracle
    rng = np.random.default_rng(n * 7 + m)
    edges = set()
    while len(edges) < m:
        v = int(rng.integers(1, n))
        edges.add((int(rng.integers(0, v)), v))
    g = graph_from_edges(n, sorted(edges), rng.integers(1, 1000, n), rng.integers(1, 50, n))
    T = n * C
    B = 64
    s, e, a = random_candidates(rng, B, n, C, T, wild=False)
    # half of the rows close to a schedule: node v computed at v*C and kept to the end, so that
    # most edges are satisfied and the unsatisfied ones stand out
    base = np.repeat(np.arange(n) * C, C).astype(np.int32)
    s[::2], e[::2] = base, T - 1
    a[::2].reshape(-1, n, C)[:, :, 1:] = 0
    a[::2].reshape(-1, n, C)[:, :, 0] = 1
    s[2::4] += rng.integers(0, 3, size=s[2::4].shape).astype(np.int32) * (s[2::4] + 3 < T)
    budget = int(g.size.sum()) // 2
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    ref = oracle.evaluate(g, budget, C, s, e, a)
    assert ref[0, F["violations"]] == 0 and ref[:, F["v_prec"]].max() > 0
    assert_results_equal(run_eval(moc, gh, s, e, a), ref, f"n={n} m={m} C={C}")
    gh.free()


@pytest.mark.parametrize("n,C,B", [(96, 3, 40000), (200, 2, 50000), (96, 3, 3000)])
def test_eval_many_launches_one_graph(moc, n, C, B):
    """Launches share the graph's work counters, which every launch must leave at zero: 40
    launches of the same batch in a row, alternating between two streams, all return the bytes
    of the first, which match the oracle.  The long batches are handed out dynamically, the
    short one is split statically."""
    import torch
    import oracle
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(n * 7 + C)
    edges = sorted({(int(u), v) for v in range(1, n) for u in rng.integers(0, v, size=3)})
    g = graph_from_edges(n, edges, rng.integers(1, 100, n), rng.integers(1, 9, n))
    T = n * C
    s, e, a = random_candidates(rng, B, n, C, T, wild=False)
    a.reshape(B, n, C)[:, :, 0] = 1
    a.reshape(B, n, C)[:, :, 1:] *= (rng.random((B, n, C - 1)) < 0.1)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, int(g.size.sum()) // 3, C)
    ds, de, da = to_dev(s, e, a)
    first = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    assert_results_equal(first, oracle_eval_parallel(g, int(g.size.sum()) // 3, C, s, e, a), f"n={n} C={C}")
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    outs = []
    for i in range(40):
        with torch.cuda.stream(streams[i % 2]):
            outs.append(moc.moc_eval_batch(gh, ds, de, da, stream=streams[i % 2]))
    torch.cuda.synchronize()
    for i, out in enumerate(outs):
        assert moc.results_to_numpy(out).tobytes() == first.tobytes(), f"launch {i} differs"
    gh.free()


def test_eval_streams_do_not_share_work_counters(moc):
    """A long launch on one stream while many short ones run on another, on one graph handle:
    a stream keeps the set of work counters it was given, so the short launches never draw
    from the counters of the long one.  Then launches on more streams than the handle has
    sets: those are split statically.  Every output equals the oracle's."""
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    n, C, B, reps = 96, 3, 40000, 24
    rng = np.random.default_rng(77)
    edges = sorted({(int(u), v) for v in range(1, n) for u in rng.integers(0, v, size=3)})
    g = graph_from_edges(n, edges, rng.integers(1, 100, n), rng.integers(1, 9, n))
    T = n * C
    s, e, a = random_candidates(rng, B, n, C, T, wild=False)
    a.reshape(B, n, C)[:, :, 0] = 1
    budget = int(g.size.sum()) // 3
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, budget, C)
    ds, de, da = to_dev(s, e, a)
    first = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    assert_results_equal(first, oracle_eval_parallel(g, budget, C, s, e, a), "short batch")
    ls, le, la = ds.repeat(reps, 1), de.repeat(reps, 1), da.repeat(reps, 1)   # the long batch: the same rows 24 times
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(sa):
        long_out = moc.moc_eval_batch(gh, ls, le, la, stream=sa)
    shorts = []
    with torch.cuda.stream(sb):
        for i in range(40):
            shorts.append(moc.moc_eval_batch(gh, ds, de, da, stream=sb))
    torch.cuda.synchronize()
    assert moc.results_to_numpy(long_out).tobytes() == np.tile(first, reps).tobytes(), "long launch"
    for i, out in enumerate(shorts):
        assert moc.results_to_numpy(out).tobytes() == first.tobytes(), f"short launch {i}"
    # the same again with the long launch issued in the middle of the short ones
    with torch.cuda.stream(sb):
        shorts = [moc.moc_eval_batch(gh, ds, de, da, stream=sb) for _ in range(10)]
    with torch.cuda.stream(sa):
        long_out = moc.moc_eval_batch(gh, ls, le, la, stream=sa)
    with torch.cuda.stream(sb):
        shorts += [moc.moc_eval_batch(gh, ds, de, da, stream=sb) for _ in range(30)]
    torch.cuda.synchronize()
    assert moc.results_to_numpy(long_out).tobytes() == np.tile(first, reps).tobytes(), "long launch, second time"
    for i, out in enumerate(shorts):
        assert moc.results_to_numpy(out).tobytes() == first.tobytes(), f"short launch {i}, second time"
    # 24 more streams on the same handle: more than it has sets of counters
    streams = [torch.cuda.Stream() for _ in range(24)]
    outs = []
    for st in streams:
        with torch.cuda.stream(st):
            outs.append(moc.moc_eval_batch(gh, ds, de, da, stream=st))
    torch.cuda.synchronize()
    for i, out in enumerate(outs):
        assert moc.results_to_numpy(out).tobytes() == first.tobytes(), f"stream {i}"
    gh.free()


def test_eval_empty_batch_and_single_candidate(moc, workloads):
    import torch
    w = workloads(0)
    gh = upload(moc, w)
    empty = [torch.empty((0, w.T), dtype=dt, device="cuda") for dt in (torch.int32, torch.int32, torch.uint8)]
    out = moc.moc_eval_batch(gh, *empty)
    assert out.shape[0] == 0
    s, e, a = w.base()
    got = run_eval(moc, gh, s[None], e[None], a[None])
    assert (got["violations"][0], got["peak"][0], got["duration"][0], got["feasible"][0]) == \
        (0, w.no_remat_peak, int(w.graph.dur.sum()), 0)
    gh.free()


def test_eval_maximum_size(moc):
    """T at the library's limit (the LDS working set of one candidate fills a compute unit)."""
    import oracle
    from paper_2304_14463_amd.inputs import graph_from_edges
    n, C = moc.MOC_MAX_T, 1
    rng = np.random.default_rng(7)
    edges = [(int(rng.integers(max(0, v - 50), v)), v) for v in range(1, n)]
    g = graph_from_edges(n, edges, rng.integers(1, 100, n), rng.integers(1, 9, n))
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 10**6, C)
    s = np.tile(np.arange(n, dtype=np.int32), (3, 1))
    e = np.minimum(s + rng.integers(0, 60, size=s.shape), n - 1).astype(np.int32)
    a = np.ones_like(s, dtype=np.uint8)
    s[1, 100] = s[1, 99]; e[2, 5000] = n   # one collision, one malformed copy
    ref = oracle.evaluate(g, 10**6, C, s, e, a)
    assert_results_equal(run_eval(moc, gh, s, e, a), ref, "T = MOC_MAX_T")
    gh.free()
    # one more copy per node does not fit
    with pytest.raises(moc.MoccasinError) as err:
        moc.moc_graph_upload(n + 1, np.zeros(n + 2, np.int32), np.zeros(0, np.int32), np.ones(n + 1, np.int32),
                             np.ones(n + 1, np.int32), 1, 1)
    assert err.value.code == -2


@pytest.mark.parametrize("C", [2, 3, 4])
def test_eval_largest_graph_per_copy_count(moc, C):
    """The largest n that moc_graph_upload accepts for C copies (the LDS working set decides;
    the optional buffers of the kernel are at their smallest there), with candidates in which
    many nodes have several live copies and some have none."""
    import oracle
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(100 + C)

    def make(n):
        edges = sorted({(int(u), v) for v in range(1, n) for u in rng.integers(max(0, v - 40), v, size=2)})
        return graph_from_edges(n, edges, rng.integers(1, 100, n), rng.integers(1, 9, n))

    def accepted(n):
        g = make(n)
        try:
            moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 10**6, C).free()
            return True
        except moc.MoccasinError as err:
            assert err.code == -2
            return False

    lo, hi = 1000, moc.MOC_MAX_T // C + 1   # accepted(lo), not accepted(hi)
    assert accepted(lo)
    if accepted(hi - 1):
        lo = hi - 1
    while hi - lo > 1 and lo < hi - 1:
        mid = (lo + hi) // 2
        if accepted(mid):
            lo = mid
        else:
            hi = mid
    n = lo
    assert n * C > 9000, f"unexpectedly small limit: n = {n}"
    g = make(n)
    T = n * C
    B = 6
    s, e, a = random_candidates(rng, B, n, C, T, wild=True)
    a.reshape(B, n, C)[:3, :, 0] = 1                        # rows 0-2: every first copy active
    a.reshape(B, n, C)[:2, :, 1:] *= (rng.random((2, n, C - 1)) < 0.05)   # rows 0-1: few other copies
    s[0].reshape(n, C)[:, 0] = np.arange(n) * C             # row 0: first copies well-formed
    e[0].reshape(n, C)[:, 0] = np.minimum(np.arange(n) * C + rng.integers(0, 90, n), T - 1)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, int(g.size.sum()) // 4, C)
    ref = oracle.evaluate(g, int(g.size.sum()) // 4, C, s, e, a)
    assert_results_equal(run_eval(moc, gh, s, e, a), ref, f"largest n={n} for C={C}")
    gh.free()
