"""GPU parity of moc_decode_batch: status, length, peak, duration and the
sequence itself equal the oracle's decode, bit-exact."""
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


def gpu_decode(moc, gh, s, a, want_seq=True):
    ds, da = to_dev(s, a)
    out, seq = moc.moc_decode_batch(gh, ds, da, want_seq=want_seq)
    return moc.results_to_numpy(out, moc.DECODE_RESULT_DTYPE), (seq.cpu().numpy() if seq is not None else None)


def assert_same(got, seq, want, want_seq, what=""):
    for i, name in enumerate(("status", "length", "peak", "duration")):
        bad = np.flatnonzero(got[name].astype(np.int64) != want[:, i])
        assert bad.size == 0, f"{what}: {name} differs at {bad[:8]}: gpu {got[name][bad[:8]]} oracle {want[bad[:8], i]}"
    if seq is not None:
        bad = np.flatnonzero((seq != want_seq).any(1))
        assert bad.size == 0, f"{what}: sequences differ at {bad[:8]}"


def orderly_candidates(rng, g, C, B):
    """Distinct starts.  Row kinds in turn: a topological order with recomputations inserted
    (valid), the same with a few steps swapped (often not valid), a random order (hardly ever
    valid), a random order of a subset of the nodes (some node missing)."""
    n, T = g.n, g.n * C
    s = rng.integers(-3, T + 3, size=(B, T)).astype(np.int32)   # fields of inactive copies: anything
    a = np.zeros((B, T), np.uint8)
    for b in range(B):
        kind = b % 4
        extra = rng.integers(0, n * (C - 1) + 1) if C > 1 else 0
        nodes = list(range(n)) + list(rng.integers(0, n, extra))
        if kind == 3:
            nodes = [v for v in nodes if v != nodes[rng.integers(0, n)]] or [0]
        times = np.zeros(n, int)
        keep = []
        for v in nodes:
            if times[v] < C:
                times[v] += 1
                keep.append(v)
        if kind <= 1:
            # recomputations anywhere after the first computation: sort by (node order with jitter)
            first = np.zeros(n, bool)
            keys = []
            for v in keep:
                keys.append(v if not first[v] else rng.uniform(v, n))
                first[v] = True
            keep = [v for _, v in sorted(zip(keys, keep), key=lambda t: t[0])]
            if kind == 1:
                for _ in range(rng.integers(1, 4)):
                    i, j = rng.integers(0, len(keep), 2)
                    keep[i], keep[j] = keep[j], keep[i]
        else:
            rng.shuffle(keep)
        pos = np.sort(rng.choice(T, size=len(keep), replace=False))
        used = np.zeros(n, int)
        for p, v in zip(pos, keep):
            i = (used[v] + b) % C
            while a[b, v * C + i]:
                i = (i + 1) % C
            s[b, v * C + i], a[b, v * C + i] = p, 1
            used[v] += 1
    return s, a


@pytest.mark.parametrize("n,C", [(1, 1), (2, 2), (5, 1), (9, 2), (17, 3), (40, 2), (64, 4), (130, 2), (257, 3),
                                 (600, 1), (1100, 2), (3, 5), (33, 5), (150, 6), (700, 5)])
def test_decode_small_graphs(moc, n, C):
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(31 * n + C)
    edges = set()
    for v in range(1, n):
        for u in rng.integers(max(0, v - 12), v, size=rng.integers(0, 4)):
            edges.add((int(u), v))
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(1, 9, n))
    T, B = n * C, 24
    s, a = orderly_candidates(rng, g, C, B)
    # rows that cannot be decoded: a shared start, a start outside the domain, and wild everything
    act = np.flatnonzero(a[4])
    if act.size >= 2:
        s[4, act[-1]] = s[4, act[0]]
    s[5, np.flatnonzero(a[5])[0]] = T
    s[6, np.flatnonzero(a[6])[0]] = -1
    s[7] = rng.integers(-3, T + 3, T); a[7] = rng.random(T) < 0.7
    a[8] = 0   # nothing active: no node occurs
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 1, C)
    want, want_seq = oracle.decode(g, C, s, a)
    got, seq = gpu_decode(moc, gh, s, a)
    assert_same(got, seq, want, want_seq, f"n={n} C={C}")
    kinds = set(want[:, 0])
    assert kinds == ({-1, 0, 1} if n > 2 else kinds)
    got2, none = gpu_decode(moc, gh, s, a, want_seq=False)
    assert none is None and (got2 == got).all()
    gh.free()


@pytest.mark.parametrize("n,C", [(70, 1), (70, 2), (70, 3), (70, 4), (2500, 2), (70, 5)])
def test_decode_rows_at_odd_addresses(moc, n, C):
    """The kernel reads the copies of a node in one load each for starts and flags: the arrays
    may begin at any int32 boundary (starts) and at any byte (flags)."""
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(977 * n + C)
    edges = set()
    for v in range(1, n):
        for u in rng.integers(max(0, v - 9), v, size=rng.integers(0, 3)):
            edges.add((int(u), v))
    g = graph_from_edges(n, sorted(edges), rng.integers(0, 50, n), rng.integers(1, 9, n))
    T, B = n * C, 12
    s, a = orderly_candidates(rng, g, C, B)
    gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, 1, C)
    want, want_seq = oracle.decode(g, C, s, a)
    for shift_s, shift_a in ((1, 1), (3, 2), (2, 3)):
        pad_s = torch.zeros(B * T + shift_s, dtype=torch.int32, device="cuda")
        pad_a = torch.zeros(B * T + shift_a, dtype=torch.uint8, device="cuda")
        pad_s[shift_s:] = torch.from_numpy(s.reshape(-1)).cuda()
        pad_a[shift_a:] = torch.from_numpy(a.reshape(-1)).cuda()
        out, seq = moc.moc_decode_batch(gh, pad_s[shift_s:], pad_a[shift_a:])
        assert_same(moc.results_to_numpy(out, moc.DECODE_RESULT_DTYPE), seq.cpu().numpy(), want, want_seq,
                    f"n={n} C={C} starts + {shift_s} words, flags + {shift_a} bytes")
    gh.free()


def test_decode_self_loop_and_duplicate_edges(moc):
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(4, [(0, 1), (0, 1), (1, 1), (1, 2), (0, 3)], [3, 5, 2, 7], [1, 2, 3, 4])
    s = np.array([[0, 4, 1, 2, 3, 0, 5, 0], [0, 0, 1, 0, 2, 0, 3, 0]], np.int32)
    a = np.array([[1, 1, 1, 1, 1, 0, 1, 0], [1, 0, 1, 0, 1, 0, 1, 0]], np.uint8)
    gh = moc.moc_graph_upload(4, g.in_ptr, g.in_idx, g.size, g.dur, 1, 2)
    want, want_seq = oracle.decode(g, 2, s, a)
    got, seq = gpu_decode(moc, gh, s, a)
    assert_same(got, seq, want, want_seq)
    assert list(want[:, 0]) == [0, 0]   # node 1 reads itself: its first computation finds nothing
    gh.free()


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_decode_workload_candidates(moc, workloads, cfg):
    """The synthetic candidates of the evaluation workloads: about half are violation-free and
    decode to valid sequences, perturbed ones mostly share starts."""
    w = workloads(cfg)
    count = min(w.B, 512)
    s, e, a = w.candidates(0, count)
    gh = upload(moc, w)
    want, want_seq = oracle.decode(w.graph, w.C, s, a)
    got, seq = gpu_decode(moc, gh, s, a)
    assert_same(got, seq, want, want_seq, f"cfg {cfg}")
    assert (want[:, 0] == 1).sum() > count // 8
    gh.free()


@pytest.mark.parametrize("cfg", [3, 4])
def test_decode_full_batch(moc, workloads, cfg):
    """Full-size launch (n=2000, C=2, B=8192; n=5000, C=3, first 16384 candidates): sampled rows
    against the oracle; on every row, properties that tie the decoder to the evaluator -- a
    candidate without violations decodes to a valid sequence of the same duration and no
    larger peak, and its length is the number of active copies."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload
    w = workloads(cfg)
    gh = upload(moc, w)
    B = min(w.B, 16384)
    ds, de, da = DeviceWorkload(w).candidates(0, B)
    out, seq = moc.moc_decode_batch(gh, ds, da)
    ev = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    torch.cuda.synchronize()
    got = moc.results_to_numpy(out, moc.DECODE_RESULT_DTYPE)
    rows = [0, 1, B // 3, B // 2 + 1, B - 2, B - 1] + list(np.random.default_rng(cfg).integers(0, B, 10))
    for b in rows:
        s, a = ds[b].cpu().numpy(), da[b].cpu().numpy()
        want, want_seq = oracle.decode(w.graph, w.C, s, a)
        assert_same(got[b:b + 1], seq[b:b + 1].cpu().numpy(), want, want_seq, f"cfg {cfg} row {b}")
    clean = ev["violations"] == 0
    assert clean.sum() > 100
    assert (got["status"][clean] == 1).all()
    assert (got["duration"][clean] == ev["duration"][clean]).all()
    assert (got["peak"][clean] <= ev["peak"][clean]).all()
    n_active = (da != 0).sum(1).cpu().numpy()
    ok = got["status"] >= 0
    assert (got["length"][ok] == n_active[ok]).all() and (got["length"][~ok] == 0).all()
    # the same launch shape on decodable rows only: the violation-free candidates, every other
    # one with the starts of a few pairs of copies exchanged (mostly no longer valid)
    idx = torch.from_numpy(np.flatnonzero(clean)).cuda()
    idx = idx[torch.arange(B, device="cuda") % idx.numel()]
    s2, a2 = ds[idx].contiguous(), da[idx].contiguous()
    rng = np.random.default_rng(100 + cfg)
    rows2 = np.arange(1, B, 2)
    for _ in range(3):
        k1, k2 = (torch.from_numpy(rng.integers(0, w.T, rows2.size)).cuda() for _ in range(2))
        r = torch.from_numpy(rows2).cuda()
        both = (a2[r, k1] != 0) & (a2[r, k2] != 0)
        r, k1, k2 = r[both], k1[both], k2[both]
        v1, v2 = s2[r, k1].clone(), s2[r, k2].clone()
        s2[r, k1], s2[r, k2] = v2, v1
    out2, seq2 = moc.moc_decode_batch(gh, s2, a2)
    got2 = moc.results_to_numpy(out2, moc.DECODE_RESULT_DTYPE)
    assert (got2["status"] >= 0).all() and (got2["status"][0::2] == 1).all()
    assert 0 < (got2["status"][1::2] == 1).sum() < rows2.size
    for b in [0, 1, 2, 3, B - 1] + list(rng.integers(0, B, 11)):
        want, want_seq = oracle.decode(w.graph, w.C, s2[b].cpu().numpy(), a2[b].cpu().numpy())
        assert_same(got2[b:b + 1], seq2[b:b + 1].cpu().numpy(), want, want_seq, f"cfg {cfg} decodable row {b}")
    # each decoded row lists `length` nodes and then -1
    seq_h = seq.cpu().numpy()
    assert ((seq_h >= 0).sum(1) == got["length"]).all()
    assert ((seq_h >= 0) == (np.arange(w.T)[None, :] < got["length"][:, None])).all()
    gh.free()


def test_decode_rejects_bad_arguments(moc):
    import ctypes
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(3, [(0, 1), (1, 2)], [1, 1, 1], [1, 1, 1])
    gh = moc.moc_graph_upload(3, g.in_ptr, g.in_idx, g.size, g.dur, 1, 2)
    s = torch.zeros((2, 6), dtype=torch.int32, device="cuda")
    a = torch.zeros((2, 6), dtype=torch.uint8, device="cuda")
    out = torch.zeros((2, 24), dtype=torch.uint8, device="cuda")
    L = moc.lib()
    vp = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    assert L.moc_decode_batch(gh._h, 2, None, vp(a), vp(out), None, None) == -1
    assert L.moc_decode_batch(gh._h, 2, vp(s), vp(a), None, None, None) == -1
    assert L.moc_decode_batch(gh._h, -1, vp(s), vp(a), vp(out), None, None) == -1
    assert L.moc_decode_batch(gh._h, 1, vp(s, 2), vp(a), vp(out), None, None) == -1     # misaligned starts
    assert L.moc_decode_batch(gh._h, 1, vp(s), vp(a), vp(out, 4), None, None) == -1     # misaligned results
    assert L.moc_decode_batch(gh._h, 0, None, None, None, None, None) == 0              # empty batch
    gh.free()
    # 2.5 words per copy of LDS: a graph the evaluator takes can be too large for this call
    n = 19000
    gl = graph_from_edges(n, [(v - 1, v) for v in range(1, n)], np.ones(n, np.int32), np.ones(n, np.int32))
    gh = moc.moc_graph_upload(n, gl.in_ptr, gl.in_idx, gl.size, gl.dur, 1, 1)
    s = torch.zeros((1, n), dtype=torch.int32, device="cuda")
    a = torch.zeros((1, n), dtype=torch.uint8, device="cuda")
    assert L.moc_decode_batch(gh._h, 1, vp(s), vp(a), vp(out), None, None) == -2
    gh.free()
