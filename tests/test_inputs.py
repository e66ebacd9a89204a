"""Host-side checks of the seeded input generators (no method arithmetic)."""
import numpy as np
import pytest

from paper_2304_14463_amd.inputs import make_workload
from paper_2304_14463_amd.inputs.hashrng import hash3, hash3_np, mix64

SHAPES = {0: (50, None, 2, 1024), 1: (442, 1247, 2, 16384), 2: (1000, 2245, 2, 65536),
          3: (2000, 6000, 2, 8192), 4: (5000, 15000, 3, 262144)}


def test_splitmix_finaliser_known_values():
    # SplitMix64 stream with seed 0: first outputs of the published generator
    # (state += golden; return mix(state)).
    golden = 0x9E3779B97F4A7C15
    assert mix64(golden) == 0xE220A8397B1DCDAF
    assert mix64(2 * golden) == 0x6E789E6AA1B965F4
    v = hash3_np(123, np.arange(5), 7, np.arange(5) * 3)
    assert [int(x) for x in v] == [hash3(123, i, 7, 3 * i) for i in range(5)]


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_workload_shapes(workloads, cfg):
    w = workloads(cfg)
    n, m, C, B = SHAPES[cfg]
    assert (w.n, w.C, w.B) == (n, C, B) and w.T == n * C
    if m is not None:
        assert w.m == m
    else:
        assert 90 <= w.m <= 110
    g = w.graph
    edges = g.edges()
    assert len(set(edges)) == len(edges) and all(u < v for u, v in edges)   # DAG, ids topological
    assert g.size.min() >= 1 and g.dur.min() >= 1
    assert C * int(g.size.sum()) < 2**31
    if cfg == 0:
        assert [len(c) for c in g.consumers()].count(0) == 1              # single sink
    # the base order is a topological order
    step = {v: j for j, v in enumerate(w.order)}
    assert all(step[u] < step[v] for u, v in edges)
    assert w.budget == (w.pct * w.no_remat_peak) // 100


@pytest.mark.parametrize("cfg", [0, 1, 4])
def test_candidates_are_deterministic_and_chunkable(workloads, cfg):
    w = workloads(cfg)
    s, e, a = w.candidates(w.B // 2 - 3, 6)
    s1, e1, a1 = w.candidates(w.B // 2 - 3, 2)
    s2, e2, a2 = w.candidates(w.B // 2 - 1, 4)
    assert (np.vstack([s1, s2]) == s).all() and (np.vstack([e1, e2]) == e).all() and (np.vstack([a1, a2]) == a).all()
    assert s.dtype == np.int32 and e.dtype == np.int32 and a.dtype == np.uint8
    assert s.shape == (6, w.T)
    assert (a.reshape(6, w.n, w.C)[:, :, 0] == 1).all()
    assert s.min() >= 0 and max(s.max(), e.max()) < w.T
    assert (s[0] != s[1]).any() or (e[0] != e[1]).any()


@pytest.mark.parametrize("cfg", [0, 4])
def test_dense_batch_structure(cfg):
    """The dense batch: nearly every copy active, copies of a node in a row on the node's own
    free slots, each kept until the next one starts."""
    w = make_workload(cfg, 64, dense=True)
    s, e, a = w.candidates(0, 64)
    n, C, T = w.n, w.C, w.T
    A = a.reshape(64, n, C) != 0
    S, E = s.reshape(64, n, C), e.reshape(64, n, C)
    assert A[:, :, 0].all() and 0.8 < A[:, :, 1:].mean() < 0.95
    first = slice(0, 32)                                           # not perturbed
    want = np.broadcast_to(w.pos[None, :, None] + np.arange(C)[None, None, :], S[first].shape)
    assert (S[first][A[first]] == want[A[first]]).all()
    for b in range(4):
        for v in range(0, n, max(1, n // 50)):
            act = [i for i in range(C) if A[b, v, i]]
            for i, j in zip(act, act[1:]):
                assert E[b, v, i] == S[b, v, j]
            assert E[b, v, act[-1]] == min(T - 1, max(w.pos[v], w.cons_pos[w.out_ptr[v]:w.out_ptr[v + 1]].max(initial=0)) + C - 1)
    assert s.min() >= 0 and max(s.max(), e.max()) < T
