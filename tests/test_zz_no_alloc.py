"""moc_eval_batch_noalloc (work counters in the library's static device array) against
moc_eval_batch, through the C ABI: bit-exact, on two calls in a row, the second with a
smaller input; then on a second graph of another shape, whose launches use the same array."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moc():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2304_14463_amd import moccasin
    moccasin.lib()
    return moccasin


def candidates(rng, B, n, C):
    T = n * C
    s = rng.integers(0, T, size=(B, T)).astype(np.int32)
    e = np.minimum(T - 1, s + rng.integers(-1, 40, size=(B, T))).astype(np.int32)
    a = (rng.random((B, T)) < 0.15).astype(np.uint8)
    a.reshape(B, n, C)[:, :, 0] = 1
    return s, e, a


def test_noalloc_matches_eval_batch(moc):
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    rng = np.random.default_rng(2024)
    for n, C, B1, B2 in ((150, 2, 60000, 9000), (700, 3, 30000, 41)):
        edges = sorted({(int(u), v) for v in range(1, n) for u in rng.integers(max(0, v - 30), v, size=2)})
        g = graph_from_edges(n, edges, rng.integers(1, 100, n), rng.integers(1, 9, n))
        gh = moc.moc_graph_upload(n, g.in_ptr, g.in_idx, g.size, g.dur, int(g.size.sum()) // 3, C)
        s, e, a = candidates(rng, B1, n, C)
        ds, de, da = (torch.from_numpy(x).cuda() for x in (s, e, a))
        want1 = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
        want2 = moc.results_to_numpy(moc.moc_eval_batch(gh, ds[:B2], de[:B2], da[:B2]))
        assert want2.tobytes() == want1[:B2].tobytes()
        out1 = torch.full((B1, 24), 0xEE, dtype=torch.uint8, device="cuda")
        out2 = torch.full((B2, 24), 0xEE, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        # two calls in a row on one stream, the second with fewer candidates (dynamic hand-out
        # in the first, static split in the second where B2 is small)
        moc.moc_eval_batch_noalloc(gh, ds, de, da, out1)
        moc.moc_eval_batch_noalloc(gh, ds[:B2], de[:B2], da[:B2], out2)
        torch.cuda.synchronize()
        assert moc.results_to_numpy(out1).tobytes() == want1.tobytes(), (n, C, "first call")
        assert moc.results_to_numpy(out2).tobytes() == want2.tobytes(), (n, C, "second call")
        # and the other way round: large after small
        out1.fill_(0xEE)
        out2.fill_(0xEE)
        moc.moc_eval_batch_noalloc(gh, ds[:B2], de[:B2], da[:B2], out2)
        moc.moc_eval_batch_noalloc(gh, ds, de, da, out1)
        torch.cuda.synchronize()
        assert moc.results_to_numpy(out1).tobytes() == want1.tobytes(), (n, C, "large after small")
        assert moc.results_to_numpy(out2).tobytes() == want2.tobytes(), (n, C, "small before large")
        # the handle's own counters are untouched by all this
        assert moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da)).tobytes() == want1.tobytes()
        gh.free()


def test_noalloc_rejects_what_it_cannot_take(moc):
    import ctypes
    import torch
    from paper_2304_14463_amd.inputs import graph_from_edges
    g = graph_from_edges(4, [(0, 1), (1, 2), (2, 3)], [1, 1, 1, 1], [1, 1, 1, 1])
    gh = moc.moc_graph_upload(4, g.in_ptr, g.in_idx, g.size, g.dur, 2, 1)
    z = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    a = torch.ones((1, 4), dtype=torch.uint8, device="cuda")
    out = torch.zeros((1, 24), dtype=torch.uint8, device="cuda")
    L = moc.lib()
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    # more candidates than one launch counts: refused before anything is queued
    assert L.moc_eval_batch_noalloc(gh._h, (1 << 31) + 1, P(z), P(z), P(a), P(out), None) == -2
    assert L.moc_eval_batch_noalloc(gh._h, -1, P(z), P(z), P(a), P(out), None) == -1
    assert L.moc_eval_batch_noalloc(gh._h, 1, None, P(z), P(a), P(out), None) == -1
    assert L.moc_eval_batch_noalloc(gh._h, 0, None, None, None, None, None) == 0
    assert L.moc_eval_batch_noalloc(gh._h, 1, P(z), P(z), P(a), P(out), None) == 0
    torch.cuda.synchronize()
    gh.free()
