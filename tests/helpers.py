"""Shared helpers of the GPU parity tests."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle

F = {name: i for i, name in enumerate(oracle.FIELDS)}


def oracle_eval_parallel(g, budget, C, s, e, a, threads=8):
    """oracle.evaluate over row chunks on several host threads (ctypes drops the GIL)."""
    B = s.shape[0]
    if B < 4 * threads:
        return oracle.evaluate(g, budget, C, s, e, a)
    cuts = np.linspace(0, B, threads + 1).astype(int)
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda i: oracle.evaluate(g, budget, C, s[cuts[i]:cuts[i + 1]], e[cuts[i]:cuts[i + 1]],
                                                      a[cuts[i]:cuts[i + 1]]), range(threads)))
    return np.vstack(parts)


def assert_results_equal(gpu, ref, what=""):
    """gpu: structured array of moc_result; ref: oracle rows.  Bit-exact on all four fields."""
    for name in ("peak", "duration", "violations", "feasible"):
        got = gpu[name].astype(np.int64)
        want = ref[:, F[name]]
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{what}: {name} differs at {bad[:8]}: gpu {got[bad[:8]]} oracle {want[bad[:8]]}"


def upload(moc, w, budget=None):
    g = w.graph
    return moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, w.budget if budget is None else budget, w.C)
