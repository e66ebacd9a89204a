"""ctypes front end of the CPU oracle (moc_oracle.cpp, moc_bruteforce.cpp,
moc_exhaustive.cpp, moc_decode.cpp).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark; never by the product path, and it imports
nothing of the HIP library.  The oracle evaluates Eq. (1)-(8) of Section 2.1
of the paper (arXiv 2304.14463) exactly as defined; see moc_oracle.cpp for
the readings taken and the pins.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SOURCES = ["moc_oracle.cpp", "moc_bruteforce.cpp", "moc_exhaustive.cpp", "moc_decode.cpp"]
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

FIELDS = ("peak", "duration", "violations", "feasible", "v_form", "v_first", "v_order", "v_start", "v_prec")


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (host only)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    if not force and os.path.exists(_LIB_PATH) and all(
            os.path.getmtime(_LIB_PATH) >= os.path.getmtime(s) for s in srcs):
        return _LIB_PATH
    cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread", "-Wall", "-o", _LIB_PATH] + srcs
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _p(arr, ctype):
    return arr.ctypes.data_as(ctypes.POINTER(ctype))


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.orc_result_fields.restype = ctypes.c_int
        _lib.bf_enumerate.restype = ctypes.c_int64
        _lib.bf_simulate.restype = ctypes.c_int
        _lib.orc_cut_apply.restype = ctypes.c_int
        _lib.orc_search_cuts.restype = ctypes.c_int
        assert _lib.orc_result_fields() == len(FIELDS)
    return _lib


def _graph_args(g):
    in_ptr = np.ascontiguousarray(g.in_ptr, dtype=np.int32)
    in_idx = np.ascontiguousarray(g.in_idx, dtype=np.int32)
    size = np.ascontiguousarray(g.size, dtype=np.int32)
    dur = np.ascontiguousarray(g.dur, dtype=np.int32)
    keep = (in_ptr, in_idx, size, dur)
    args = (ctypes.c_int32(g.n), _p(in_ptr, ctypes.c_int32), _p(in_idx, ctypes.c_int32),
            _p(size, ctypes.c_int32), _p(dur, ctypes.c_int32))
    return keep, args


def _cand(x, dtype, K):
    x = np.ascontiguousarray(x, dtype=dtype)
    return x.reshape(-1, K)


def evaluate(g, budget, C, starts, ends, active, T=None):
    """Evaluate candidates [B][n*C]; returns int64 [B][9], columns = FIELDS."""
    K = g.n * C
    T = K if T is None else T
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    B = s.shape[0]
    out = np.zeros((B, len(FIELDS)), dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_eval(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), ctypes.c_int32(T), ctypes.c_int64(B),
                   _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8), _p(out, ctypes.c_int64))
    return out


def evaluate_staged(g, budget, C, index, starts, ends, active):
    """Evaluate candidates [B][n*C] in the stage-restricted domain of Section 2.3: positions in
    [0, n(n+1)/2), node v only at slot index[v] of a stage, first copy at slot index[v] of stage
    index[v].  Returns int64 [B][9], columns = FIELDS."""
    K = g.n * C
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    idx = np.ascontiguousarray(index, dtype=np.int32).reshape(g.n)
    B = s.shape[0]
    out = np.zeros((B, len(FIELDS)), dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_eval_staged(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), _p(idx, ctypes.c_int32), ctypes.c_int64(B),
                          _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8), _p(out, ctypes.c_int64))
    return out


def profile(g, budget, C, starts, ends, active, T=None):
    """One candidate: (result row, memory in use at every position)."""
    K = g.n * C
    T = K if T is None else T
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    assert s.shape[0] == 1
    out = np.zeros(len(FIELDS), dtype=np.int64)
    prof = np.zeros(T, dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_profile(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), ctypes.c_int32(T),
                      _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8),
                      _p(out, ctypes.c_int64), _p(prof, ctypes.c_int64))
    return out, prof


def neighbours(g, budget, C, starts, ends, active, R, moves=None, T=None):
    """Scores of single-field moves of one candidate by full re-evaluation.

    Returns (scores int64 [count][2] = (violations, peak) or (-1,-1),
    best = (move, violations, peak)); `moves` = None scores all n*C*4R moves.
    """
    K = g.n * C
    T = K if T is None else T
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    assert s.shape[0] == 1
    if moves is None:
        n_moves, mv, count = 0, None, K * 4 * R
    else:
        mv = np.ascontiguousarray(moves, dtype=np.int64)
        n_moves = count = mv.shape[0]
    scores = np.zeros((count, 2), dtype=np.int64)
    best = np.zeros(3, dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_neighbours(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), ctypes.c_int32(T),
                         _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8),
                         ctypes.c_int32(R), ctypes.c_int64(n_moves),
                         _p(mv, ctypes.c_int64) if mv is not None else None,
                         _p(scores, ctypes.c_int64), _p(best, ctypes.c_int64))
    return scores, tuple(int(x) for x in best)


def toggles(g, budget, C, starts, ends, active, T=None):
    """Scores of the n*C candidates that differ from this one in one active flag, by full
    re-evaluation: int64 [n*C][3] = (violations, peak, duration)."""
    K = g.n * C
    T = K if T is None else T
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    assert s.shape[0] == 1
    scores = np.zeros((K, 3), dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_toggles(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), ctypes.c_int32(T),
                      _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8), _p(scores, ctypes.c_int64))
    return scores


def cuts(g, budget, C, starts, ends, active, T=None, with_at_peak=False, mode=0):
    """Scores of the m*C cut-and-recompute moves of one candidate (in-edge x in CSR order,
    consumer copy i; q = x*C + i) by full re-evaluation of the edited candidate:
    int64 [m*C][3] = (violations, peak, duration), (-1, -1, 0) where not applicable.
    with_at_peak adds a fourth column: the positions at which the edited candidate's memory
    still reaches the peak of the candidate as given."""
    K = g.n * C
    T = K if T is None else T
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    assert s.shape[0] == 1
    m = int(np.asarray(g.in_ptr)[-1])
    scores = np.zeros((m * C, 4), dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_cuts(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), ctypes.c_int32(T),
                   _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8), _p(scores, ctypes.c_int64),
                   ctypes.c_int32(mode))
    return scores if with_at_peak else np.ascontiguousarray(scores[:, :3])


def cut_apply(g, C, starts, ends, active, x, i, T=None, mode=0):
    """The candidate after the cut for in-edge x and consumer copy i: (applicable, s, e, a)."""
    K = g.n * C
    T = K if T is None else T
    s, e, a = _cand(starts, np.int32, K), _cand(ends, np.int32, K), _cand(active, np.uint8, K)
    s2, e2, a2 = np.zeros(K, np.int32), np.zeros(K, np.int32), np.zeros(K, np.uint8)
    keep, ga = _graph_args(g)
    ok = lib().orc_cut_apply(*ga, ctypes.c_int32(C), ctypes.c_int32(T), _p(s, ctypes.c_int32),
                             _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8), ctypes.c_int32(x), ctypes.c_int32(i),
                             _p(s2, ctypes.c_int32), _p(e2, ctypes.c_int32), _p(a2, ctypes.c_uint8), ctypes.c_int32(mode))
    return bool(ok), s2, e2, a2


def search_cuts(g, budget, C, starts, ends, active, max_steps, T=None, mode=0):
    """Greedy descent by cuts on one candidate: (steps applied, s, e, a) after up to max_steps."""
    K = g.n * C
    T = K if T is None else T
    s = np.array(starts, dtype=np.int32).reshape(K).copy()
    e = np.array(ends, dtype=np.int32).reshape(K).copy()
    a = np.array(active, dtype=np.uint8).reshape(K).copy()
    keep, ga = _graph_args(g)
    steps = lib().orc_search_cuts(*ga, ctypes.c_int64(budget), ctypes.c_int32(C), ctypes.c_int32(T),
                                  _p(s, ctypes.c_int32), _p(e, ctypes.c_int32), _p(a, ctypes.c_uint8),
                                  ctypes.c_int32(max_steps), ctypes.c_int32(mode))
    return int(steps), s, e, a


def search_moves(g, budget, C, starts, ends, active, R, max_steps, T=None):
    """Greedy descent by single-field moves on one candidate, out of the oracle's own pieces:
    at every step the best move of neighbours() is applied if it lowers
    (violations, max(peak, M), peak) against evaluate() of the candidate as it stands.
    Returns (steps applied, s, e)."""
    K = g.n * C
    T = K if T is None else T
    s = np.array(starts, dtype=np.int32).reshape(K).copy()
    e = np.array(ends, dtype=np.int32).reshape(K).copy()
    a = np.array(active, dtype=np.uint8).reshape(K)
    applied = 0
    for _ in range(max_steps):
        base = evaluate(g, budget, C, s, e, a, T=T)[0]
        v0, p0 = int(base[FIELDS.index("violations")]), int(base[FIELDS.index("peak")])
        _, (q, v1, p1) = neighbours(g, budget, C, s, e, a, R, T=T)
        if q < 0 or not ((v1, max(p1, budget), p1) < (v0, max(p0, budget), p0)):
            break
        d, field, k = q % (2 * R), (q // (2 * R)) % 2, q // (4 * R)
        (s if field == 0 else e)[k] += d - R if d < R else d - R + 1
        applied += 1
    return applied, s, e


def merge_candidates(C, starts, ends, active, T, K):
    """The merge moves of one candidate, at most K of them: for every live copy, in order of its
    index, that has an earlier live copy of the same node, the candidate in which the nearest
    such earlier copy is kept until the later of the two ends and the copy itself is switched
    off (the node is computed once less, Eq. (1), and its output is held across the gap instead,
    Eq. (4)).  Returns (copy indices [count], starts, ends, active [count][n*C])."""
    s, e, a = (np.asarray(x).reshape(-1) for x in (starts, ends, active))
    live = (a != 0) & (s >= 0) & (s <= e) & (e <= T - 1)
    picks, S, E, A = [], [], [], []
    for k in range(len(s)):
        if len(picks) == K:
            break
        if not live[k]:
            continue
        v, i = divmod(k, C)
        prev = [v * C + j for j in range(i) if live[v * C + j]]
        if not prev:
            continue
        s2, e2, a2 = s.copy(), e.copy(), a.copy()
        e2[prev[-1]] = max(e2[prev[-1]], e2[k])
        a2[k] = 0
        picks.append(k)
        S.append(s2); E.append(e2); A.append(a2)
    n = len(s)
    return (np.array(picks, np.int64), np.array(S, np.int32).reshape(-1, n), np.array(E, np.int32).reshape(-1, n),
            np.array(A, np.uint8).reshape(-1, n))


def search_merges(g, budget, C, starts, ends, active, max_steps, K, T=None):
    """Descent by merges on one candidate (the duration-reducing half of a local search: Phase 2
    of Section 2.4 minimises Eq. (1) subject to everything else): up to max_steps times, evaluate
    the first K merge moves, and apply the one whose result is feasible (no violation, peak
    within the budget) with the lowest duration, then the lowest peak, then the lowest copy
    index; stop when none is feasible.  Returns (steps applied, s, e, a)."""
    K_ = g.n * C
    T = K_ if T is None else T
    s = np.array(starts, dtype=np.int32).reshape(K_).copy()
    e = np.array(ends, dtype=np.int32).reshape(K_).copy()
    a = np.array(active, dtype=np.uint8).reshape(K_).copy()
    applied = 0
    for _ in range(max_steps):
        picks, S, E, A = merge_candidates(C, s, e, a, T, K)
        if len(picks) == 0:
            break
        res = evaluate(g, budget, C, S, E, A, T=T)
        ok = np.flatnonzero(res[:, FIELDS.index("feasible")] == 1)
        if ok.size == 0:
            break
        best = min(ok, key=lambda r: (res[r, FIELDS.index("duration")], res[r, FIELDS.index("peak")], picks[r]))
        s, e, a = S[best].copy(), E[best].copy(), A[best].copy()
        applied += 1
    return applied, s, e, a


def search_two_phase(g, budget, C, starts, ends, active, max_cuts, max_merges, K, T=None):
    """Phase 1: descent by cuts that keep the inputs (search_cuts, mode 1) towards the budget;
    Phase 2: descent by merges from there.  Returns (cuts applied, merges applied, s, e, a)."""
    k1, s, e, a = search_cuts(g, budget, C, starts, ends, active, max_cuts, T=T, mode=1)
    k2, s, e, a = search_merges(g, budget, C, s, e, a, max_merges, K, T=T)
    return k1, k2, s, e, a


def decode(g, C, starts, active, T=None):
    """Sequences the candidates stand for (active copies in start order) and their own
    liveness footprint.  Returns (int64 [B][4] = status, length, peak, duration;
    int32 [B][T] sequences padded with -1).  status 1 valid, 0 not a valid sequence,
    -1 not decodable."""
    K = g.n * C
    T = K if T is None else T
    s, a = _cand(starts, np.int32, K), _cand(active, np.uint8, K)
    B = s.shape[0]
    res = np.zeros((B, 4), dtype=np.int64)
    seq = np.zeros((B, T), dtype=np.int32)
    keep, ga = _graph_args(g)
    for b in range(B):
        lib().dec_decode(*ga, ctypes.c_int32(C), ctypes.c_int32(T), _p(s[b], ctypes.c_int32),
                         _p(a[b], ctypes.c_uint8), _p(seq[b], ctypes.c_int32), _p(res[b], ctypes.c_int64))
    return res, seq


def simulate_sequence(g, seq):
    """Independent liveness simulation of a rematerialisation sequence.
    Returns (valid, peak, duration)."""
    sq = np.ascontiguousarray(seq, dtype=np.int32)
    peak = ctypes.c_int64(0)
    dur = ctypes.c_int64(0)
    keep, ga = _graph_args(g)
    ok = lib().bf_simulate(*ga, ctypes.c_int32(sq.shape[0]), _p(sq, ctypes.c_int32),
                           ctypes.byref(peak), ctypes.byref(dur))
    return bool(ok), peak.value, dur.value


def enumerate_sequences(g, C, max_extra, cap=2_000_000):
    """All valid sequences with <= C occurrences per node and <= max_extra
    recomputations, with simulated peak/duration and canonical candidates."""
    K = g.n * C
    seq_len = np.zeros(cap, dtype=np.int32)
    seqs = np.zeros((cap, K), dtype=np.int32)
    peak = np.zeros(cap, dtype=np.int64)
    dur = np.zeros(cap, dtype=np.int64)
    s = np.zeros((cap, K), dtype=np.int32)
    e = np.zeros((cap, K), dtype=np.int32)
    a = np.zeros((cap, K), dtype=np.uint8)
    keep, ga = _graph_args(g)
    cnt = lib().bf_enumerate(*ga, ctypes.c_int32(C), ctypes.c_int32(max_extra), ctypes.c_int64(cap),
                             _p(seq_len, ctypes.c_int32), _p(seqs, ctypes.c_int32), _p(peak, ctypes.c_int64),
                             _p(dur, ctypes.c_int64), _p(s, ctypes.c_int32), _p(e, ctypes.c_int32),
                             _p(a, ctypes.c_uint8))
    if cnt > cap:
        raise RuntimeError(f"{cnt} sequences exceed cap {cap}")
    return dict(count=int(cnt), seq_len=seq_len[:cnt], seqs=seqs[:cnt], peak=peak[:cnt], duration=dur[:cnt],
                starts=s[:cnt], ends=e[:cnt], active=a[:cnt])


def exhaustive_c2(g, n_threads=8):
    """Every C=2 assignment on a DAG with n <= 4 (see moc_exhaustive.cpp).
    Returns (counts = evaluated, violation-free, failed checks; min_peak[mask])."""
    assert g.n <= 4
    counts = np.zeros(3, dtype=np.int64)
    min_peak = np.zeros(1 << g.n, dtype=np.int64)
    keep, ga = _graph_args(g)
    lib().orc_exhaustive_c2(*ga, ctypes.c_int32(n_threads), _p(counts, ctypes.c_int64), _p(min_peak, ctypes.c_int64))
    return counts, min_peak
