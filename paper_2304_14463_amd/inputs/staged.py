"""Seeded candidate batches in the stage-restricted domain (Section 2.3 of arXiv 2304.14463).

Positions run over n(n+1)/2 events: stage j (0-based) holds the j + 1 positions
j(j+1)/2 .. j(j+1)/2 + j; a node with place k in the topological order is computed only at
slot k of a stage, its first time at slot k of stage k.  Host generator only (numpy): the
batches the stage-restricted evaluator is tested and timed on are small enough to be uploaded.
The generator draws structure; it evaluates nothing.

* base   : node with place k: copy 0 = [slot k of stage k, first start of its last consumer],
           the other copies inactive with s = e = 0.
* type A : (b < B/2) for every eligible node (the plain generator's rule: >= 2 consumers, no
           eligible predecessor), walking copies i = 1..C-1: with probability 1/4 the previous
           copy is cut back to the first start of an earlier consumer c and copy i is computed
           again at the node's slot of a stage after c's, no later than the next consumer's
           stage and than the last stage in which all inputs of the node are still kept; it is
           kept to the last consumer.  Violation-free by construction.
* type B : (b >= B/2) type A, then every start of an active copy, with probability 1/4, moves
           either by U{-4..4} positions (which mostly leaves its slot) or to its slot in a stage
           U{-2..2} away; every end, with probability 1/4, moves by U{-4..4} stages' worth of
           positions; all clamped to the domain.
"""
from __future__ import annotations

import numpy as np

from .hashrng import hash3_np

STAGED_SEED_XOR = 0x57A6ED


def stage_start(j):
    """First position of stage j."""
    return j * (j + 1) // 2


def slot_position(j, k):
    """Position of slot k (k <= j) of stage j."""
    return j * (j + 1) // 2 + k


def staged_tables(graph, order):
    """index[v] = place of v in `order`; per node the sorted places of its consumers (CSR:
    out_ptr, cons_idx); win_stage[v] = last stage in which every input of v is still kept by the
    base candidate (n - 1 for a source); ncut[v] as in the plain generator, in stages."""
    n = graph.n
    index = np.zeros(n, dtype=np.int32)
    for j, v in enumerate(order):
        index[v] = j
    cons = graph.consumers()
    out_ptr = np.zeros(n + 1, dtype=np.int32)
    ci = []
    for v in range(n):
        ci.extend(sorted(int(index[w]) for w in cons[v]))
        out_ptr[v + 1] = len(ci)
    ci = np.asarray(ci, dtype=np.int32).reshape(-1)
    last = [int(ci[out_ptr[v + 1] - 1]) if out_ptr[v + 1] > out_ptr[v] else int(index[v]) for v in range(n)]
    win_stage = np.full(n, n - 1, dtype=np.int32)
    ncut = np.zeros(n, dtype=np.int32)
    eligible = [False] * n
    for v in order:
        preds = [int(u) for u in graph.in_idx[graph.in_ptr[v]:graph.in_ptr[v + 1]]]
        for u in preds:
            win_stage[v] = min(int(win_stage[v]), last[u])
        d = int(out_ptr[v + 1] - out_ptr[v])
        if d < 2 or any(eligible[u] for u in preds):
            continue
        cuts = sum(1 for c in range(d - 1) if ci[out_ptr[v] + c] < win_stage[v])
        if cuts:
            eligible[v] = True
            ncut[v] = cuts
    return index, out_ptr, ci, win_stage, ncut


def staged_base(n, C, index, out_ptr, cons_idx):
    """The no-rematerialisation candidate of the order in the stage layout, shape [n*C]."""
    s = np.zeros(n * C, dtype=np.int32)
    e = np.zeros(n * C, dtype=np.int32)
    a = np.zeros(n * C, dtype=np.uint8)
    for v in range(n):
        k = int(index[v])
        d = out_ptr[v + 1] - out_ptr[v]
        jl = int(cons_idx[out_ptr[v + 1] - 1]) if d else k
        s[v * C] = slot_position(k, k)
        e[v * C] = slot_position(jl, jl)
        a[v * C] = 1
    return s, e, a


def gen_staged_candidates(seed, graph, order, C, B_total, b0, count, tables=None):
    """Candidates b0 .. b0+count-1 of a batch of B_total: (starts, ends int32 [count][n*C],
    active uint8 [count][n*C])."""
    n = graph.n
    index, out_ptr, cons_idx, win_stage, ncut = tables if tables is not None else staged_tables(graph, order)
    D = n * (n + 1) // 2
    starts = np.zeros((count, n * C), dtype=np.int64)
    ends = np.zeros((count, n * C), dtype=np.int64)
    active = np.zeros((count, n * C), dtype=np.uint8)
    b = np.arange(b0, b0 + count, dtype=np.uint64)
    type_b = b >= np.uint64(B_total // 2)
    sd = seed ^ STAGED_SEED_XOR
    u64 = np.uint64
    for v in range(n):
        k = int(index[v])
        o0, o1 = int(out_ptr[v]), int(out_ptr[v + 1])
        d = o1 - o0
        ci = cons_idx[o0:o1].astype(np.int64)
        jl = int(ci[-1]) if d else k
        s = np.zeros((count, C), dtype=np.int64)
        e = np.zeros((count, C), dtype=np.int64)
        a = np.zeros((count, C), dtype=np.uint8)
        st = np.full((count, C), k, dtype=np.int64)     # stage of every copy's start
        s[:, 0], e[:, 0], a[:, 0] = slot_position(k, k), slot_position(jl, jl), 1
        nc = int(ncut[v])
        if nc >= 1:
            lo = np.zeros(count, dtype=np.int64)
            alive = np.ones(count, dtype=bool)
            for i in range(1, C):
                avail = nc - lo
                gate = hash3_np(sd, b, v, 2 * i)
                pick = hash3_np(sd, b, v, 2 * i + 1)
                take = alive & (avail >= 1) & ((gate & u64(3)) == u64(0))
                if not take.any():
                    break
                c = lo + ((pick & u64(0xFFFFFFFF)) % np.maximum(avail, 1).astype(np.uint64)).astype(np.int64)
                c = np.minimum(c, d - 2)
                cut = ci[c]                                           # stage of the consumer the previous copy is kept for
                hi = np.minimum(ci[c + 1], int(win_stage[v]))         # last stage the new copy may be computed in
                span = np.maximum(hi - cut, 1).astype(np.uint64)
                j = cut + 1 + ((pick >> u64(32)) % span).astype(np.int64)
                e[:, i - 1] = np.where(take, slot_position(cut, cut), e[:, i - 1])
                s[:, i] = np.where(take, slot_position(j, k), 0)
                st[:, i] = np.where(take, j, 0)
                e[:, i] = np.where(take, slot_position(jl, jl), 0)
                a[:, i] = take.astype(np.uint8)
                lo = np.where(take, c + 1, lo)
                alive = take
        if type_b.any():
            for i in range(C):
                rs = hash3_np(sd, b, v, 16 + 2 * i)
                re = hash3_np(sd, b, v, 16 + 2 * i + 1)
                on = type_b & (a[:, i] != 0)
                d9 = ((rs >> u64(8)) % u64(9)).astype(np.int64) - 4
                d5 = ((rs >> u64(16)) % u64(5)).astype(np.int64) - 2
                by_pos = on & ((rs & u64(7)) == u64(0))
                by_stage = on & ((rs & u64(7)) == u64(1))
                j2 = np.clip(st[:, i] + d5, k, n - 1)
                s[:, i] = np.where(by_pos, np.clip(s[:, i] + d9, 0, D - 1), s[:, i])
                s[:, i] = np.where(by_stage, slot_position(j2, k), s[:, i])
                move_e = on & ((re & u64(3)) == u64(0))
                de = (((re >> u64(8)) % u64(9)).astype(np.int64) - 4) * (jl + 1)
                e[:, i] = np.where(move_e, np.clip(e[:, i] + de, 0, D - 1), e[:, i])
        starts[:, v * C:(v + 1) * C] = s
        ends[:, v * C:(v + 1) * C] = e
        active[:, v * C:(v + 1) * C] = a
    return starts.astype(np.int32), ends.astype(np.int32), active
