"""Seeded candidate batches: host generator (numpy).

A candidate assigns to every copy k = v*C + i an active flag, a start position
and a retention end (Section 2.1: variables a, s, e), laid out as three
[B][T] arrays, T = n*C.  The generator builds them from a base topological
order; it draws structure, it does not evaluate anything:

* base      : order index j -> position j*C (so C-1 free slots follow every
              compute event); copy 0 = [pos, position of the last consumer],
              the other copies inactive with s = e = 0.
* type A    : (b < B/2) walking copies i = 1..C-1 of every eligible node: with
              probability 1/4 cut the previous copy's end back to an earlier
              consumer and activate copy i at a free slot after that consumer
              and before the next one, retained to the last consumer; stop at
              the first copy that is not activated.  A node is eligible if it
              has >= 2 consumers and no eligible predecessor, and its new
              copies start no later than win_hi[v], the last position at which
              all its inputs are still retained by the base candidate -- so a
              type-A candidate keeps every precedence satisfied and only
              collides when two nodes pick the same free slot.
* type B    : (b >= B/2) type A, then every start and end of an active copy is
              moved by U{-4..+4} with probability 1/4, clamped to [0, T).

* dense     : (a batch of its own, for measuring how the evaluator's speed depends on how
              many copies are live) every node is computed C times in a row: copy i >= 1 is
              active with probability 7/8 and starts in the free slot pos + i; an active
              copy is kept until the next active copy of its node starts, the last one until
              C - 1 positions past the last consumer (so that the consumer's own later
              copies are served too).  The first half of the batch is violation-free as it
              stands, the second half is perturbed as type B.

Every draw is hash3(seed, b, v, j) with a fixed counter j per decision, so the
device generator (gen_candidates.hip) reproduces the same bits.
"""
from __future__ import annotations

import numpy as np

from .hashrng import GOLDEN, MASK64, mix64_np

_G = np.uint64(GOLDEN)
CAND_SEED_XOR = 0xC0FFEE5EED


def candidate_tables(graph, order, C):
    """Static per-node tables of the generator.

    pos[v] = C * (index of v in order); out_ptr/cons_pos = per node, the
    positions of its consumers in increasing order; win_hi[v] = last position
    at which every input of v is retained by the base candidate (T-1 for a
    source); ncut[v] = number of consumers c (in position order, the last one
    excluded) after which an eligible node may be cut, 0 for other nodes."""
    n = graph.n
    pos = np.zeros(n, dtype=np.int32)
    for j, v in enumerate(order):
        pos[v] = j * C
    cons = graph.consumers()
    out_ptr = np.zeros(n + 1, dtype=np.int32)
    cp = []
    for v in range(n):
        cp.extend(sorted(int(pos[w]) for w in cons[v]))
        out_ptr[v + 1] = len(cp)
    cp = np.asarray(cp, dtype=np.int32).reshape(-1)
    last = [int(cp[out_ptr[v + 1] - 1]) if out_ptr[v + 1] > out_ptr[v] else int(pos[v]) for v in range(n)]
    win_hi = np.full(n, n * C - 1, dtype=np.int32)
    ncut = np.zeros(n, dtype=np.int32)
    eligible = [False] * n
    for v in order:
        preds = [int(u) for u in graph.in_idx[graph.in_ptr[v]:graph.in_ptr[v + 1]]]
        for u in preds:
            win_hi[v] = min(int(win_hi[v]), last[u])
        d = int(out_ptr[v + 1] - out_ptr[v])
        if C < 2 or d < 2 or any(eligible[u] for u in preds):
            continue
        cuts = sum(1 for c in range(d - 1) if cp[out_ptr[v] + c] < win_hi[v])
        if cuts:
            eligible[v] = True
            ncut[v] = cuts
    return pos, out_ptr, cp, win_hi, ncut


def base_candidate(n, C, pos, out_ptr, cons_pos):
    """The no-rematerialisation candidate of the base order, shape [T]."""
    T = n * C
    s = np.zeros(T, dtype=np.int32)
    e = np.zeros(T, dtype=np.int32)
    a = np.zeros(T, dtype=np.uint8)
    for v in range(n):
        k = v * C
        s[k] = pos[v]
        d = out_ptr[v + 1] - out_ptr[v]
        e[k] = max(int(pos[v]), int(cons_pos[out_ptr[v + 1] - 1])) if d else pos[v]
        a[k] = 1
    return s, e, a


def gen_candidates(seed, n, C, B_total, pos, out_ptr, cons_pos, win_hi, ncut, b0, count, dense=False):
    """Candidates b0 .. b0+count-1 of a batch of B_total.

    Returns (starts int32 [count][T], ends int32 [count][T], active uint8 [count][T]).
    """
    T = n * C
    u64 = np.uint64
    starts = np.zeros((count, T), dtype=np.int32)
    ends = np.zeros((count, T), dtype=np.int32)
    active = np.zeros((count, T), dtype=np.uint8)
    if count == 0 or n == 0:
        return starts, ends, active
    b = np.arange(b0, b0 + count, dtype=np.uint64)
    type_b = (b >= u64(B_total // 2))
    with np.errstate(over="ignore"):
        kb = mix64_np(u64((seed ^ CAND_SEED_XOR) & MASK64) + _G * (b + u64(1)))
    for v in range(n):
        with np.errstate(over="ignore"):
            kv = mix64_np(kb + _G * u64(v + 1))

        def draw(j):
            with np.errstate(over="ignore"):
                return mix64_np(kv + _G * u64(j + 1))

        o0, o1 = int(out_ptr[v]), int(out_ptr[v + 1])
        d = o1 - o0
        cp = cons_pos[o0:o1].astype(np.int64)
        pv = int(pos[v])
        end_default = max(pv, int(cp[-1])) if d else pv
        s = np.zeros((count, C), dtype=np.int64)
        e = np.zeros((count, C), dtype=np.int64)
        a = np.zeros((count, C), dtype=np.uint8)
        s[:, 0] = pv
        e[:, 0] = end_default
        a[:, 0] = 1
        nc = int(ncut[v])
        if dense:
            nxt = np.full(count, min(end_default + C - 1, T - 1), dtype=np.int64)   # end of the copy at hand
            for i in range(C - 1, 0, -1):
                keep = (draw(8 + i) & u64(7)) != u64(0)
                a[:, i] = keep.astype(np.uint8)
                s[:, i] = np.where(keep, pv + i, 0)
                e[:, i] = np.where(keep, nxt, 0)
                nxt = np.where(keep, pv + i, nxt)
            e[:, 0] = nxt
        elif nc >= 1:
            wh = int(win_hi[v])
            lo = np.zeros(count, dtype=np.int64)
            alive = np.ones(count, dtype=bool)
            for i in range(1, C):
                avail = nc - lo
                gate = draw(2 * i)
                pick = draw(2 * i + 1)
                take = alive & (avail >= 1) & ((gate & u64(3)) == u64(0))
                if not take.any():
                    break
                safe_avail = np.maximum(avail, 1).astype(np.uint64)
                c = lo + ((pick & u64(0xFFFFFFFF)) % safe_avail).astype(np.int64)
                c = np.minimum(c, d - 2)          # only matters where take is False
                cut = cp[c]
                span = np.minimum(cp[c + 1] - 1, wh) - cut
                nfree = np.maximum(span - span // C, 1).astype(np.uint64)
                q = ((pick >> u64(32)) % nfree).astype(np.int64)
                si = cut + 1 + q + q // (C - 1)
                e[:, i - 1] = np.where(take, cut, e[:, i - 1])
                s[:, i] = np.where(take, si, 0)
                e[:, i] = np.where(take, end_default, 0)
                a[:, i] = take.astype(np.uint8)
                lo = np.where(take, c + 1, lo)
                alive = take
        if type_b.any():
            for i in range(C):
                for f, arr in ((0, s), (1, e)):
                    r = draw(16 + 2 * i + f)
                    move = type_b & (a[:, i] != 0) & ((r & u64(3)) == u64(0))
                    delta = ((r >> u64(8)) % u64(9)).astype(np.int64) - 4
                    arr[:, i] = np.where(move, np.clip(arr[:, i] + delta, 0, T - 1), arr[:, i])
        starts[:, v * C:(v + 1) * C] = s
        ends[:, v * C:(v + 1) * C] = e
        active[:, v * C:(v + 1) * C] = a
    return starts, ends, active
