#!/usr/bin/env python3
"""Benchmark of the batched candidate evaluator on one MI355X.

A step is one pass of the whole hot path (moc_eval_batch: load, structural
checks, start collisions, memory profile, peak, precedence, objective, store)
over one resident batch of synthetic candidates.  Default workload: the
n=5000, C=3, B=262144 configuration (35.4 GB of candidates resident in HBM);
the n=442 and n=1000 configurations are timed as well and reported under
"also" and "also_n1000".

Prints ONE JSON line.  `value` is candidates evaluated per second with inputs
resident in HBM; `roofline` prices the evaluation kernel against the 8 TB/s
HBM peak using its algorithmic bytes (9*T + 24 per candidate); `cpu_baseline`
times the CPU oracle on a bounded sample of the same candidates.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

HBM_PEAK_GBS = 8000.0

# HBM traffic of the evaluation kernel on the default workload, from rocprofv3 counter runs
# (profiles/eval_batch_kernel_n5000_C3_B262144.md): KiB per dispatch and the factors that the same
# counters need to reproduce a 1 GiB device copy.  Valid for the kernel sources they were taken with.
TRAFFIC = {"workload": 4, "B": 262144, "fetch_kib": 17327257.7, "fetch_scale": 2.0, "write_kib": 20496.5,
           "write_scale": 1.0, "sources_sha256": "9a6d2d0cddaeda5267f32f0e1a805490aebad3e0c100055868d8f89440dd056c"}
KERNEL_SOURCES = ("csrc/moc_eval.hip", "csrc/moc_internal.h", "build.py")   # the kernel and how it is compiled


def kernel_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    base = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2304_14463_amd")
    for name in KERNEL_SOURCES:
        with open(os.path.join(base, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(cfg, B):
    """HBM bytes per launch from the committed counter runs, or None when they do not apply
    (another workload, or the kernel has changed since they were taken)."""
    if cfg != TRAFFIC["workload"] or B != TRAFFIC["B"]:
        return None
    try:
        if kernel_sources_sha256() != TRAFFIC["sources_sha256"]:
            return None
    except OSError:
        return None
    return (TRAFFIC["fetch_kib"] * TRAFFIC["fetch_scale"] + TRAFFIC["write_kib"] * TRAFFIC["write_scale"]) * 1024.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=4, choices=[0, 1, 2, 3, 4])
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the secondary (n=442, n=1000) measurements")
    ap.add_argument("--no-neighbours", action="store_true", help="skip the neighbourhood (n=2000) measurement")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run one 1 GiB device copy first (reference dispatch for the HBM byte counters)")
    return ap.parse_args()


def time_eval(moc, gh, cand, steps, warmup):
    """Returns (ms per step over the whole timed region, mean kernel ms from per-launch events)."""
    import torch
    ds, de, da = cand
    B = ds.shape[0]
    out = torch.empty((B, moc.RESULT_DTYPE.itemsize), dtype=torch.uint8, device=ds.device)
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        moc.moc_eval_batch(gh, ds, de, da, out=out, stream=stream)
    torch.cuda.synchronize()
    # launches of well under a millisecond: keep the device busy for a while first, so that the
    # timed steps do not run while its clocks are still coming up
    t0 = time.perf_counter()
    moc.moc_eval_batch(gh, ds, de, da, out=out, stream=stream)
    torch.cuda.synchronize()
    one = max(time.perf_counter() - t0, 1e-6)
    if one < 2e-3:
        for _ in range(int(0.1 / one)):
            moc.moc_eval_batch(gh, ds, de, da, out=out, stream=stream)
        torch.cuda.synchronize()
    begins = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    finishes = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        begins[i].record(stream)
        moc.moc_eval_batch(gh, ds, de, da, out=out, stream=stream)
        finishes[i].record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    kernel_ms = [b.elapsed_time(f) for b, f in zip(begins, finishes)]
    return wall_ms / steps, KernelTimes(kernel_ms), out


class KernelTimes:
    """Per-launch durations (HIP events on the launch stream around every launch)."""

    def __init__(self, ms):
        ms = sorted(ms)
        self.avg, self.min = sum(ms) / len(ms), ms[0]
        self.median = ms[len(ms) // 2] if len(ms) % 2 else 0.5 * (ms[len(ms) // 2 - 1] + ms[len(ms) // 2])


def time_stream_read(cand, steps):
    """The read-only kernel over the same three arrays: best of a few grid sizes.
    Returns (GB/s, workgroups of 1024 threads it was best with)."""
    import torch
    from paper_2304_14463_amd.inputs import stream_read
    nbytes = sum(t.numel() * t.element_size() for t in cand)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    best = (0.0, 0)
    for per_cu in (1, 4, 16):
        blocks = cus * per_cu
        out = stream_read(cand, blocks)
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        ms = []
        for _ in range(max(3, min(steps, 10))):
            b, f = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            b.record(stream)
            stream_read(cand, blocks, out=out)
            f.record(stream)
            f.synchronize()
            ms.append(b.elapsed_time(f))
        gbs = nbytes / (KernelTimes(ms).median * 1e-3) / 1e9
        if gbs > best[0]:
            best = (gbs, blocks)
    return best


def measure(moc, cfg, steps, warmup, batch=None, dense=False):
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload, make_workload
    w = make_workload(cfg, batch, dense=dense)
    g = w.graph
    gh = moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, w.budget, w.C)
    cand = DeviceWorkload(w).candidates()
    torch.cuda.synchronize()
    ms_step, kt, out = time_eval(moc, gh, cand, steps, warmup)
    res = moc.results_to_numpy(out)
    bytes_per_cand = 9 * w.T + 24
    # how many of the copies are active, and how many nodes have an active copy besides the first
    rows = min(w.B, 4096)
    act = (cand[2][:rows] != 0).view(rows, w.n, w.C)
    info = {
        "workload": w.name, "n": w.n, "m": w.m, "C": w.C, "T": w.T, "B": w.B,
        "budget_pct_of_no_remat_peak": w.pct, "bytes_per_candidate": bytes_per_cand,
        "frac_violation_free": float((res["violations"] == 0).mean()),
        "frac_feasible": float(res["feasible"].mean()),
        "frac_copies_active": float(act.float().mean()),
        "frac_nodes_with_further_copies": float(act[:, :, 1:].any(dim=2).float().mean()) if w.C > 1 else 0.0,
    }
    gbs = w.B * bytes_per_cand / (kt.avg * 1e-3) / 1e9
    return w, gh, cand, res, info, ms_step, kt, gbs


def secondary(moc, cfg, steps, warmup, batch=None, dense=False):
    """One more evaluation line: config, rate, per-launch times, fraction of the HBM peak."""
    import torch
    w, gh, cand, res, info, ms, kt, gbs = measure(moc, cfg, steps, warmup, batch, dense)
    line = {"config": info, "value": w.B / (ms * 1e-3), "unit": "candidates/s", "ms_per_step": ms,
            "kernel_ms_avg": kt.avg, "kernel_ms_median": kt.median, "kernel_ms_min": kt.min, "achieved_GBs": gbs,
            "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    if kt.avg < 1.0:
        # Launches this short: a pair of events around one launch adds a few microseconds to it.
        # The same launches queued one behind the other between one pair of events give the time
        # a launch takes in a stream of them (what a search that evaluates batch after batch sees).
        ds, de, da = cand
        out = torch.empty((w.B, moc.RESULT_DTYPE.itemsize), dtype=torch.uint8, device=ds.device)
        stream = torch.cuda.current_stream()
        count = 200
        b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        b0.record(stream)
        for _ in range(count):
            moc.moc_eval_batch(gh, ds, de, da, out=out, stream=stream)
        b1.record(stream)
        b1.synchronize()
        each = b0.elapsed_time(b1) / count
        line["kernel_ms_in_a_stream_of_200"] = each
        line["frac_of_hbm_peak_in_a_stream"] = w.B * info["bytes_per_candidate"] / (each * 1e-3) / 1e9 / HBM_PEAK_GBS
    gh.free()
    del cand
    torch.cuda.empty_cache()
    return line


def measure_neighbours(moc, steps, warmup, with_cpu_baseline=True):
    """moc_eval_neighbours on the n=2000, C=2, R=8 workload: all 128000 moves of 8192 bases."""
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload, make_workload
    w = make_workload(3)
    g = w.graph
    gh = moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, w.budget, w.C)
    ds, de, da = DeviceWorkload(w).candidates()
    n_moves = w.T * 4 * w.R
    out = {}
    for mode, (wm, wb) in (("full_table", (True, True)), ("best_only", (False, True))):
        om, ob = moc.moc_eval_neighbours(gh, ds, de, da, w.R, want_moves=wm, want_best=wb)
        for _ in range(warmup):
            moc.moc_eval_neighbours(gh, ds, de, da, w.R, want_moves=wm, want_best=wb, out_moves=om, out_best=ob)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            moc.moc_eval_neighbours(gh, ds, de, da, w.R, want_moves=wm, want_best=wb, out_moves=om, out_best=ob)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        out[mode] = {"ms_per_step": ms, "moves_per_s": w.B * n_moves / (ms * 1e-3),
                     "bytes_written": (w.B * n_moves * 8 if wm else 0) + w.B * 16}
        del om, ob
    if with_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = cpu_baseline_neighbours(moc, w, gh, (ds, de, da))
    # the moves that change the objective: one active flag flipped, B x T of them
    ot = moc.moc_eval_toggles(gh, ds, de, da)
    for _ in range(warmup):
        moc.moc_eval_toggles(gh, ds, de, da, out=ot)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        moc.moc_eval_toggles(gh, ds, de, da, out=ot)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    out["toggles"] = {"ms_per_step": ms, "moves_per_s": w.B * w.T / (ms * 1e-3), "bytes_written": w.B * w.T * 16}
    del ot
    # the moves that trade duration for memory: one per in-edge and copy of its consumer
    oc, ob = moc.moc_eval_cuts(gh, ds, de, da, want_best=True)
    ms_cuts = {}
    for mode, (om, wm) in (("table_and_best", (oc, True)), ("best_only", (None, False))):
        for _ in range(warmup):
            moc.moc_eval_cuts(gh, ds, de, da, want_moves=wm, want_best=True, out_moves=om, out_best=ob)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            moc.moc_eval_cuts(gh, ds, de, da, want_moves=wm, want_best=True, out_moves=om, out_best=ob)
        torch.cuda.synchronize()
        ms_cuts[mode] = (time.perf_counter() - t0) * 1e3 / steps
    ms = ms_cuts["table_and_best"]
    applicable = float((moc.results_to_numpy(oc[:64], moc.TOGGLE_SCORE_DTYPE)["violations"] >= 0).mean())
    out["cuts"] = {"ms_per_step": ms, "moves_per_s": w.B * w.m * w.C / (ms * 1e-3),
                   "bytes_written": w.B * w.m * w.C * 16, "frac_applicable": applicable,
                   "best_only_ms_per_step": ms_cuts["best_only"]}
    # the cuts of the two-phase search's first phase: the producer's missing inputs are kept until the recomputation
    keep_steps = max(1, steps // 2)
    moc.moc_eval_cuts(gh, ds, de, da, want_moves=True, want_best=True, out_moves=oc, out_best=ob, keep_inputs=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(keep_steps):
        moc.moc_eval_cuts(gh, ds, de, da, want_moves=True, want_best=True, out_moves=oc, out_best=ob, keep_inputs=True)
    torch.cuda.synchronize()
    ms_keep = (time.perf_counter() - t0) * 1e3 / keep_steps
    out["cuts"]["keep_inputs"] = {
        "ms_per_step": ms_keep, "moves_per_s": w.B * w.m * w.C / (ms_keep * 1e-3),
        "frac_applicable": float((moc.results_to_numpy(oc[:64], moc.TOGGLE_SCORE_DTYPE)["violations"] >= 0).mean())}
    del oc, ob
    # greedy descent by cuts from the violation-free bases: 16 steps of score, choose, apply
    ev0 = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    walkers = torch.from_numpy((ev0["violations"] == 0).nonzero()[0]).cuda()
    walkers = walkers[torch.arange(w.B, device="cuda") % walkers.numel()]
    ws, we, wa = ds[walkers].contiguous(), de[walkers].contiguous(), da[walkers].contiguous()
    ev0 = moc.results_to_numpy(moc.moc_eval_batch(gh, ws, we, wa))
    search_steps = 16
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    applied = moc.moc_search_cuts(gh, ws, we, wa, search_steps)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    ev1 = moc.results_to_numpy(moc.moc_eval_batch(gh, ws, we, wa))
    # what comes out is still a schedule: decode every walker and cost the sequence on its own terms
    cert = moc.results_to_numpy(moc.moc_decode_batch(gh, ws, wa, want_seq=False)[0], moc.DECODE_RESULT_DTYPE)
    certified = bool(((cert["status"] == 1) & (cert["duration"] == ev1["duration"]) & (cert["peak"] <= ev1["peak"])).all())
    gap0 = (ev0["peak"] - w.budget).clip(min=0).astype(float)
    gap1 = (ev1["peak"] - w.budget).clip(min=0).astype(float)
    out["search_cuts"] = {
        "steps": search_steps, "ms_total": ms, "ms_per_step": ms / search_steps,
        "walkers": w.B, "mean_moves_applied": float(applied.float().mean()),
        "violations_after": int(ev1["violations"].max()), "decoded_and_certified": certified,
        "mean_gap_to_budget_closed": float(1.0 - gap1.sum() / max(gap0.sum(), 1.0)),
        "frac_feasible_before": float(ev0["feasible"].mean()), "frac_feasible_after": float(ev1["feasible"].mean()),
        "mean_duration_increase_pct": float(100.0 * (ev1["duration"] / ev0["duration"] - 1.0).mean())}
    # the same walkers, descent by single-field moves (no duration at stake)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    moved = moc.moc_search_moves(gh, ws, we, wa, w.R, search_steps)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    ev2 = moc.results_to_numpy(moc.moc_eval_batch(gh, ws, we, wa))
    out["search_moves"] = {"steps": search_steps, "R": w.R, "ms_total": ms, "ms_per_step": ms / search_steps,
                           "walkers": w.B, "mean_moves_applied": float(moved.float().mean()),
                           "violations_after": int(ev2["violations"].max()),
                           "mean_peak_change_pct": float(100.0 * (ev2["peak"] / ev1["peak"] - 1.0).mean())}
    del ws, we, wa
    # back to sequences: every base decoded and costed, sequences written out
    # -- of the candidates a search would decode: the violation-free bases, repeated to B rows
    ev = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    clean = torch.from_numpy((ev["violations"] == 0).nonzero()[0]).cuda()
    pick = clean[torch.arange(w.B, device="cuda") % clean.numel()]
    ds, da = ds[pick].contiguous(), da[pick].contiguous()
    del de
    od, oq = moc.moc_decode_batch(gh, ds, da)
    valid = float((moc.results_to_numpy(od, moc.DECODE_RESULT_DTYPE)["status"] == 1).mean())
    for _ in range(warmup):
        moc.moc_decode_batch(gh, ds, da, out=od, out_seq=oq)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        moc.moc_decode_batch(gh, ds, da, out=od, out_seq=oq)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    dec_bytes = w.B * (5 * w.T + 4 * w.T + 24)
    out["decode"] = {"ms_per_step": ms, "candidates_per_s": w.B / (ms * 1e-3), "bytes_per_candidate": 9 * w.T + 24,
                     "frac_valid": valid, "distinct_candidates": int(clean.numel()), "gb_per_s": dec_bytes / (ms * 1e-3) / 1e9}
    del od, oq
    gh.free()
    return {"workload": w.name, "n": w.n, "m": w.m, "C": w.C, "T": w.T, "B": w.B, "R": w.R,
            "moves_per_candidate": n_moves, **out}


def cpu_baseline(w, cand, res, target_seconds=15.0):
    """Times oracle.evaluate (single thread, as it stands) on the first candidates of the batch."""
    import numpy as np
    import oracle
    ds, de, da = cand
    probe = 8
    s, e, a = ds[:probe].cpu().numpy(), de[:probe].cpu().numpy(), da[:probe].cpu().numpy()
    t0 = time.perf_counter()
    oracle.evaluate(w.graph, w.budget, w.C, s, e, a)
    per = max((time.perf_counter() - t0) / probe, 1e-7)
    count = int(max(probe, min(w.B, target_seconds / per)))
    s, e, a = ds[:count].cpu().numpy(), de[:count].cpu().numpy(), da[:count].cpu().numpy()
    t0 = time.perf_counter()
    ref = oracle.evaluate(w.graph, w.budget, w.C, s, e, a)
    dt = time.perf_counter() - t0
    ok = all((res[name][:count].astype(np.int64) == ref[:, i]).all()
             for i, name in enumerate(("peak", "duration", "violations", "feasible")))
    # same function on all host cores (disjoint candidate ranges, one thread each)
    cores = min(os.cpu_count() or 1, 16)
    cuts = np.linspace(0, count, cores + 1).astype(int)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(lambda i: oracle.evaluate(w.graph, w.budget, w.C, s[cuts[i]:cuts[i + 1]],
                                              e[cuts[i]:cuts[i + 1]], a[cuts[i]:cuts[i + 1]]), range(cores)))
    dt_all = time.perf_counter() - t0
    return ({"value": count / dt, "unit": "candidates/s", "cores": 1, "kind": "oracle",
             "sample": f"first {count} candidates of the batch, single-threaded oracle.evaluate",
             "matches_gpu": bool(ok)},
            {"value": count / dt_all, "unit": "candidates/s", "cores": cores, "kind": "oracle",
             "sample": f"same {count} candidates split over {cores} host threads"})


def measure_staged(moc, steps, warmup, with_cpu_baseline=True):
    """moc_eval_batch_staged (stage-restricted domain of Section 2.3) on the n=1000 training-shaped
    graph: 8192 staged candidates generated on the host, repeated to 65536 rows on the device."""
    import numpy as np
    import torch
    from paper_2304_14463_amd.inputs import make_workload
    from paper_2304_14463_amd.inputs.staged import gen_staged_candidates, staged_tables
    w = make_workload(2)
    g = w.graph
    unique, reps = 8192, 8
    tables = staged_tables(g, w.order)
    s, e, a = gen_staged_candidates(w.seed, g, w.order, w.C, unique, 0, unique, tables)
    gh = moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, w.budget, w.C)
    moc.moc_graph_set_order(gh, w.order)
    ds, de, da = (torch.from_numpy(x).cuda().repeat(reps, 1) for x in (s, e, a))
    B = unique * reps
    out = moc.moc_eval_batch_staged(gh, ds, de, da)
    for _ in range(warmup):
        moc.moc_eval_batch_staged(gh, ds, de, da, out=out)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    ms = []
    for _ in range(steps):
        b, f = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        b.record(stream)
        moc.moc_eval_batch_staged(gh, ds, de, da, out=out)
        f.record(stream)
        f.synchronize()
        ms.append(b.elapsed_time(f))
    kt = KernelTimes(ms)
    res = moc.results_to_numpy(out)
    line = {"workload": w.name + "-staged", "n": w.n, "m": w.m, "C": w.C, "positions": w.n * (w.n + 1) // 2, "B": B,
            "distinct_candidates": unique, "kernel_ms_avg": kt.avg, "kernel_ms_median": kt.median, "kernel_ms_min": kt.min,
            "candidates_per_s": B / (kt.median * 1e-3), "bytes_per_candidate": 9 * w.T + 24,
            "achieved_GBs": B * (9 * w.T + 24) / (kt.median * 1e-3) / 1e9,
            "frac_of_hbm_peak": B * (9 * w.T + 24) / (kt.median * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "frac_violation_free": float((res["violations"] == 0).mean())}
    if with_cpu_baseline:
        import oracle
        count = 128
        t0 = time.perf_counter()
        ref = oracle.evaluate_staged(g, w.budget, w.C, tables[0], s[:count], e[:count], a[:count])
        dt = time.perf_counter() - t0
        ok = all((res[name][:count].astype(np.int64) == ref[:, i]).all()
                 for i, name in enumerate(("peak", "duration", "violations", "feasible")))
        line["cpu_baseline"] = {"value": count / dt, "unit": "candidates/s", "cores": 1, "kind": "oracle",
                                "sample": f"first {count} candidates, single-threaded oracle.evaluate_staged",
                                "matches_gpu": bool(ok)}
    gh.free()
    return line


def measure_two_phase(moc, cfg, walkers, max_cuts, max_merges, K):
    """moc_search_two_phase from the violation-free candidates of a workload: how many walkers
    end within the budget, at what increase of the total duration over the plain schedule (the
    paper's TDI %), and whether every result decodes to a valid sequence of that cost."""
    import numpy as np
    import torch
    from paper_2304_14463_amd.inputs import DeviceWorkload, make_workload
    w = make_workload(cfg, 4 * walkers)
    g = w.graph
    gh = moc.moc_graph_upload(g.n, g.in_ptr, g.in_idx, g.size, g.dur, w.budget, w.C)
    ds, de, da = DeviceWorkload(w).candidates(0, 2 * walkers)       # the first half of a batch: no perturbed rows
    ev = moc.results_to_numpy(moc.moc_eval_batch(gh, ds, de, da))
    clean = torch.from_numpy((ev["violations"] == 0).nonzero()[0]).cuda()
    pick = clean[torch.arange(walkers, device="cuda") % clean.numel()]
    ws, we, wa = ds[pick].contiguous(), de[pick].contiguous(), da[pick].contiguous()
    base = w.base()
    for x, row in zip((ws, we, wa), base):
        x[0] = torch.from_numpy(row).cuda()                          # walker 0: the plain schedule itself
    ev0 = moc.results_to_numpy(moc.moc_eval_batch(gh, ws, we, wa))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    cuts, merges = moc.moc_search_two_phase(gh, ws, we, wa, max_cuts, max_merges, K)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    ev1 = moc.results_to_numpy(moc.moc_eval_batch(gh, ws, we, wa))
    cert = moc.results_to_numpy(moc.moc_decode_batch(gh, ws, wa, want_seq=False)[0], moc.DECODE_RESULT_DTYPE)
    certified = bool(((cert["status"] == 1) & (cert["duration"] == ev1["duration"]) & (cert["peak"] <= ev1["peak"])).all())
    total_w = float(g.dur.sum())
    tdi = 100.0 * (ev1["duration"] / total_w - 1.0)
    ok = ev1["feasible"] == 1
    gh.free()
    return {"workload": w.name, "n": w.n, "m": w.m, "C": w.C, "budget_pct_of_no_remat_peak": w.pct, "walkers": walkers,
            "distinct_starts": int(clean.numel()), "max_cuts": max_cuts, "max_merges": max_merges, "K": K,
            "ms_total": ms, "mean_cuts_applied": float(cuts.float().mean()), "mean_merges_applied": float(merges.float().mean()),
            "frac_feasible_before": float(ev0["feasible"].mean()), "frac_feasible_after": float(ok.mean()),
            "violations_after": int(ev1["violations"].max()), "decoded_and_certified": certified,
            "tdi_pct_mean_of_feasible": float(tdi[ok].mean()) if ok.any() else None,
            "tdi_pct_min_of_feasible": float(tdi[ok].min()) if ok.any() else None,
            "tdi_pct_plain_schedule_walker": float(tdi[0]), "plain_schedule_walker_feasible": bool(ok[0]),
            "mean_peak_pct_of_no_remat_peak_after": float(100.0 * ev1["peak"].mean() / w.no_remat_peak)}


def cpu_baseline_neighbours(moc, w, gh, cand, target_seconds=10.0):
    """Times oracle.neighbours (full re-evaluation of every move, as it stands) on a sample of the
    moves of the first bases: every 16th move of base 0 on one thread, then every 16th move of
    as many bases as there are host threads, one base per thread; compared with the GPU's table."""
    import numpy as np
    import torch
    import oracle
    ds, de, da = cand
    R = w.R
    n_moves = w.T * 4 * R
    cores = min(os.cpu_count() or 1, 16)
    host = [(ds[b].cpu().numpy(), de[b].cpu().numpy(), da[b].cpu().numpy()) for b in range(cores)]
    probe = np.arange(0, n_moves, n_moves // 64, dtype=np.int64)
    t0 = time.perf_counter()
    oracle.neighbours(w.graph, w.budget, w.C, *host[0], R, moves=probe)
    per = max((time.perf_counter() - t0) / len(probe), 1e-7)
    stride = max(1, int(n_moves * per / target_seconds))
    pick = np.arange(0, n_moves, stride, dtype=np.int64)
    t0 = time.perf_counter()
    ref0, _ = oracle.neighbours(w.graph, w.budget, w.C, *host[0], R, moves=pick)
    dt = time.perf_counter() - t0
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        refs = list(ex.map(lambda b: oracle.neighbours(w.graph, w.budget, w.C, *host[b], R, moves=pick)[0], range(cores)))
    dt_all = time.perf_counter() - t0
    om, _ = moc.moc_eval_neighbours(gh, ds[:cores], de[:cores], da[:cores], R, want_moves=True, want_best=False)
    table = moc.results_to_numpy(om, moc.MOVE_SCORE_DTYPE)
    ok = all((table[b]["violations"][pick] == refs[b][:, 0]).all() and (table[b]["peak"][pick] == refs[b][:, 1]).all()
             for b in range(cores)) and (refs[0] == ref0).all()
    del om
    return ({"value": len(pick) / dt, "unit": "moves/s", "cores": 1, "kind": "oracle",
             "sample": f"every {stride}th of the {n_moves} moves of base 0 ({len(pick)} moves), single-threaded "
                       "oracle.neighbours", "matches_gpu": bool(ok)},
            {"value": cores * len(pick) / dt_all, "unit": "moves/s", "cores": cores, "kind": "oracle",
             "sample": f"the same {len(pick)} moves of bases 0..{cores - 1}, one base per host thread"})


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU only (candidates shard trivially by batch; "
                 "no multi-GPU path is built). Use --gpus 1.")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the evaluator has no CPU fallback.")
    from paper_2304_14463_amd import moccasin as moc
    moc.lib()
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    w, gh, cand, res, info, ms_step, kt, gbs = measure(moc, args.workload, args.steps, args.warmup, args.batch)
    read_gbs, read_blocks = time_stream_read(cand, args.steps)
    line = {
        "metric": "candidate schedules evaluated/sec",
        "value": w.B / (ms_step * 1e-3),
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": info,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": measured_traffic(args.workload, w.B),
                     "kernel": "eval_batch_kernel", "kernel_ms_avg": kt.avg, "kernel_ms_median": kt.median,
                     "kernel_ms_min": kt.min,
                     "algorithmic_bytes_per_launch": w.B * info["bytes_per_candidate"],
                     # what a kernel that only reads the same three arrays reaches on this GPU
                     "stream_read_GBs": read_gbs, "stream_read_workgroups": read_blocks,
                     "frac_of_stream_read": gbs / read_gbs},
    }
    if not args.no_cpu_baseline:
        one, allc = cpu_baseline(w, cand, res)
        line["cpu_baseline"] = one
        line["cpu_baseline_all_cores"] = allc
    del cand
    gh.free()
    torch.cuda.empty_cache()
    if not args.no_also and args.workload != 1:
        line["also"] = secondary(moc, 1, max(args.steps, 50), args.warmup)
        # the smallest configuration with n >= 1000: training-shaped graph, B = 65536
        line["also_n1000"] = secondary(moc, 2, max(args.steps, 50), args.warmup)
        # the default workload's graph with the dense batch (nearly every copy live): how far the
        # rate depends on the candidates having few copies beyond the first
        line["also_dense"] = secondary(moc, args.workload, args.steps, args.warmup, batch=65536, dense=True)
    if not args.no_also:
        torch.cuda.empty_cache()
        line["staged"] = measure_staged(moc, max(5, args.steps // 2), 2, not args.no_cpu_baseline)
    if not args.no_also:
        torch.cuda.empty_cache()
        line["two_phase"] = [measure_two_phase(moc, 1, 1024, 64, 48, 64), measure_two_phase(moc, 2, 1024, 128, 48, 128),
                             measure_two_phase(moc, 3, 256, 640, 32, 128)]
    if not args.no_neighbours:
        torch.cuda.empty_cache()
        line["neighbours"] = measure_neighbours(moc, max(3, args.steps // 4), 1, not args.no_cpu_baseline)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
