"""Python binding of libmoccasin_hip.so (C ABI in include/moccasin.h).

Argument marshalling only: every step of the evaluation runs in the HIP
kernels of the library.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams); graph arrays are host numpy arrays.  There is
no CPU fallback: a missing library or GPU raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoccasin_hip.so")
_lib = None

MOC_MAX_T = 19455

# numpy views of the result structs of include/moccasin.h
RESULT_DTYPE = np.dtype([("peak", "<i8"), ("duration", "<i8"), ("violations", "<i4"), ("feasible", "<i4")])
MOVE_SCORE_DTYPE = np.dtype([("violations", "<i4"), ("peak", "<i4")])
BEST_MOVE_DTYPE = np.dtype([("move", "<i4"), ("violations", "<i4"), ("peak", "<i8")])
TOGGLE_SCORE_DTYPE = np.dtype([("violations", "<i4"), ("peak", "<i4"), ("duration", "<i8")])
DECODE_RESULT_DTYPE = np.dtype([("status", "<i4"), ("length", "<i4"), ("peak", "<i8"), ("duration", "<i8")])

EXPORTS = ("moc_graph_upload", "moc_graph_info", "moc_eval_batch", "moc_eval_batch_noalloc", "moc_graph_set_order", "moc_eval_batch_staged", "moc_eval_neighbours", "moc_eval_toggles",
           "moc_eval_cuts", "moc_eval_cuts_keep", "moc_search_cuts", "moc_search_two_phase", "moc_search_moves", "moc_decode_batch", "moc_graph_free", "moc_strerror", "moc_last_hip_error")


class MoccasinError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = lib().moc_strerror(code).decode()
        hip = lib().moc_last_hip_error() if code == -4 else 0
        super().__init__(f"{where}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))


def lib():
    """Load the shared library (build it first with `python -m paper_2304_14463_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run python -m paper_2304_14463_amd.build")
        L = ctypes.CDLL(LIB_PATH)
        P, I32, I64, VP = ctypes.POINTER, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.moc_graph_upload.argtypes = [I32, VP, VP, VP, VP, I64, I32, P(VP)]
        L.moc_graph_upload.restype = ctypes.c_int
        L.moc_graph_info.argtypes = [VP, P(I32), P(I32), P(I32), P(I32)]
        L.moc_graph_info.restype = ctypes.c_int
        L.moc_eval_batch.argtypes = [VP, I64, VP, VP, VP, VP, VP]
        L.moc_eval_batch.restype = ctypes.c_int
        L.moc_eval_batch_noalloc.argtypes = [VP, I64, VP, VP, VP, VP, VP]
        L.moc_eval_batch_noalloc.restype = ctypes.c_int
        L.moc_graph_set_order.argtypes = [VP, VP]
        L.moc_graph_set_order.restype = ctypes.c_int
        L.moc_eval_batch_staged.argtypes = [VP, I64, VP, VP, VP, VP, VP]
        L.moc_eval_batch_staged.restype = ctypes.c_int
        L.moc_eval_neighbours.argtypes = [VP, I64, VP, VP, VP, I32, VP, VP, VP]
        L.moc_eval_neighbours.restype = ctypes.c_int
        L.moc_eval_toggles.argtypes = [VP, I64, VP, VP, VP, VP, VP]
        L.moc_eval_toggles.restype = ctypes.c_int
        L.moc_eval_cuts.argtypes = [VP, I64, VP, VP, VP, VP, VP, VP]
        L.moc_eval_cuts.restype = ctypes.c_int
        L.moc_eval_cuts_keep.argtypes = [VP, I64, VP, VP, VP, VP, VP, VP]
        L.moc_eval_cuts_keep.restype = ctypes.c_int
        L.moc_search_two_phase.argtypes = [VP, I64, VP, VP, VP, I32, I32, I32, VP, VP, VP, VP, VP, VP, VP, VP, VP]
        L.moc_search_two_phase.restype = ctypes.c_int
        L.moc_search_cuts.argtypes = [VP, I64, VP, VP, VP, I32, VP, VP, VP]
        L.moc_search_cuts.restype = ctypes.c_int
        L.moc_search_moves.argtypes = [VP, I64, VP, VP, VP, I32, I32, VP, VP, VP, VP]
        L.moc_search_moves.restype = ctypes.c_int
        L.moc_decode_batch.argtypes = [VP, I64, VP, VP, VP, VP, VP]
        L.moc_decode_batch.restype = ctypes.c_int
        L.moc_graph_free.argtypes = [VP]
        L.moc_graph_free.restype = None
        L.moc_strerror.argtypes = [ctypes.c_int]
        L.moc_strerror.restype = ctypes.c_char_p
        L.moc_last_hip_error.argtypes = []
        L.moc_last_hip_error.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(code, where):
    if code != 0:
        raise MoccasinError(code, where)


def _host(arr, n):
    a = np.ascontiguousarray(arr, dtype=np.int32).reshape(-1)
    if a.shape[0] != n:
        raise ValueError(f"expected {n} int32 values, got {a.shape[0]}")
    return a


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _on(stream):
    """Context in which tensors are allocated for use on `stream`: a workspace that this module
    allocates and drops while kernels queued on `stream` still use it must belong to that
    stream for torch's allocator, or it could be handed to work on another stream too early."""
    import contextlib
    import torch
    return torch.cuda.stream(stream) if stream is not None else contextlib.nullcontext()


class Graph:
    """Handle of an uploaded problem instance (moc_graph_upload / moc_graph_free)."""

    def __init__(self, handle, n, m, C):
        self._h = handle
        self.n, self.m, self.C, self.T = n, m, C, n * C

    def free(self):
        if self._h is not None:
            lib().moc_graph_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def moc_graph_upload(n, in_ptr, in_idx, size, dur, budget, C) -> Graph:
    in_ptr = _host(in_ptr, n + 1)
    m = int(in_ptr[-1])
    in_idx = _host(in_idx, len(np.asarray(in_idx).reshape(-1)))
    size, dur = _host(size, n), _host(dur, n)
    h = ctypes.c_void_p()
    code = lib().moc_graph_upload(n, in_ptr.ctypes.data, in_idx.ctypes.data if in_idx.size else None,
                                  size.ctypes.data, dur.ctypes.data, int(budget), int(C), ctypes.byref(h))
    _check(code, "moc_graph_upload")
    return Graph(h, n, m, int(C))


def _cand_ptrs(g, B, starts, ends, active):
    import torch
    for t, dt in ((starts, torch.int32), (ends, torch.int32), (active, torch.uint8)):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous() or t.numel() != B * g.T:
            raise ValueError("candidate arrays must be contiguous CUDA tensors [B][T]: int32, int32, uint8")
    return ctypes.c_void_p(starts.data_ptr()), ctypes.c_void_p(ends.data_ptr()), ctypes.c_void_p(active.data_ptr())


def moc_eval_batch(g: Graph, starts, ends, active, out=None, stream=None):
    """Evaluate B candidates; returns a uint8 CUDA tensor [B][24] holding moc_result records
    (see results_to_numpy).  Asynchronous on `stream` (default: torch's current stream)."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    if out is None:
        out = torch.empty((B, RESULT_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    code = lib().moc_eval_batch(g._h, B, ps, pe, pa, ctypes.c_void_p(out.data_ptr()), _stream_handle(stream))
    _check(code, "moc_eval_batch")
    return out


def moc_eval_batch_noalloc(g: Graph, starts, ends, active, out, stream=None):
    """moc_eval_batch with the work counters in the library's static device array; `out` is the
    caller's uint8 CUDA tensor [B][24].  Nothing is allocated, here or in the library."""
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    if not (out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= B * RESULT_DTYPE.itemsize):
        raise ValueError("out must be a contiguous CUDA tensor of at least B * 24 bytes")
    code = lib().moc_eval_batch_noalloc(g._h, B, ps, pe, pa, ctypes.c_void_p(out.data_ptr()), _stream_handle(stream))
    _check(code, "moc_eval_batch_noalloc")
    return out


def moc_graph_set_order(g: Graph, order):
    """Give the graph the topological order of the stage-restricted domain (host array [n])."""
    order = _host(order, g.n)
    _check(lib().moc_graph_set_order(g._h, order.ctypes.data), "moc_graph_set_order")


def moc_eval_batch_staged(g: Graph, starts, ends, active, out=None, stream=None):
    """Evaluate B candidates in the stage-restricted domain; returns a uint8 CUDA tensor [B][24]
    of moc_result records."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    if out is None:
        out = torch.empty((B, RESULT_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    code = lib().moc_eval_batch_staged(g._h, B, ps, pe, pa, ctypes.c_void_p(out.data_ptr()), _stream_handle(stream))
    _check(code, "moc_eval_batch_staged")
    return out


def moc_eval_neighbours(g: Graph, starts, ends, active, R, want_moves=True, want_best=True, out_moves=None,
                        out_best=None, stream=None):
    """Score all single-field moves of B candidates.  Returns (moves, best): uint8 CUDA tensors
    [B][T*4R][8] (moc_move_score) and [B][16] (moc_best_move), or None where not requested."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    if want_moves and out_moves is None:
        out_moves = torch.empty((B, g.T * 4 * R, MOVE_SCORE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    if want_best and out_best is None:
        out_best = torch.empty((B, BEST_MOVE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    code = lib().moc_eval_neighbours(
        g._h, B, ps, pe, pa, int(R),
        ctypes.c_void_p(out_moves.data_ptr()) if out_moves is not None else None,
        ctypes.c_void_p(out_best.data_ptr()) if out_best is not None else None, _stream_handle(stream))
    _check(code, "moc_eval_neighbours")
    return out_moves, out_best


def moc_eval_toggles(g: Graph, starts, ends, active, out=None, stream=None):
    """Score the B x T candidates that differ from a base in one active flag.  Returns a uint8
    CUDA tensor [B][T][16] (moc_toggle_score)."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    if out is None:
        out = torch.empty((B, g.T, TOGGLE_SCORE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    code = lib().moc_eval_toggles(g._h, B, ps, pe, pa, ctypes.c_void_p(out.data_ptr()), _stream_handle(stream))
    _check(code, "moc_eval_toggles")
    return out


def moc_eval_cuts(g: Graph, starts, ends, active, want_moves=True, want_best=False, out_moves=None, out_best=None,
                  stream=None, keep_inputs=False):
    """Score the B x m*C cut-and-recompute moves.  Returns (uint8 CUDA tensor [B][m*C][16] of
    moc_cut_score or None, uint8 CUDA tensor [B][16] of moc_best_move or None)."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    if out_moves is None and want_moves:
        out_moves = torch.empty((B, g.m * g.C, TOGGLE_SCORE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    if out_best is None and want_best:
        out_best = torch.empty((B, BEST_MOVE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    call = lib().moc_eval_cuts_keep if keep_inputs else lib().moc_eval_cuts
    code = call(
        g._h, B, ps, pe, pa, ctypes.c_void_p(out_moves.data_ptr()) if out_moves is not None else None,
        ctypes.c_void_p(out_best.data_ptr()) if out_best is not None else None, _stream_handle(stream))
    _check(code, "moc_eval_cuts")
    return out_moves, out_best


def moc_search_cuts(g: Graph, starts, ends, active, max_steps, work_best=None, out_steps=None, stream=None):
    """Greedy descent by cut-and-recompute moves, in place.  Returns the int32 CUDA tensor [B] of
    moves applied per candidate."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    with _on(stream):
        if work_best is None:
            work_best = torch.empty((B, BEST_MOVE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
        if out_steps is None:
            out_steps = torch.empty((B,), dtype=torch.int32, device=starts.device)
    code = lib().moc_search_cuts(g._h, B, ps, pe, pa, int(max_steps), ctypes.c_void_p(work_best.data_ptr()),
                                 ctypes.c_void_p(out_steps.data_ptr()), _stream_handle(stream))
    _check(code, "moc_search_cuts")
    return out_steps


def moc_search_two_phase(g: Graph, starts, ends, active, max_cuts, max_merges, K=64, stream=None):
    """Two-phase local search in place (cuts that keep the inputs towards the budget, then merges
    that lower the duration).  Returns (cuts, merges): int32 CUDA tensors [B] of moves applied."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    dev = starts.device
    with _on(stream):
        work_best = torch.empty((B, BEST_MOVE_DTYPE.itemsize), dtype=torch.uint8, device=dev)
        rows = B * K if max_merges > 0 else 0
        ws = torch.empty((rows, g.T), dtype=torch.int32, device=dev)
        we = torch.empty((rows, g.T), dtype=torch.int32, device=dev)
        wa = torch.empty((rows, g.T), dtype=torch.uint8, device=dev)
        wl = torch.empty((rows,), dtype=torch.int32, device=dev)
        wr = torch.empty((rows, RESULT_DTYPE.itemsize), dtype=torch.uint8, device=dev)
        cuts = torch.empty((B,), dtype=torch.int32, device=dev)
        merges = torch.empty((B,), dtype=torch.int32, device=dev)
    P = lambda t: ctypes.c_void_p(t.data_ptr()) if t.numel() else None
    code = lib().moc_search_two_phase(g._h, B, ps, pe, pa, int(max_cuts), int(max_merges), int(K), P(work_best), P(ws),
                                      P(we), P(wa), P(wl), P(wr), P(cuts), P(merges), _stream_handle(stream))
    _check(code, "moc_search_two_phase")
    return cuts, merges


def moc_search_moves(g: Graph, starts, ends, active, R, max_steps, out_steps=None, stream=None):
    """Greedy descent by single-field start/end moves of radius R, in place.  Returns the int32
    CUDA tensor [B] of moves applied per candidate."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    ps, pe, pa = _cand_ptrs(g, B, starts, ends, active)
    with _on(stream):
        work_results = torch.empty((B, RESULT_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
        work_best = torch.empty((B, BEST_MOVE_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
        if out_steps is None:
            out_steps = torch.empty((B,), dtype=torch.int32, device=starts.device)
    code = lib().moc_search_moves(g._h, B, ps, pe, pa, int(R), int(max_steps),
                                  ctypes.c_void_p(work_results.data_ptr()), ctypes.c_void_p(work_best.data_ptr()),
                                  ctypes.c_void_p(out_steps.data_ptr()), _stream_handle(stream))
    _check(code, "moc_search_moves")
    return out_steps


def moc_decode_batch(g: Graph, starts, active, want_seq=True, out=None, out_seq=None, stream=None):
    """Decode B candidates to their sequences.  Returns (uint8 CUDA tensor [B][24] of
    moc_decode_result, int32 CUDA tensor [B][T] of sequences or None)."""
    import torch
    B = starts.numel() // g.T if g.T else 0
    for t, dt in ((starts, torch.int32), (active, torch.uint8)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and t.numel() == B * g.T):
            raise ValueError("candidate arrays must be contiguous CUDA tensors [B][T]: int32 starts, uint8 active")
    if out is None:
        out = torch.empty((B, DECODE_RESULT_DTYPE.itemsize), dtype=torch.uint8, device=starts.device)
    if out_seq is None and want_seq:
        out_seq = torch.empty((B, g.T), dtype=torch.int32, device=starts.device)
    code = lib().moc_decode_batch(
        g._h, B, ctypes.c_void_p(starts.data_ptr()), ctypes.c_void_p(active.data_ptr()),
        ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(out_seq.data_ptr()) if out_seq is not None else None,
        _stream_handle(stream))
    _check(code, "moc_decode_batch")
    return out, out_seq


def results_to_numpy(out, dtype=RESULT_DTYPE):
    """Copy a record tensor to the host (synchronises) and view it as a structured array."""
    host = out.cpu().numpy()
    return host.reshape(-1).view(dtype).reshape(host.shape[:-1])
