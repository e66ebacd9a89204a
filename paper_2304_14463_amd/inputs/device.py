"""Device side of the candidate generator: ctypes binding of
libmoc_inputs_hip.so (csrc/gen_candidates.hip) and a holder of the generator
tables in HBM.  Emits the same bits as inputs.candidates.gen_candidates."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoc_inputs_hip.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run python -m paper_2304_14463_amd.build")
        L = ctypes.CDLL(LIB_PATH)
        VP, I32, I64, U64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
        L.mocgen_candidates.argtypes = [U64, I32, I32, I64, VP, VP, VP, VP, VP, I64, I64, I32, VP, VP, VP, VP]
        L.mocgen_candidates.restype = ctypes.c_int
        L.mocgen_stream_read.argtypes = [VP, U64, VP, U64, VP, U64, I32, VP, VP]
        L.mocgen_stream_read.restype = ctypes.c_int
        _lib = L
    return _lib


class DeviceWorkload:
    """Generator tables of a Workload resident on the GPU."""

    def __init__(self, w, device="cuda:0"):
        import torch
        self.w = w
        self.device = torch.device(device)
        put = lambda a: torch.from_numpy(a.astype("int32")).to(self.device)
        self.pos, self.out_ptr, self.cons_pos = put(w.pos), put(w.out_ptr), put(w.cons_pos)
        self.win_hi, self.ncut = put(w.win_hi), put(w.ncut)
        if self.cons_pos.numel() == 0:
            self.cons_pos = torch.zeros(1, dtype=torch.int32, device=self.device)

    def candidates(self, b0=0, count=None, out=None, stream=None):
        """(starts, ends, active) CUDA tensors [count][T] for candidates b0 .. b0+count-1."""
        import torch
        w = self.w
        if count is None:
            count = w.B - b0
        if out is None:
            out = (torch.empty((count, w.T), dtype=torch.int32, device=self.device),
                   torch.empty((count, w.T), dtype=torch.int32, device=self.device),
                   torch.empty((count, w.T), dtype=torch.uint8, device=self.device))
        s, e, a = out
        if stream is None:
            stream = torch.cuda.current_stream()
        rc = lib().mocgen_candidates(w.seed & ((1 << 64) - 1), w.n, w.C, w.B, self.pos.data_ptr(),
                                     self.out_ptr.data_ptr(), self.cons_pos.data_ptr(), self.win_hi.data_ptr(),
                                     self.ncut.data_ptr(), b0, count, int(w.dense), s.data_ptr(), e.data_ptr(), a.data_ptr(),
                                     ctypes.c_void_p(stream.cuda_stream))
        if rc != 0:
            raise RuntimeError(f"mocgen_candidates: hipError {rc}")
        return s, e, a


def stream_read(tensors, blocks, out=None, stream=None):
    """Queues one launch that reads the three CUDA tensors once and does nothing else
    (csrc/stream_read.hip): what a read of these bytes costs on this GPU at the least.
    Returns the scratch tensor the kernel writes one word per thread to."""
    import torch
    x0, x1, x2 = tensors
    if out is None:
        out = torch.empty(blocks * 1024, dtype=torch.int32, device=x0.device)
    if stream is None:
        stream = torch.cuda.current_stream()
    nbytes = lambda t: t.numel() * t.element_size()
    rc = lib().mocgen_stream_read(x0.data_ptr(), nbytes(x0), x1.data_ptr(), nbytes(x1), x2.data_ptr(), nbytes(x2),
                                  int(blocks), out.data_ptr(), ctypes.c_void_p(stream.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"mocgen_stream_read: hipError {rc}")
    return out
