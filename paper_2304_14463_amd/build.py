"""Builds the HIP shared libraries in-tree with hipcc for gfx950.

  paper_2304_14463_amd/libmoccasin_hip.so          the C-ABI evaluator (include/moccasin.h)
  paper_2304_14463_amd/inputs/libmoc_inputs_hip.so device twin of the candidate generator

hipcc cross-compiles without a GPU.  Run as `python -m paper_2304_14463_amd.build`.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libmoccasin_hip.so")
INPUTS_LIB = os.path.join(PKG, "inputs", "libmoc_inputs_hip.so")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               # a one-lane atomic is to stay one instruction whose result is waited for where it
               # is used: the evaluator draws its next candidate index that way, far ahead
               "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
               "-Wall", "-Wno-unused-result"]
# Per source file.  The evaluation kernels are scheduled for instruction-level parallelism
# rather than for occupancy (their workgroup sizes fix the waves per SIMD anyway): n = 5000,
# C = 3 gains 1.7 points of HBM peak (64.4 -> 66.1 %; repeated on four machines), the other
# evaluation workloads stay within what two runs differ by.  In the neighbourhood file the
# toggles kernel gains 3 % and the cuts kernel under 1 % (both repeated), the neighbourhood
# kernel itself does not move.  Decode and the staged evaluator stay within 1 % either way
# and keep the default.
FILE_FLAGS = {"moc_eval.hip": ["-mllvm", "-amdgpu-sched-strategy=max-ilp"],
              "moc_neighbours.hip": ["-mllvm", "-amdgpu-sched-strategy=max-ilp"]}


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({' '.join(cmd)}):\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")


def _hipcc(out, sources, extra=()):
    """One object file per source, compiled side by side, then linked."""
    from concurrent.futures import ThreadPoolExecutor
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory() as tmp:
        objs = [os.path.join(tmp, os.path.basename(s) + ".o") for s in sources]
        with ThreadPoolExecutor(min(len(sources), os.cpu_count() or 1, 16)) as ex:
            list(ex.map(lambda so: _run(["hipcc", *flags, *FILE_FLAGS.get(os.path.basename(so[0]), []), *extra,
                                         "-c", "-o", so[1], so[0]]), zip(sources, objs)))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs])
    return out


def build_library():
    srcs = sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))
    return _hipcc(LIB, srcs, ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc")])


def build_inputs():
    srcs = sorted(glob.glob(os.path.join(PKG, "inputs", "csrc", "*.hip")))
    return _hipcc(INPUTS_LIB, srcs)


def build_all():
    return [build_library(), build_inputs()]


if __name__ == "__main__":
    for path in build_all():
        print("built", path)
