"""The built C-ABI library loads on a machine without a GPU and exports every
symbol that include/moccasin.h declares (no compute calls here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moccasin.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moc_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    from paper_2304_14463_amd import moccasin
    assert declared_functions() == sorted(moccasin.EXPORTS)


def test_library_exports_every_declared_symbol():
    from paper_2304_14463_amd import moccasin
    assert os.path.exists(moccasin.LIB_PATH), "build first: python -m paper_2304_14463_amd.build"
    lib = ctypes.CDLL(moccasin.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), name
    # calls that touch no device
    lib.moc_strerror.restype = ctypes.c_char_p
    assert lib.moc_strerror(0) == b"ok" and b"invalid" in lib.moc_strerror(-1)
    assert lib.moc_last_hip_error() == 0
    lib.moc_graph_free(None)
    assert lib.moc_graph_info(None, None, None, None, None) == -1
    assert lib.moc_eval_batch(None, 0, None, None, None, None, None) == -1
    assert lib.moc_eval_toggles(None, 0, None, None, None, None, None) == -1
    assert lib.moc_decode_batch(None, 0, None, None, None, None, None) == -1
    assert lib.moc_eval_cuts(None, 0, None, None, None, None, None, None) == -1
    assert lib.moc_search_cuts(None, 0, None, None, None, 1, None, None, None) == -1
    assert lib.moc_search_moves(None, 0, None, None, None, 1, 1, None, None, None, None) == -1
    out = ctypes.c_void_p(1)
    assert lib.moc_graph_upload(0, None, None, None, None, 0, 1, ctypes.byref(out)) == -1 and not out.value


def test_result_struct_layout():
    from paper_2304_14463_amd import moccasin
    assert moccasin.RESULT_DTYPE.itemsize == 24 and moccasin.MOVE_SCORE_DTYPE.itemsize == 8
    assert moccasin.BEST_MOVE_DTYPE.itemsize == 16 and moccasin.TOGGLE_SCORE_DTYPE.itemsize == 16
    assert moccasin.DECODE_RESULT_DTYPE.itemsize == 24


def test_device_generator_library_loads():
    from paper_2304_14463_amd.inputs import device
    assert os.path.exists(device.LIB_PATH)
    assert hasattr(ctypes.CDLL(device.LIB_PATH), "mocgen_candidates")
