"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sparge.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparge_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_boundary():
    names = declared_functions()
    for need in ("sparge_quantize", "sparge_predict", "sparge_attn", "sparge_forward", "sparge_workspace_bytes",
                 "sparge_last_error"):
        assert need in names


def test_library_exports_every_declared_symbol():
    import paper_2502_18137_amd as sp
    if not os.path.exists(sp.library_path()):
        from paper_2502_18137_amd.build import build_library
        build_library(verbose=False)
    lib = ctypes.CDLL(sp.library_path())
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sp.sparge_version() >= 100


def test_argument_validation_needs_no_gpu():
    import paper_2502_18137_amd as sp
    from paper_2502_18137_amd.binding import _Desc
    lib = sp.load_library()
    n = ctypes.c_size_t(0)
    good = _Desc(1, 2, 2048, 64, 0, 2 * 2048 * 64, 2048 * 64, 64)
    assert lib.sparge_workspace_bytes(ctypes.byref(good), sp.WS_FORWARD, ctypes.byref(n)) == 0
    assert n.value > 2 * 2048 * 64 * 2           # holds at least Q-hat and K-hat
    bad_d = _Desc(1, 2, 2048, 96, 0, 2 * 2048 * 96, 2048 * 96, 96)
    assert lib.sparge_workspace_bytes(ctypes.byref(bad_d), sp.WS_FORWARD, ctypes.byref(n)) == -2
    assert b"head dim" in lib.sparge_last_error()
    bad_n = _Desc(1, 2, 0, 64, 0, 0, 0, 64)
    assert lib.sparge_workspace_bytes(ctypes.byref(bad_n), sp.WS_FORWARD, ctypes.byref(n)) == -1
    too_long = _Desc(1, 1, 64 * 4096 + 1, 64, 1, 0, 0, 64)
    assert lib.sparge_workspace_bytes(ctypes.byref(too_long), sp.WS_ATTN, ctypes.byref(n)) == -2
    # NULL tensors / bad hyper-parameters are rejected before anything is enqueued
    tau = (ctypes.c_float * 2)(0.9, 1.5)
    theta = (ctypes.c_float * 2)(0.5, 0.5)
    rc = lib.sparge_predict(None, None, ctypes.byref(good), tau, theta, 0.0, 0, None, None, None, None, 0, None)
    assert rc == -1


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2502_18137_amd.binding as b
    monkeypatch.setattr(b, "_LIB", None)
    monkeypatch.setattr(b, "library_path", lambda: "/nonexistent/libsparge.so")
    with pytest.raises(b.SpargeError):
        b.load_library()
