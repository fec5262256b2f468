"""Host-side checks that need no GPU: the built library loads, exports every symbol that
include/moska.h declares, and rejects bad problems before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2511_06010_amd as moska
from moska_inputs import Problem, config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moska.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moska_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert declared_symbols() == sorted(moska.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(moska.LIB_PATH):
        pytest.skip("libmoska.so not built (python -m paper_2511_06010_amd.build)")
    lib = moska.load_library()
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert lib.moska_status_string(0) == b"ok"
    assert lib.moska_status_string(-3) == b"workspace too small"


def test_problem_validation_on_host():
    if not os.path.exists(moska.LIB_PATH):
        pytest.skip("libmoska.so not built")
    for i in range(5):
        assert moska.workspace_bytes(config(i)) > 0
    ok = Problem(B=4, Hq=8, Hkv=2, D=128, C=8, L=64, k=2, U=16)
    for bad, msg in ((ok.with_(k=9), "invalid"), (ok.with_(Hq=7), "invalid"), (ok.with_(B=0), "invalid"),
                     (ok.with_(scale=0.0), "invalid"), (ok.with_(D=100), "unsupported"),
                     (ok.with_(q_dtype="f32"), "unsupported"), (ok.with_(C=20000, k=2), "unsupported")):
        with pytest.raises(moska.MoskaError, match=msg):
            moska.workspace_bytes(bad)
    # null pointers are argument errors, reported before any launch
    lib = moska.load_library()
    cp = moska.problem_t(ok)
    assert lib.moska_route(ctypes.byref(cp), None, None, None, None, None, ctypes.c_size_t(0), None) == -1
    assert lib.moska_merge(ctypes.byref(cp), None, None, None, None, None) == -1
    assert lib.moska_workspace_bytes(None, None) == -1


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2511_06010_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libmoska.so")
    with pytest.raises(moska.MoskaError, match="missing"):
        b.load_library()
