"""Host-side checks that need no GPU: the shared library builds/loads and exports every symbol that
include/nnrescal.h declares; argument validation that happens before any device work."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "nnrescal.h")).read()
    return sorted(set(re.findall(r"NNRESCAL_API[^;(]*?\b(nnrescal_\w+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = _declared()
    for must in ("nnrescal_init", "nnrescal_mu_step", "nnrescal_fit", "nnrescal_select_k"):
        assert must in names
    assert len(names) >= 10


def test_library_loads_and_exports_every_declared_symbol():
    import paper_2202_09512_amd as nn
    if not os.path.exists(nn.lib_path()):
        from paper_2202_09512_amd import build
        build.build(verbose=False)
    lib = nn.load()
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(nn.EXPORTED_SYMBOLS) == _declared()


def test_validation_without_device_work():
    import paper_2202_09512_amd as nn
    from paper_2202_09512_amd import binding as b
    lib = nn.load()
    out = ctypes.c_void_p()
    # NULL tensor / NULL params are rejected with a message, nothing is dereferenced
    assert lib.nnrescal_init(ctypes.byref(out), None, None) == 1
    assert b"NULL" in lib.nnrescal_last_error(None)
    t = b._Tensor(format=7, n=10, m=1)
    assert lib.nnrescal_init(ctypes.byref(out), ctypes.byref(t), None) == 1
    assert b"format" in lib.nnrescal_last_error(None)
    t = b._Tensor(format=0, n=0, m=1)
    assert lib.nnrescal_init(ctypes.byref(out), ctypes.byref(t), None) == 1
    assert lib.nnrescal_mu_step(None) == 4 and lib.nnrescal_fit(None, 1, None) == 4
    lib.nnrescal_destroy(None)
