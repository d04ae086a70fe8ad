"""Compiled twin of the perturbation (oracle/csrc/perturb_fast.c), for the full-size parity tests.

Test infrastructure only (see package docstring).  The NumPy functions of `philox.py` and `perturb.py` are the
definition; the C routines here compute the same values for inputs of billions of elements, where NumPy's
temporaries make the definition take hours.  `tests/test_oracle_fast.py` pins them: the generator to the published
known-answer vectors, the perturbed values bit for bit to `perturb.perturb_dense` / `perturb.perturb_coo`.

Build: `python -m oracle.build` (gcc -O2 -fopenmp -ffp-contract=off) writes `oracle/liboracle_fast.so`;
`load()` builds it when it is missing.
"""
import ctypes as C
import os

import numpy as np

from .perturb import _constants

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def lib_path():
    return os.path.join(_HERE, "liboracle_fast.so")


def load():
    global _LIB
    if _LIB is None:
        if not os.path.exists(lib_path()):
            from . import build
            build.build(verbose=False)
        lib = C.CDLL(lib_path())
        lib.oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_int64, C.c_uint32, C.c_uint32]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_perturb_dense_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32,
                                                  C.c_uint64, C.c_int32, C.c_float]
        lib.oracle_perturb_dense_rows.restype = None
        lib.oracle_perturb_coo.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                           C.c_int32, C.c_uint64, C.c_int32, C.c_float]
        lib.oracle_perturb_coo.restype = None
        lib.oracle_init_stream.argtypes = [C.c_void_p, C.c_int64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
        lib.oracle_init_stream.restype = None
        _LIB = lib
    return _LIB


def philox_blocks(counters, k0, k1):
    """counters: uint32 [count, 4] -> outputs uint32 [count, 4]."""
    out = np.ascontiguousarray(counters, dtype=np.uint32).copy()
    load().oracle_philox4x32_10(out.ctypes.data, out.shape[0], int(k0), int(k1))
    return out


def perturb_dense_slice(Xt, t, seed, member, delta, i0=0):
    """Rows [i0, i0 + Xt.shape[0]) of slice t of a dense tensor with Xt.shape[1] columns (fp32) -> perturbed fp32."""
    Xt = np.ascontiguousarray(Xt, dtype=np.float32)
    if delta == 0:
        return Xt.copy()
    _constants(delta)            # raises for amplitudes whose constant c the definition cannot form exactly
    out = np.empty_like(Xt)
    load().oracle_perturb_dense_rows(Xt.ctypes.data, out.ctypes.data, Xt.shape[1], int(i0), Xt.shape[0], int(t),
                                     int(seed) & 0xFFFFFFFFFFFFFFFF, int(member), float(np.float32(delta)))
    return out


def perturb_coo(rows, cols, vals, t, n, seed, member, delta):
    """Stored non-zeros of slice t in coordinate form -> perturbed fp32 values (same order)."""
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    if delta == 0:
        return vals.copy()
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    _constants(delta)
    out = np.empty_like(vals)
    load().oracle_perturb_coo(rows.ctypes.data, cols.ctypes.data, vals.ctypes.data, out.ctypes.data, vals.size, int(n),
                              int(t), int(seed) & 0xFFFFFFFFFFFFFFFF, int(member), float(np.float32(delta)))
    return out


def init_A(seed, member, n, k):
    """perturb.init_A(seed, member, n, k) for factors of 1e7 rows."""
    out = np.empty((n, k), dtype=np.float32)
    load().oracle_init_stream(out.ctypes.data, out.size, int(k), 1, int(member), int(seed) & 0xFFFFFFFFFFFFFFFF)
    return out


def init_R(seed, member, m, k):
    """perturb.init_R(seed, member, m, k)."""
    out = np.empty((m, k, k), dtype=np.float32)
    load().oracle_init_stream(out.ctypes.data, out.size, int(k), 2, int(member), int(seed) & 0xFFFFFFFFFFFFFFFF)
    return out
