"""Python access to the CPU oracle (``distal_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.

Every function takes numpy arrays of one dtype (float32 or float64), passes
them unchanged to the C routine and returns the oracle's binary64 result.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "distal_oracle.c")
_LIB = os.path.join(_HERE, "libdistal_oracle.so")
_lock = threading.Lock()
_lib = None

F32, F64 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-ffp-contract=off", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path: str):
    """ctypes prototypes for an oracle shared object."""
    lib = ctypes.CDLL(path)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.oracle_gemm.argtypes = [ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp]
    lib.oracle_ttv.argtypes = [ci, i64, i64, i64, vp, vp, vp]
    lib.oracle_innerprod.argtypes = [ci, i64, i64, i64, vp, vp, vp]
    lib.oracle_ttm.argtypes = [ci, i64, i64, i64, i64, vp, vp, vp]
    lib.oracle_mttkrp.argtypes = [ci, i64, i64, i64, i64, vp, vp, vp, vp]
    lib.oracle_ttv_mode.argtypes = [ci, ci, i64, i64, i64, vp, vp, vp]
    lib.oracle_ttv_mode.restype = ci
    lib.oracle_ttm_mode.argtypes = [ci, ci, i64, i64, i64, i64, vp, vp, vp]
    lib.oracle_mttkrp_mode.argtypes = [ci, ci, i64, i64, i64, i64, vp, vp, vp, vp]
    for f in (lib.oracle_ttm_mode, lib.oracle_mttkrp_mode, lib.oracle_gemm, lib.oracle_ttv, lib.oracle_innerprod, lib.oracle_ttm,
              lib.oracle_mttkrp, lib.oracle_version, lib.oracle_long_double_digits,
              lib.oracle_max_threads):
        f.restype = ci
    if lib.oracle_long_double_digits() < 64:
        raise RuntimeError("oracle needs a long double with a 64-bit significand")
    return lib


def _load():
    global _lib
    with _lock:
        if _lib is None:
            _lib = _bind(build())
    return _lib


class Variant:
    """The same Python front end over another build of the C source.  Tests use it to plant a
    mistake in a COPY of the oracle and check that the pins notice; nothing else may."""

    def __init__(self, lib_path: str):
        self._lib = _bind(lib_path)

    def _call(self, name, *a, **k):
        global _lib
        with _lock:
            saved, _lib = _lib, self._lib
        try:
            return globals()[name](*a, **k)
        finally:
            with _lock:
                _lib = saved

    def gemm(self, *a, **k): return self._call("gemm", *a, **k)
    def ttv(self, *a, **k): return self._call("ttv", *a, **k)
    def innerprod(self, *a, **k): return self._call("innerprod", *a, **k)
    def ttm(self, *a, **k): return self._call("ttm", *a, **k)
    def mttkrp(self, *a, **k): return self._call("mttkrp", *a, **k)
    def ttv_mode(self, *a, **k): return self._call("ttv_mode", *a, **k)
    def ttm_mode(self, *a, **k): return self._call("ttm_mode", *a, **k)
    def mttkrp_mode(self, *a, **k): return self._call("mttkrp_mode", *a, **k)


def max_threads() -> int:
    """OpenMP threads the oracle's loops use on this host."""
    return int(_load().oracle_max_threads())


def _dt(*arrays) -> int:
    dts = {a.dtype for a in arrays}
    if len(dts) != 1:
        raise TypeError("all operands must share one dtype")
    d = dts.pop()
    if d == np.float32:
        return F32
    if d == np.float64:
        return F64
    raise TypeError("operands must be float32 or float64")


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _rows(a: np.ndarray, name: str) -> int:
    """Leading dimension (elements) of a 2-D array whose rows are contiguous."""
    if a.ndim != 2:
        raise ValueError(f"{name} must be 2-D")
    if a.size == 0:
        return max(a.shape[1], 1)
    if a.shape[1] > 1 and a.strides[1] != a.itemsize:
        raise ValueError(f"{name}: rows must be contiguous")
    if a.shape[0] > 1:
        if a.strides[0] % a.itemsize or a.strides[0] < a.shape[1] * a.itemsize:
            raise ValueError(f"{name}: bad row stride")
        return a.strides[0] // a.itemsize
    return max(a.shape[1], 1)


def _check(rc: int):
    if rc != 0:
        raise ValueError("oracle rejected its arguments")


def gemm(A: np.ndarray, B: np.ndarray, init: np.ndarray | None = None) -> np.ndarray:
    """out = [init +] A @ B by the definition.  Row-strided 2-D views are accepted."""
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise ValueError("inner extents differ")
    ops = (A, B) if init is None else (A, B, init)
    dt = _dt(*ops)
    out = np.empty((M, N), dtype=np.float64)
    lda, ldb = max(_rows(A, "A"), K), max(_rows(B, "B"), N)
    if init is None:
        rc = _load().oracle_gemm(dt, M, N, K, _p(A), lda, _p(B), ldb, None, 0, 0, _p(out))
    else:
        if init.shape != (M, N):
            raise ValueError("init has the wrong shape")
        rc = _load().oracle_gemm(dt, M, N, K, _p(A), lda, _p(B), ldb, _p(init),
                                 max(_rows(init, "init"), N), 1, _p(out))
    _check(rc)
    return out


def ttv(B: np.ndarray, c: np.ndarray) -> np.ndarray:
    I, J, K = B.shape
    if c.shape != (K,):
        raise ValueError("c has the wrong shape")
    B, c = np.ascontiguousarray(B), np.ascontiguousarray(c)
    out = np.empty((I, J), dtype=np.float64)
    _check(_load().oracle_ttv(_dt(B, c), I, J, K, _p(B), _p(c), _p(out)))
    return out


def innerprod(B: np.ndarray, C: np.ndarray) -> float:
    if B.shape != C.shape or B.ndim != 3:
        raise ValueError("B and C must be 3-D of equal shape")
    B, C = np.ascontiguousarray(B), np.ascontiguousarray(C)
    I, J, K = B.shape
    out = np.empty(1, dtype=np.float64)
    _check(_load().oracle_innerprod(_dt(B, C), I, J, K, _p(B), _p(C), _p(out)))
    return float(out[0])


def ttm(B: np.ndarray, C: np.ndarray) -> np.ndarray:
    I, J, K = B.shape
    K2, L = C.shape
    if K != K2:
        raise ValueError("inner extents differ")
    B, C = np.ascontiguousarray(B), np.ascontiguousarray(C)
    out = np.empty((I, J, L), dtype=np.float64)
    _check(_load().oracle_ttm(_dt(B, C), I, J, K, L, _p(B), _p(C), _p(out)))
    return out


def mttkrp(B: np.ndarray, C: np.ndarray, D: np.ndarray) -> np.ndarray:
    I, J, K = B.shape
    if C.ndim != 2 or D.ndim != 2 or C.shape[0] != J or D.shape[0] != K or C.shape[1] != D.shape[1]:
        raise ValueError("factor shapes do not match B")
    L = C.shape[1]
    B, C, D = (np.ascontiguousarray(x) for x in (B, C, D))
    out = np.empty((I, L), dtype=np.float64)
    _check(_load().oracle_mttkrp(_dt(B, C, D), I, J, K, L, _p(B), _p(C), _p(D), _p(out)))
    return out


def ttm_mode(mode: int, B: np.ndarray, C: np.ndarray) -> np.ndarray:
    """Tensor times matrix along `mode` of B: that mode's extent is replaced by C's columns."""
    if B.ndim != 3 or C.ndim != 2 or mode not in (0, 1, 2) or C.shape[0] != B.shape[mode]:
        raise ValueError("C must have one row per index of the contracted mode")
    I, J, K = B.shape
    R = C.shape[1]
    B, C = np.ascontiguousarray(B), np.ascontiguousarray(C)
    shape = [I, J, K]
    shape[mode] = R
    out = np.empty(shape, dtype=np.float64)
    _check(_load().oracle_ttm_mode(_dt(B, C), mode, I, J, K, R, _p(B), _p(C), _p(out)))
    return out


def mttkrp_mode(mode: int, B: np.ndarray, C: np.ndarray, D: np.ndarray) -> np.ndarray:
    """MTTKRP along `mode` of B; C and D are the factors of the other two modes, in mode order."""
    if B.ndim != 3 or C.ndim != 2 or D.ndim != 2 or mode not in (0, 1, 2):
        raise ValueError("bad operands")
    others = [m for m in (0, 1, 2) if m != mode]
    if C.shape[0] != B.shape[others[0]] or D.shape[0] != B.shape[others[1]] or C.shape[1] != D.shape[1]:
        raise ValueError("factor shapes do not match B")
    I, J, K = B.shape
    L = C.shape[1]
    B, C, D = (np.ascontiguousarray(x) for x in (B, C, D))
    out = np.empty((B.shape[mode], L), dtype=np.float64)
    _check(_load().oracle_mttkrp_mode(_dt(B, C, D), mode, I, J, K, L, _p(B), _p(C), _p(D), _p(out)))
    return out


def ttv_mode(mode: int, B: np.ndarray, c: np.ndarray) -> np.ndarray:
    """Tensor times vector along `mode` of B: that mode disappears from the output."""
    if B.ndim != 3 or c.ndim != 1 or mode not in (0, 1, 2) or c.shape[0] != B.shape[mode]:
        raise ValueError("c must have one entry per index of the contracted mode")
    I, J, K = B.shape
    B, c = np.ascontiguousarray(B), np.ascontiguousarray(c)
    out = np.empty([n for m, n in enumerate(B.shape) if m != mode], dtype=np.float64)
    _check(_load().oracle_ttv_mode(_dt(B, c), mode, I, J, K, _p(B), _p(c), _p(out)))
    return out
