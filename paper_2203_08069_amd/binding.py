"""Thin ctypes binding over ``libdistal.so`` (declared in ``include/distal.h``).

Argument marshalling only: every arithmetic step runs in the HIP kernels of the
library.  torch is used for device memory and streams.  There is no fallback:
if the shared library is missing or an argument is not a contiguous device
tensor of the right dtype, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistal.so")

F32, F64 = 0, 1
OK = 0
STATUS_NAMES = {
    0: "DISTAL_OK", 1: "DISTAL_ERR_NULL", 2: "DISTAL_ERR_SHAPE", 3: "DISTAL_ERR_DTYPE",
    4: "DISTAL_ERR_STRIDE", 5: "DISTAL_ERR_ALIAS", 6: "DISTAL_ERR_WORKSPACE", 7: "DISTAL_ERR_LAUNCH",
    8: "DISTAL_ERR_MODE",
}

# every symbol include/distal.h declares
EXPORTS = (
    "distal_gemm", "distal_ttm", "distal_mttkrp", "distal_ttv", "distal_innerprod",
    "distal_ttv_mode", "distal_ttm_mode", "distal_mttkrp_mode", "distal_mttkrp_mode_workspace_bytes",
    "distal_mttkrp_workspace_bytes", "distal_innerprod_workspace_bytes", "distal_gemm_plan",
    "distal_status_string", "distal_version", "distal_innerprod_noalloc", "distal_gemm_tiled",
    "distal_gemm_ws", "distal_gemm_workspace_bytes", "distal_gemm_peeled_columns",
    "distal_ttm_slices_per_wave",
)


class DistalError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load the built library; raises if it has not been built (no CPU fallback)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(
            f"{p} is missing: build it with `python -m paper_2203_08069_amd.build` "
            "(hipcc, gfx950). There is no fallback path.")
    lib = ctypes.CDLL(p)
    i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.distal_gemm.argtypes = [ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp]
    lib.distal_gemm_tiled.argtypes = [ci, ci, ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp]
    lib.distal_gemm_tiled.restype = ci
    lib.distal_gemm_ws.argtypes = [ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp, sz, vp]
    lib.distal_gemm_ws.restype = ci
    lib.distal_gemm_workspace_bytes.argtypes = [ci, i64, i64, i64]
    lib.distal_gemm_workspace_bytes.restype = sz
    lib.distal_ttm.argtypes = [ci, i64, i64, i64, i64, vp, vp, vp, vp]
    lib.distal_ttv_mode.argtypes = [ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.distal_ttv_mode.restype = ci
    lib.distal_ttm_mode.argtypes = [ci, ci, i64, i64, i64, i64, vp, vp, vp, vp]
    lib.distal_mttkrp_mode.argtypes = [ci, ci, i64, i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.distal_mttkrp_mode_workspace_bytes.argtypes = [ci, ci, i64, i64, i64, i64]
    lib.distal_mttkrp_mode_workspace_bytes.restype = sz
    lib.distal_mttkrp.argtypes = [ci, i64, i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.distal_ttv.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp]
    lib.distal_innerprod.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp, sz, vp]
    lib.distal_innerprod_noalloc.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp]
    lib.distal_innerprod_noalloc.restype = ci
    lib.distal_mttkrp_workspace_bytes.argtypes = [ci, i64, i64, i64, i64]
    lib.distal_innerprod_workspace_bytes.argtypes = [ci, i64, i64, i64]
    lib.distal_status_string.argtypes = [ci]
    lib.distal_version.argtypes = []
    ip = ctypes.POINTER(ctypes.c_int)
    lib.distal_gemm_plan.argtypes = [ci, ci, i64, i64, i64, i64, ci, ip, ip, ctypes.POINTER(ctypes.c_int64), ip]
    lib.distal_gemm_plan.restype = ci
    lib.distal_ttm_slices_per_wave.argtypes = [ci, i64, i64, i64]
    lib.distal_ttm_slices_per_wave.restype = ci
    lib.distal_gemm_peeled_columns.argtypes = [ci, ci, i64, i64, i64, i64, ci]
    lib.distal_gemm_peeled_columns.restype = i64
    for name in ("distal_gemm", "distal_ttm", "distal_mttkrp", "distal_ttv", "distal_innerprod",
                 "distal_ttm_mode", "distal_mttkrp_mode", "distal_version"):
        getattr(lib, name).restype = ci
    lib.distal_mttkrp_workspace_bytes.restype = sz
    lib.distal_innerprod_workspace_bytes.restype = sz
    lib.distal_status_string.restype = ctypes.c_char_p
    if path is None:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().distal_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().distal_version())


# ------------------------------------------------------------------ helpers

def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float64:
        return F64
    raise TypeError(f"unsupported dtype {t.dtype}; use float32 or float64")


def _check(t, name: str, ndim: int):
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if t.dim() != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions")


def _dense(t, name: str, ndim: int):
    _check(t, name, ndim)
    if not t.is_contiguous():
        raise ValueError(f"{name} must be dense row-major (contiguous)")


def _same(*ts):
    dts = {t.dtype for t in ts}
    devs = {t.device for t in ts}
    if len(dts) != 1 or len(devs) != 1:
        raise TypeError("all operands must share one dtype and one device")
    return _dtype_code(ts[0])


def _row_stride(t, name: str) -> int:
    """Leading dimension (elements) of a 2-D view with unit column stride.  Rows must not
    overlap: a row stride smaller than the row length (an expanded or overlapping view) is
    refused here, since the kernels would read or write past the buffer behind such a view."""
    if t.dim() != 2:
        raise ValueError(f"{name} must have 2 dimensions")
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise ValueError(f"{name}: columns must be contiguous")
    if t.shape[0] > 1:
        ld = int(t.stride(0))
        if ld < int(t.shape[1]):
            raise ValueError(f"{name}: row stride {ld} is smaller than the row length {int(t.shape[1])}")
        return ld
    return max(int(t.shape[1]), 1)


def _ld(t, name: str) -> int:
    _check(t, name, 2)
    return _row_stride(t, name)


def _stream(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(_torch().cuda.current_stream(t.device).cuda_stream)


def _ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(t.data_ptr())


def _raise(rc: int, where: str):
    if rc != OK:
        raise DistalError(rc, where)


_workspaces = {}


def _workspace(device, nbytes: int):
    """Scratch tensor of the current stream of `device`, grown on demand (torch memory; the
    library allocates nothing).  One per (device, stream): calls issued on different streams
    never share partial sums, and a tensor that is outgrown is only dropped after it has been
    marked as in use on its stream, so the caching allocator does not hand its block to another
    stream while kernels may still read it.  Callers who manage streams themselves can pass
    their own workspace instead."""
    torch = _torch()
    nbytes = max(int(nbytes), 256)
    stream = torch.cuda.current_stream(device)
    key = (device, stream.cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            ws.record_stream(stream)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


# ------------------------------------------------------------------ the five calls

def gemm_workspace_bytes(dtype_code: int, M: int, N: int, K: int) -> int:
    """Bytes of scratch distal_gemm_ws needs for these extents (0: the product is not cut along k)."""
    return int(load_library().distal_gemm_workspace_bytes(dtype_code, M, N, K))


def distal_gemm_ws(A, B, C, accumulate: bool = False, workspace=None):
    """distal_gemm with scratch memory: a small output with a long contracted index is cut along k
    (see gemm_workspace_bytes); without a `workspace` the binding's scratch of the current stream is used."""
    dt = _same(A, B, C)
    lda, ldb, ldc = _ld(A, "A"), _ld(B, "B"), _ld(C, "C")
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not match C(M,N) = A(M,K) B(K,N)")
    need = gemm_workspace_bytes(dt, M, N, K)
    ws = workspace if workspace is not None else _workspace(A.device, need)
    with _torch().cuda.device(A.device):
        rc = load_library().distal_gemm_ws(dt, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                                           int(bool(accumulate)), _ptr(ws), ws.numel() * ws.element_size(), _stream(A))
    _raise(rc, "distal_gemm_ws")
    return C


def distal_gemm(A, B, C, accumulate: bool = False):
    """C(i,j) = [C(i,j) +] sum_k A(i,k) B(k,j); operands may be row-strided 2-D views."""
    dt = _same(A, B, C)
    lda, ldb, ldc = _ld(A, "A"), _ld(B, "B"), _ld(C, "C")
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not match C(M,N) = A(M,K) B(K,N)")
    with _torch().cuda.device(A.device):
        rc = load_library().distal_gemm(dt, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                                        int(bool(accumulate)), _stream(A))
    _raise(rc, "distal_gemm")
    return C


def distal_gemm_tiled(tile, A, B, C, accumulate: bool = False, transposed_left: bool = False):
    """distal_gemm run on tiles of ``tile = (BM, BN)``; with ``transposed_left`` A is stored K x M."""
    dt = _same(A, B, C)
    lda, ldb, ldc = _ld(A, "A"), _ld(B, "B"), _ld(C, "C")
    (K, M) = A.shape if transposed_left else A.shape[::-1]
    K2, N = B.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not match C(M,N) = A(M,K) B(K,N)")
    with _torch().cuda.device(A.device):
        rc = load_library().distal_gemm_tiled(dt, int(bool(transposed_left)), int(tile[0]), int(tile[1]), M, N, K,
                                              _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                                              int(bool(accumulate)), _stream(A))
    _raise(rc, "distal_gemm_tiled")
    return C


def distal_ttm(B, C, A):
    """A(i,j,l) = sum_k B(i,j,k) C(k,l)."""
    dt = _same(B, C, A)
    _dense(B, "B", 3), _dense(C, "C", 2), _dense(A, "A", 3)
    I, J, K = B.shape
    K2, L = C.shape
    if K != K2 or tuple(A.shape) != (I, J, L):
        raise ValueError("shapes do not match A(I,J,L) = B(I,J,K) C(K,L)")
    with _torch().cuda.device(B.device):
        rc = load_library().distal_ttm(dt, I, J, K, L, _ptr(B), _ptr(C), _ptr(A), _stream(B))
    _raise(rc, "distal_ttm")
    return A


def distal_ttm_mode(mode, B, C, A):
    """Tensor times matrix along `mode` of B: A is B with that mode's extent replaced by C's columns."""
    dt = _same(B, C, A)
    _dense(B, "B", 3), _dense(C, "C", 2), _dense(A, "A", 3)
    I, J, K = B.shape
    if mode not in (0, 1, 2):
        raise ValueError("mode must be 0, 1 or 2")
    R = C.shape[1]
    want = [I, J, K]
    want[mode] = R
    if C.shape[0] != B.shape[mode] or list(A.shape) != want:
        raise ValueError("shapes do not match a mode-%d tensor-times-matrix product" % mode)
    with _torch().cuda.device(B.device):
        rc = load_library().distal_ttm_mode(dt, mode, I, J, K, R, _ptr(B), _ptr(C), _ptr(A), _stream(B))
    _raise(rc, "distal_ttm_mode")
    return A


def mttkrp_workspace_bytes(dtype_code: int, I: int, J: int, K: int, L: int) -> int:
    return int(load_library().distal_mttkrp_workspace_bytes(dtype_code, I, J, K, L))


def distal_mttkrp(B, C, D, A, workspace=None):
    """A(i,l) = sum_jk B(i,j,k) C(j,l) D(k,l)."""
    dt = _same(B, C, D, A)
    _dense(B, "B", 3), _dense(C, "C", 2), _dense(D, "D", 2), _dense(A, "A", 2)
    I, J, K = B.shape
    L = C.shape[1]
    if C.shape[0] != J or tuple(D.shape) != (K, L) or tuple(A.shape) != (I, L):
        raise ValueError("shapes do not match A(I,L) = B(I,J,K) C(J,L) D(K,L)")
    need = mttkrp_workspace_bytes(dt, I, J, K, L)
    ws = workspace if workspace is not None else _workspace(B.device, need)
    with _torch().cuda.device(B.device):
        rc = load_library().distal_mttkrp(dt, I, J, K, L, _ptr(B), _ptr(C), _ptr(D), _ptr(A),
                                          _ptr(ws), ws.numel() * ws.element_size(), _stream(B))
    _raise(rc, "distal_mttkrp")
    return A


def mttkrp_mode_workspace_bytes(dtype_code: int, mode: int, I: int, J: int, K: int, L: int) -> int:
    return int(load_library().distal_mttkrp_mode_workspace_bytes(dtype_code, mode, I, J, K, L))


def distal_mttkrp_mode(mode, B, C, D, A, workspace=None):
    """MTTKRP along `mode` of B; C and D are the factors of the two other modes, in mode order."""
    dt = _same(B, C, D, A)
    _dense(B, "B", 3), _dense(C, "C", 2), _dense(D, "D", 2), _dense(A, "A", 2)
    if mode not in (0, 1, 2):
        raise ValueError("mode must be 0, 1 or 2")
    I, J, K = B.shape
    L = C.shape[1]
    a, b = [m for m in (0, 1, 2) if m != mode]
    if (tuple(C.shape) != (B.shape[a], L) or tuple(D.shape) != (B.shape[b], L)
            or tuple(A.shape) != (B.shape[mode], L)):
        raise ValueError("shapes do not match a mode-%d MTTKRP" % mode)
    need = mttkrp_mode_workspace_bytes(dt, mode, I, J, K, L)
    ws = workspace if workspace is not None else _workspace(B.device, need)
    with _torch().cuda.device(B.device):
        rc = load_library().distal_mttkrp_mode(dt, mode, I, J, K, L, _ptr(B), _ptr(C), _ptr(D), _ptr(A),
                                               _ptr(ws), ws.numel() * ws.element_size(), _stream(B))
    _raise(rc, "distal_mttkrp_mode")
    return A


def distal_ttv(B, c, A):
    """A(i,j) = sum_k B(i,j,k) c(k)."""
    dt = _same(B, c, A)
    _dense(B, "B", 3), _dense(c, "c", 1), _dense(A, "A", 2)
    I, J, K = B.shape
    if c.shape[0] != K or tuple(A.shape) != (I, J):
        raise ValueError("shapes do not match A(I,J) = B(I,J,K) c(K)")
    with _torch().cuda.device(B.device):
        rc = load_library().distal_ttv(dt, I, J, K, _ptr(B), _ptr(c), _ptr(A), _stream(B))
    _raise(rc, "distal_ttv")
    return A


def distal_ttv_mode(mode, B, c, A):
    """Tensor times vector along `mode` of B: A keeps the two other modes, in order."""
    dt = _same(B, c, A)
    _dense(B, "B", 3), _dense(c, "c", 1), _dense(A, "A", 2)
    if mode not in (0, 1, 2):
        raise ValueError("mode must be 0, 1 or 2")
    I, J, K = B.shape
    keep = [n for m, n in enumerate(B.shape) if m != mode]
    if c.shape[0] != B.shape[mode] or list(A.shape) != keep:
        raise ValueError("shapes do not match a mode-%d tensor-times-vector product" % mode)
    with _torch().cuda.device(B.device):
        rc = load_library().distal_ttv_mode(dt, mode, I, J, K, _ptr(B), _ptr(c), _ptr(A), _stream(B))
    _raise(rc, "distal_ttv_mode")
    return A


def gemm_plan(dtype_code: int, transposed_left: bool, M: int, N: int, K: int, batch: int = 1, accumulate: bool = False):
    """How the library runs an aligned M x N x K product (host-only query):
    ((BM, BN, BK), split, cut, (BM, BN, BK) of the second launch); split 0 = one launch,
    1 = rows [0, cut) then [cut, M), 2 = columns [0, cut) then [cut, N)."""
    tile, rest = (ctypes.c_int * 3)(), (ctypes.c_int * 3)()
    split, cut = ctypes.c_int(), ctypes.c_int64()
    rc = load_library().distal_gemm_plan(dtype_code, int(bool(transposed_left)), M, N, K, batch, int(bool(accumulate)),
                                         tile, ctypes.byref(split), ctypes.byref(cut), rest)
    _raise(rc, "distal_gemm_plan")
    return tuple(tile), split.value, cut.value, tuple(rest)


def gemm_peeled_columns(dtype_code: int, transposed_left: bool, M: int, N: int, K: int, batch: int = 1,
                        accumulate: bool = False) -> int:
    """Trailing columns of the product that run in the streaming kernel instead of the tiled
    launches (host-only query); -1 for invalid arguments."""
    return int(load_library().distal_gemm_peeled_columns(dtype_code, int(bool(transposed_left)), M, N, K, batch,
                                                         int(bool(accumulate))))


def ttm_slices_per_wave(dtype_code: int, rows: int, K: int, L: int) -> int:
    """Host-only query: 1 ... 4 when distal_ttm runs a tensor of `rows` = I*J rows of K elements against
    a K x L factor in the kernel that keeps the factor in registers, 0 when it runs the tiled product."""
    return int(load_library().distal_ttm_slices_per_wave(dtype_code, rows, K, L))


def gemm_tile(dtype_code: int, transposed_left: bool, M: int, N: int, K: int, batch: int = 1, accumulate: bool = False):
    """(BM, BN, BK) of the first launch of gemm_plan()."""
    return gemm_plan(dtype_code, transposed_left, M, N, K, batch, accumulate)[0]


def innerprod_workspace_bytes(dtype_code: int, I: int, J: int, K: int) -> int:
    return int(load_library().distal_innerprod_workspace_bytes(dtype_code, I, J, K))


def distal_innerprod(B, C, a, workspace=None):
    """a = sum_ijk B(i,j,k) C(i,j,k); ``a`` is a one-element device tensor."""
    dt = _same(B, C, a)
    _dense(B, "B", 3), _dense(C, "C", 3)
    if tuple(B.shape) != tuple(C.shape) or a.numel() != 1 or not a.is_cuda:
        raise ValueError("B and C must have equal shapes and a must hold one element on the device")
    I, J, K = B.shape
    need = innerprod_workspace_bytes(dt, I, J, K)
    ws = workspace if workspace is not None else _workspace(B.device, need)
    with _torch().cuda.device(B.device):
        rc = load_library().distal_innerprod(dt, I, J, K, _ptr(B), _ptr(C), _ptr(a), _ptr(ws),
                                             ws.numel() * ws.element_size(), _stream(B))
    _raise(rc, "distal_innerprod")
    return a


def distal_innerprod_noalloc(B, C, a):
    """distal_innerprod on the library's own scratch array: no workspace, nothing allocated."""
    dt = _same(B, C, a)
    _dense(B, "B", 3), _dense(C, "C", 3)
    if tuple(B.shape) != tuple(C.shape) or a.numel() != 1 or not a.is_cuda:
        raise ValueError("B and C must have equal shapes and a must hold one element on the device")
    I, J, K = B.shape
    with _torch().cuda.device(B.device):
        rc = load_library().distal_innerprod_noalloc(dt, I, J, K, _ptr(B), _ptr(C), _ptr(a), _stream(B))
    _raise(rc, "distal_innerprod_noalloc")
    return a
