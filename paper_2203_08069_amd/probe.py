"""ctypes binding of the measurement aid ``libdistal_probe.so`` (include/distal_probe.h).

Used by bench.py only: a synthetic stream + MFMA kernel timed next to the MTTKRP kernel.
Nothing of the library's product path goes through here.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistal_probe.so")
EXPORTS = ("distal_probe_stream_mfma", "distal_probe_out_bytes", "distal_probe_mfma_peak",
           "distal_probe_mfma_peak_out_bytes", "distal_probe_mfma_peak_flops", "distal_probe_hbm_read",
           "distal_probe_hbm_read_out_bytes")

_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2203_08069_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.distal_probe_stream_mfma.argtypes = [i64, i64, i64, vp, vp, ctypes.c_int, vp, ctypes.c_size_t, vp]
        lib.distal_probe_stream_mfma.restype = ctypes.c_int
        lib.distal_probe_out_bytes.argtypes = [i64, i64, i64]
        lib.distal_probe_out_bytes.restype = ctypes.c_size_t
        lib.distal_probe_mfma_peak.argtypes = [ctypes.c_int, i64, vp, ctypes.c_size_t, vp]
        lib.distal_probe_mfma_peak.restype = ctypes.c_int
        lib.distal_probe_mfma_peak_out_bytes.argtypes = [ctypes.c_int]
        lib.distal_probe_mfma_peak_out_bytes.restype = ctypes.c_size_t
        lib.distal_probe_mfma_peak_flops.argtypes = [ctypes.c_int, i64]
        lib.distal_probe_mfma_peak_flops.restype = ctypes.c_double
        lib.distal_probe_hbm_read.argtypes = [vp, i64, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp]
        lib.distal_probe_hbm_read.restype = ctypes.c_int
        lib.distal_probe_hbm_read_out_bytes.argtypes = [ctypes.c_int]
        lib.distal_probe_hbm_read_out_bytes.restype = ctypes.c_size_t
        _lib = lib
    return _lib


def out_bytes(I: int, J: int, K: int) -> int:
    return int(load_library().distal_probe_out_bytes(I, J, K))


def stream_mfma(B, F, out, lds: bool):
    """One launch of the probe on the float32 device tensor B (I x J x K) on torch's current stream."""
    import torch
    assert B.is_cuda and B.is_contiguous() and B.dtype == torch.float32 and B.dim() == 3
    assert F.is_cuda and F.is_contiguous() and F.dtype == torch.float32 and F.numel() >= 1024
    assert out.is_cuda and out.is_contiguous()
    I, J, K = B.shape
    rc = load_library().distal_probe_stream_mfma(
        I, J, K, ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(F.data_ptr()), int(bool(lds)),
        ctypes.c_void_p(out.data_ptr()), out.numel() * out.element_size(),
        ctypes.c_void_p(torch.cuda.current_stream(B.device).cuda_stream))
    if rc != 0:
        raise RuntimeError(f"distal_probe_stream_mfma failed with status {rc}")


def mfma_peak_out_bytes(f64: bool) -> int:
    return int(load_library().distal_probe_mfma_peak_out_bytes(int(bool(f64))))


def mfma_peak_flops(f64: bool, iters: int) -> float:
    return float(load_library().distal_probe_mfma_peak_flops(int(bool(f64)), int(iters)))


def mfma_peak(f64: bool, iters: int, out):
    """One launch of the register-only matrix-instruction loop on torch's current stream."""
    import torch
    assert out.is_cuda and out.is_contiguous()
    rc = load_library().distal_probe_mfma_peak(
        int(bool(f64)), int(iters), ctypes.c_void_p(out.data_ptr()), out.numel() * out.element_size(),
        ctypes.c_void_p(torch.cuda.current_stream(out.device).cuda_stream))
    if rc != 0:
        raise RuntimeError(f"distal_probe_mfma_peak failed with status {rc}")


def hbm_read_out_bytes(blocks: int) -> int:
    return int(load_library().distal_probe_hbm_read_out_bytes(int(blocks)))


def hbm_read(src, blocks: int, in_flight: int, out):
    """One launch of the read-only stream over the whole device tensor `src` on torch's current stream."""
    import torch
    assert src.is_cuda and src.is_contiguous() and out.is_cuda and out.is_contiguous()
    rc = load_library().distal_probe_hbm_read(
        ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(), int(blocks), int(in_flight),
        ctypes.c_void_p(out.data_ptr()), out.numel() * out.element_size(),
        ctypes.c_void_p(torch.cuda.current_stream(src.device).cuda_stream))
    if rc != 0:
        raise RuntimeError(f"distal_probe_hbm_read failed with status {rc}")
