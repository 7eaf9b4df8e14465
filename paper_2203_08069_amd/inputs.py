"""Seeded synthetic input tensors for the leaf kernels and for their CPU checker.

This module only produces input values.  It holds none of the arithmetic of the
tensor expressions themselves, so both the GPU path and the independent CPU
checker may be fed from it without sharing any part of the method.

Element ``n`` (row-major linear index) of tensor number ``ordinal`` under seed
``seed`` is a pure function ``g(seed, ordinal, n)``: generation is independent
of order, chunking and thread count, and any slice of a 4 GiB tensor can be
regenerated on its own (which is how full-size results are spot-checked).

The paper evaluates on synthetic dense row-major tensors whose contents it does
not state (evaluation section, higher-order kernels); uniform values in [-1, 1)
and small signed integers are this build's stand-ins.

Bit mixer: the 64-bit finaliser of SplitMix64 (Steele, Lea, Flood, "Fast
splittable pseudorandom number generators", OOPSLA 2014), applied to a
Weyl sequence offset by a per-(seed, ordinal) key.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Iterator, Sequence, Tuple

import numpy as np

_MASK = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

UNIFORM = "uniform"      # iid uniform on [-1, 1), 53 random bits, then rounded to dtype
SMALLINT = "smallint"    # iid integers in {-r..r}


def _mix_scalar(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, ordinal: int) -> int:
    """64-bit key of the value stream of tensor ``ordinal`` under ``seed``."""
    if seed < 0 or ordinal < 0:
        raise ValueError("seed and ordinal must be non-negative")
    return _mix_scalar(_mix_scalar(seed + 1) ^ ((_GAMMA * (ordinal + 1)) & _MASK))


def raw_bits(seed: int, ordinal: int, start: int, count: int) -> np.ndarray:
    """uint64 random words for linear indices start .. start+count-1."""
    if start < 0 or count < 0:
        raise ValueError("start and count must be non-negative")
    key = np.uint64(stream_key(seed, ordinal))
    with np.errstate(over="ignore"):
        z = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z *= np.uint64(_GAMMA)
        z += key
        z ^= z >> np.uint64(30)
        z *= np.uint64(_M1)
        z ^= z >> np.uint64(27)
        z *= np.uint64(_M2)
        z ^= z >> np.uint64(31)
    return z


def values(seed: int, ordinal: int, start: int, count: int, dtype,
           kind: str = UNIFORM, r: int = 3) -> np.ndarray:
    """Flat slice [start, start+count) of a tensor's values, as ``dtype``."""
    dtype = np.dtype(dtype)
    if dtype not in (np.dtype(np.float32), np.dtype(np.float64)):
        raise ValueError("dtype must be float32 or float64")
    bits = raw_bits(seed, ordinal, start, count)
    if kind == UNIFORM:
        # u = top 53 bits * 2^-53 in [0,1); 2u-1 is exact in binary64.
        x = (bits >> np.uint64(11)).astype(np.float64)
        x *= 2.0 ** -52
        x -= 1.0
        return x.astype(dtype)
    if kind == SMALLINT:
        if r < 0:
            raise ValueError("r must be non-negative")
        m = (bits >> np.uint64(32)) % np.uint64(2 * r + 1)
        return (m.astype(np.int64) - r).astype(dtype)
    raise ValueError(f"unknown kind {kind!r}")


_BLOCK = 1 << 16   # elements generated per numpy pass (stays in cache)


def fill(out: np.ndarray, seed: int, ordinal: int, start: int = 0,
         kind: str = UNIFORM, r: int = 3, threads: int = 1) -> np.ndarray:
    """Fill the flat array ``out`` with elements start .. start+out.size-1."""
    if out.ndim != 1 or not out.flags.c_contiguous:
        raise ValueError("out must be a flat contiguous array")
    n = out.size
    offs = range(0, n, _BLOCK)

    def one(o: int) -> None:
        m = min(_BLOCK, n - o)
        out[o:o + m] = values(seed, ordinal, start + o, m, out.dtype, kind, r)

    if threads <= 1 or n <= _BLOCK:
        for o in offs:
            one(o)
    else:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(one, offs))
    return out


def tensor(seed: int, ordinal: int, shape: Sequence[int], dtype,
           kind: str = UNIFORM, r: int = 3, threads: int = 1) -> np.ndarray:
    """Whole dense row-major tensor (host memory)."""
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape, dtype=np.int64)) if shape else 1
    out = np.empty(n, dtype=np.dtype(dtype))
    fill(out, seed, ordinal, 0, kind, r, threads)
    return out.reshape(shape)


def chunks(seed: int, ordinal: int, total: int, dtype, kind: str = UNIFORM,
           r: int = 3, chunk_elems: int = 1 << 24, threads: int = 1,
           buffer: np.ndarray | None = None) -> Iterator[Tuple[int, np.ndarray]]:
    """Yield (start, values) pieces covering [0, total) in increasing order.

    A 2^30-element tensor can be streamed to the device through one staging
    buffer (``buffer``, e.g. pinned memory) without holding a host copy.  The
    yielded array is a view of that buffer and is overwritten by the next step.
    """
    if buffer is None:
        buffer = np.empty(min(chunk_elems, max(total, 1)), dtype=np.dtype(dtype))
    cap = buffer.size
    for s in range(0, total, cap):
        m = min(cap, total - s)
        yield s, fill(buffer[:m], seed, ordinal, s, kind, r, threads)


# Tensor ordinals per expression, in argument order.
ORDINALS = {
    "gemm": {"A": 0, "B": 1, "C": 2},
    "ttv": {"B": 0, "c": 1},
    "innerprod": {"B": 0, "C": 2},
    "ttm": {"B": 0, "C": 1},
    "mttkrp": {"B": 0, "C": 1, "D": 2},
}
