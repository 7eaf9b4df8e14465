"""Place seeded synthetic tensors (see ``inputs``) in device memory.

``device_tensor`` generates the values on the host with ``inputs`` in pieces and copies them
through one pinned staging buffer, so a 4 GiB tensor never needs a host copy.
``generate_on_device`` evaluates the same counter-based generator with torch integer
operations where the tensor lives (the benchmark and the full-size tests fill several
4-8 GiB tensors; on the host that is a minute of numpy per run).  Either way the bytes on the
device are exactly those ``inputs.values`` returns for the same indices: the generator is
integer arithmetic modulo 2^64 followed by conversions that are exact up to the final
rounding to the dtype, which both sides do in round-to-nearest-even.
"""
from __future__ import annotations

import os
from typing import Sequence

import numpy as np

from . import inputs

_TORCH_DTYPES = {"float32": "float32", "float64": "float64"}


def default_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def device_tensor(seed: int, ordinal: int, shape: Sequence[int], dtype, kind: str = inputs.UNIFORM,
                  r: int = 3, device: str = "cuda:0", threads: int | None = None,
                  stage_elems: int = 1 << 24):
    import torch
    npdt = np.dtype(dtype)
    tdt = getattr(torch, _TORCH_DTYPES[npdt.name])
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape, dtype=np.int64)) if shape else 1
    out = torch.empty(n, dtype=tdt, device=device)
    if n == 0:
        return out.view(shape)
    threads = default_threads() if threads is None else threads
    stage = torch.empty(min(stage_elems, n), dtype=tdt, pin_memory=True)
    buf = stage.numpy()
    for start, vals in inputs.chunks(seed, ordinal, n, npdt, kind, r, threads=threads, buffer=buf):
        out[start:start + vals.size].copy_(stage[:vals.size])
    torch.cuda.synchronize(out.device)
    return out.view(shape)


def _wrap(v: int) -> int:
    """The unsigned 64-bit constant v as the int64 with the same bits."""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(z, k: int):
    """Logical right shift of int64 words (torch shifts int64 arithmetically)."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def generate_on_device(seed: int, ordinal: int, shape: Sequence[int], dtype, kind: str = inputs.UNIFORM,
                       r: int = 3, device: str = "cuda:0", chunk_elems: int = 1 << 26):
    """The tensor ``inputs.tensor(seed, ordinal, shape, dtype, kind, r)``, computed on ``device``.

    int64 multiplication and addition in torch wrap modulo 2^64, which is the generator's own
    arithmetic; shifts are made logical by masking.  Works on "cpu" as well (that is how the
    host-only test pins it to ``inputs``)."""
    import torch
    npdt = np.dtype(dtype)
    tdt = getattr(torch, _TORCH_DTYPES[npdt.name])
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape, dtype=np.int64)) if shape else 1
    out = torch.empty(n, dtype=tdt, device=device)
    key = _wrap(inputs.stream_key(seed, ordinal))
    gamma, m1, m2 = _wrap(inputs._GAMMA), _wrap(inputs._M1), _wrap(inputs._M2)
    for start in range(0, n, chunk_elems):
        m = min(chunk_elems, n - start)
        z = torch.arange(start + 1, start + m + 1, dtype=torch.int64, device=device)
        z = z * gamma + key
        z = (z ^ _lsr(z, 30)) * m1
        z = (z ^ _lsr(z, 27)) * m2
        z = z ^ _lsr(z, 31)
        if kind == inputs.UNIFORM:
            x = _lsr(z, 11).to(torch.float64)          # < 2^53: exact
            x = x * (2.0 ** -52) - 1.0                 # exact in binary64
            out[start:start + m] = x.to(tdt)
        elif kind == inputs.SMALLINT:
            out[start:start + m] = (_lsr(z, 32) % (2 * r + 1) - r).to(tdt)
        else:
            raise ValueError(f"unknown kind {kind!r}")
        del z
    return out.view(shape)
