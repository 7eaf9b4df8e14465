"""Place seeded synthetic tensors (see ``inputs``) in device memory.

Values are generated on the host by ``inputs`` in pieces and copied through one
pinned staging buffer, so a 4 GiB tensor never needs a host copy.  The bytes on
the device are exactly those ``inputs.values`` returns for the same indices.
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
