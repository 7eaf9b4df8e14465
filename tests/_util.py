"""Shared helpers for the GPU parity tests (comparison rules only, no arithmetic of the method)."""
import math

import numpy as np

from paper_2203_08069_amd import inputs

NP = {"f32": np.float32, "f64": np.float64}


def tol(dtype, reduction_length):
    """Normwise relative tolerance: 1e-12 for binary64, 1e-5*sqrt(K) for binary32,
    K being the number of terms summed per output element."""
    if np.dtype(dtype) == np.float64:
        return 1e-12
    return 1e-5 * math.sqrt(max(int(reduction_length), 1))


def normwise_err(got, ref):
    """max|got - ref| / max|ref| over the whole output (ref is the oracle's binary64 result)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if got.size == 0:
        return 0.0
    assert np.all(np.isfinite(got))
    scale = float(np.max(np.abs(ref)))
    err = float(np.max(np.abs(got - ref)))
    return err if scale == 0.0 else err / scale


def assert_close(got, ref, dtype, reduction_length):
    e = normwise_err(got, ref)
    assert e <= tol(dtype, reduction_length), f"normwise error {e:.3e} > {tol(dtype, reduction_length):.3e}"


def assert_componentwise(got, ref, absref, dtype, nterms):
    """Every element within the worst-case bound of floating-point summation in ANY order:
    |got - ref| <= (n + 8) u * sum|terms|, u the unit roundoff of dtype, n the number of terms
    (gamma_n of the standard analysis; the 8 covers the extra roundings of three-factor terms and
    of partial results).  absref = the same expression evaluated by the oracle on |inputs|."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    absref = np.asarray(absref, dtype=np.float64)
    assert got.shape == ref.shape == absref.shape
    u = 2.0 ** -53 if np.dtype(dtype) == np.float64 else 2.0 ** -24
    bound = (int(nterms) + 8) * u * absref
    bad = np.abs(got - ref) > bound
    assert not bad.any(), f"{int(bad.sum())} of {got.size} elements exceed the componentwise bound"


def assert_exact(got, ref):
    """Integer-valued inputs: every partial sum is exact, so the match is bit for bit
    (+0 and -0 compare equal: the sign of an exact zero depends on summation order)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref), f"{int((got != ref).sum())} of {got.size} elements differ"


def gen(seed, ordinal, shape, dtype, kind=inputs.UNIFORM, r=3):
    return inputs.tensor(seed, ordinal, shape, dtype, kind, r, threads=4)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.detach().cpu().numpy()
