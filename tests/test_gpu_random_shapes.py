"""GPU parity on seeded random shapes: a net under the host-side dispatch (tile plans, edge
and trailing-K forms, transposed and batched products, vector / ragged / element-load variants
of the tensor kernels).  Every case runs through the C ABI and is compared with the oracle:
integer-valued inputs bit for bit, uniform inputs within the normwise tolerance and the
element-by-element summation bound."""
import numpy as np
import pytest

from paper_2203_08069_amd import inputs

import _util as U

pytestmark = pytest.mark.gpu

DT = [np.float32, np.float64]


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2203_08069_amd import binding
    binding.load_library()
    return binding


def empty(shape, dtype):
    import torch
    return torch.full(tuple(shape), float("nan"), dtype=getattr(torch, np.dtype(dtype).name), device="cuda:0")


def check(got, ref, absref, dtype, kind, nterms):
    if kind == inputs.SMALLINT:
        U.assert_exact(got, ref)
    else:
        U.assert_close(got, ref, dtype, nterms)
        U.assert_componentwise(got, ref, absref(), dtype, nterms)


def extent(rng, hi):
    """Sizes that favour tile, vector and slice boundaries and their neighbours."""
    base = int(rng.choice([1, 2, 3, 4, 8, 16, 32, 48, 64, 96, 128, 192, 256, 320, 512, hi]))
    return max(1, min(hi, base + int(rng.integers(-3, 4))))


def cases(seed, n, draw):
    rng = np.random.default_rng(seed)
    return [draw(rng) for _ in range(n)]


GEMM_CASES = cases(101, 48, lambda r: (extent(r, 700), extent(r, 700), extent(r, 400), int(r.integers(0, 3)),
                                       int(r.integers(0, 3)), int(r.integers(0, 3)), bool(r.integers(0, 2))))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", [inputs.UNIFORM, inputs.SMALLINT])
@pytest.mark.parametrize("M,N,K,pa,pb,pc,acc", GEMM_CASES)
def test_gemm_random(lib, oracle, dtype, kind, M, N, K, pa, pb, pc, acc):
    """Operands are blocks of wider matrices (row padding 0, one vector, or an odd count) with accumulate on or off."""
    vec = 16 // np.dtype(dtype).itemsize
    pad = lambda p: (0, vec, 3)[p]
    wa, wb, wc = (U.gen(60, 0, (M, K + pad(pa)), dtype, kind), U.gen(60, 1, (K, N + pad(pb)), dtype, kind),
                  U.gen(60, 2, (M, N + pad(pc)), dtype, kind))
    dC = U.dev(wc)
    lib.distal_gemm(U.dev(wa)[:, :K], U.dev(wb)[:, :N], dC[:, :N], accumulate=acc)
    A, B, C0 = np.ascontiguousarray(wa[:, :K]), np.ascontiguousarray(wb[:, :N]), np.ascontiguousarray(wc[:, :N])
    out = U.host(dC)
    check(out[:, :N], oracle.gemm(A, B, init=C0 if acc else None),
          lambda: oracle.gemm(np.abs(A), np.abs(B), init=np.abs(C0) if acc else None), dtype, kind, K + 1)
    assert np.array_equal(out[:, N:], wc[:, N:])           # the padding columns are untouched


TENSOR_CASES = cases(202, 36, lambda r: (extent(r, 150), extent(r, 150), extent(r, 300), extent(r, 70)))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", [inputs.UNIFORM, inputs.SMALLINT])
@pytest.mark.parametrize("I,J,K,R", TENSOR_CASES)
def test_tensor_calls_random(lib, oracle, dtype, kind, I, J, K, R):
    """TTM, MTTKRP and TTV along every mode and the inner product on one random tensor."""
    shape = (I, J, K)
    B = U.gen(61, 0, shape, dtype, kind, 2)
    dB = U.dev(B)
    for mode in (0, 1, 2):
        n = shape[mode]
        a, b = [m for m in (0, 1, 2) if m != mode]
        C = U.gen(61, 1 + mode, (n, R), dtype, kind, 2)
        out_shape = list(shape)
        out_shape[mode] = R
        A = empty(out_shape, dtype)
        lib.distal_ttm_mode(mode, dB, U.dev(C), A)
        check(U.host(A), oracle.ttm_mode(mode, B, C), lambda: oracle.ttm_mode(mode, np.abs(B), np.abs(C)), dtype, kind, n)

        F1, F2 = U.gen(61, 4, (shape[a], R), dtype, kind, 2), U.gen(61, 5, (shape[b], R), dtype, kind, 2)
        A = empty((n, R), dtype)
        lib.distal_mttkrp_mode(mode, dB, U.dev(F1), U.dev(F2), A)
        check(U.host(A), oracle.mttkrp_mode(mode, B, F1, F2),
              lambda: oracle.mttkrp_mode(mode, np.abs(B), np.abs(F1), np.abs(F2)), dtype, kind, shape[a] * shape[b])

        c = U.gen(61, 6, (n,), dtype, kind, 2)
        A = empty((shape[a], shape[b]), dtype)
        lib.distal_ttv_mode(mode, dB, U.dev(c), A)
        check(U.host(A), oracle.ttv_mode(mode, B, c), lambda: oracle.ttv_mode(mode, np.abs(B), np.abs(c)), dtype, kind, n)

    C = U.gen(61, 7, shape, dtype, kind, 2)
    s = empty((1,), dtype)
    lib.distal_innerprod(dB, U.dev(C), s)
    ref = oracle.innerprod(B, C)
    got = float(U.host(s)[0])
    if kind == inputs.SMALLINT:
        assert got == ref
    else:
        assert got == float(np.asarray(ref, dtype=dtype)) or abs(got - ref) <= U.tol(dtype, I * J * K) * abs(ref)
