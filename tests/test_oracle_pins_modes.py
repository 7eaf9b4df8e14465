"""Pins for the oracle's mode-n TTM and MTTKRP (the contractions of the evaluation
section's list taken along the other modes of B, as the Tucker and CP decompositions
it names need them).  Checked against exact rational brute force written out here,
numpy's exact int64 arithmetic, selection/identity closed forms, and the already
pinned last-mode / first-mode functions applied to a transposed copy of the tensor
(a transposition moves data and does no arithmetic).  No GPU needed.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from paper_2203_08069_amd import inputs

DTYPES = [np.float32, np.float64]
SHAPES = [(2, 3, 4), (4, 1, 3), (1, 5, 2), (3, 2, 1)]
EINSUM_TTV = {0: "ijk,i->jk", 1: "ijk,j->ik", 2: "ijk,k->ij"}
EINSUM_TTM = {0: "ijk,ir->rjk", 1: "ijk,jr->irk", 2: "ijk,kr->ijr"}
EINSUM_MTTKRP = {0: "ijk,jl,kl->il", 1: "ijk,il,kl->jl", 2: "ijk,il,jl->kl"}


def F(x):
    return Fraction(float(x))


def rnd(seed, ordinal, shape, dtype, kind=inputs.UNIFORM, r=3):
    return inputs.tensor(seed, ordinal, shape, dtype, kind, r)


def near(got, exact, ulps=1):
    ex = float(exact)
    return abs(float(got) - ex) <= ulps * np.spacing(max(abs(ex), 2.0 ** -60))


def others(mode):
    return [m for m in (0, 1, 2) if m != mode]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_ttm_mode_brute_force(oracle, dtype, shape, mode):
    R = 3
    B, C = rnd(70, 0, shape, dtype), rnd(70, 1, (shape[mode], R), dtype)
    out = oracle.ttm_mode(mode, B, C)
    oshape = list(shape)
    oshape[mode] = R
    assert out.shape == tuple(oshape)
    for idx in itertools.product(*(range(n) for n in oshape)):
        ex = Fraction(0)
        for x in range(shape[mode]):
            src = list(idx)
            src[mode] = x
            ex += F(B[tuple(src)]) * F(C[x, idx[mode]])
        assert near(out[idx], ex), (mode, idx)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_mttkrp_mode_brute_force(oracle, dtype, shape, mode):
    L = 2
    a, b = others(mode)
    B = rnd(71, 0, shape, dtype)
    C, D = rnd(71, 1, (shape[a], L), dtype), rnd(71, 2, (shape[b], L), dtype)
    out = oracle.mttkrp_mode(mode, B, C, D)
    assert out.shape == (shape[mode], L)
    for x, l in itertools.product(range(shape[mode]), range(L)):
        ex = Fraction(0)
        for p, q in itertools.product(range(shape[a]), range(shape[b])):
            src = [0, 0, 0]
            src[mode], src[a], src[b] = x, p, q
            ex += F(B[tuple(src)]) * F(C[p, l]) * F(D[q, l])
        assert near(out[x, l], ex, ulps=4), (mode, x, l)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_modes_against_int64(oracle, dtype, mode):
    shape = (5, 7, 6)
    a, b = others(mode)
    B = rnd(72, 0, shape, dtype, inputs.SMALLINT)
    C = rnd(72, 1, (shape[mode], 4), dtype, inputs.SMALLINT)
    got = oracle.ttm_mode(mode, B, C)
    ref = np.einsum(EINSUM_TTM[mode], B.astype(np.int64), C.astype(np.int64))
    assert np.array_equal(got, ref.astype(np.float64))
    Cf = rnd(72, 1, (shape[a], 3), dtype, inputs.SMALLINT, 2)
    Df = rnd(72, 2, (shape[b], 3), dtype, inputs.SMALLINT, 2)
    got = oracle.mttkrp_mode(mode, B, Cf, Df)
    ref = np.einsum(EINSUM_MTTKRP[mode], B.astype(np.int64), Cf.astype(np.int64), Df.astype(np.int64))
    assert np.array_equal(got, ref.astype(np.float64))


@pytest.mark.parametrize("dtype", DTYPES)
def test_last_and_first_mode_are_the_papers_statements(oracle, dtype):
    B = rnd(73, 0, (3, 4, 5), dtype)
    assert np.array_equal(oracle.ttm_mode(2, B, rnd(73, 1, (5, 6), dtype)),
                          oracle.ttm(B, rnd(73, 1, (5, 6), dtype)))
    C, D = rnd(73, 1, (4, 3), dtype), rnd(73, 2, (5, 3), dtype)
    assert np.array_equal(oracle.mttkrp_mode(0, B, C, D), oracle.mttkrp(B, C, D))


@pytest.mark.parametrize("dtype", DTYPES)
def test_modes_are_transposed_tensors(oracle, dtype):
    """Moving the contracted (or kept) mode into the position the paper's statement uses and
    calling the already pinned function gives the same sums in the same order: bit-identical."""
    B = rnd(74, 0, (4, 5, 6), dtype)
    # ttm mode 1: contract j.  Bt(i,k,j) = B(i,j,k); ttm gives (i,k,r); move r back to the middle
    C1 = rnd(74, 1, (5, 3), dtype)
    ref = oracle.ttm(np.ascontiguousarray(B.transpose(0, 2, 1)), C1).transpose(0, 2, 1)
    assert np.array_equal(oracle.ttm_mode(1, B, C1), ref)
    # ttm mode 0: contract i.  Bt(j,k,i) = B(i,j,k); ttm gives (j,k,r); move r to the front
    C0 = rnd(74, 1, (4, 3), dtype)
    ref = oracle.ttm(np.ascontiguousarray(B.transpose(1, 2, 0)), C0).transpose(2, 0, 1)
    assert np.array_equal(oracle.ttm_mode(0, B, C0), ref)
    # mttkrp mode 1: output rows j.  Bt(j,i,k); factors (i, k)
    Ci, Dk = rnd(74, 1, (4, 2), dtype), rnd(74, 2, (6, 2), dtype)
    ref = oracle.mttkrp(np.ascontiguousarray(B.transpose(1, 0, 2)), Ci, Dk)
    assert np.array_equal(oracle.mttkrp_mode(1, B, Ci, Dk), ref)
    # mttkrp mode 2: output rows k.  Bt(k,i,j); factors (i, j)
    Dj = rnd(74, 2, (5, 2), dtype)
    ref = oracle.mttkrp(np.ascontiguousarray(B.transpose(2, 0, 1)), Ci, Dj)
    assert np.array_equal(oracle.mttkrp_mode(2, B, Ci, Dj), ref)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_identity_and_selection(oracle, dtype, mode):
    shape = (3, 4, 5)
    a, b = others(mode)
    B = rnd(75, 0, shape, dtype)
    # the identity along the contracted mode returns B; a permutation permutes that mode
    n = shape[mode]
    assert np.array_equal(oracle.ttm_mode(mode, B, np.eye(n, dtype=dtype)), B.astype(np.float64))
    perm = np.roll(np.arange(n), 1)
    P = np.ascontiguousarray(np.eye(n, dtype=dtype)[:, perm])
    assert np.array_equal(oracle.ttm_mode(mode, B, P), np.take(B, perm, axis=mode).astype(np.float64))
    # unit columns in both factors select one fibre of B: A(x, l) = B(.., p_l, .., q_l, ..)
    L = 3
    ps, qs = [1, 0, 2], [2, 3, 0]
    C = np.zeros((shape[a], L), dtype=dtype)
    D = np.zeros((shape[b], L), dtype=dtype)
    for l in range(L):
        C[ps[l] % shape[a], l] = 1
        D[qs[l] % shape[b], l] = 1
    out = oracle.mttkrp_mode(mode, B, C, D)
    for x, l in itertools.product(range(n), range(L)):
        src = [0, 0, 0]
        src[mode], src[a], src[b] = x, ps[l] % shape[a], qs[l] % shape[b]
        assert out[x, l] == float(B[tuple(src)])
    # all-ones factors: sums over the two other modes
    ones = oracle.mttkrp_mode(mode, B, np.ones((shape[a], 1), dtype=dtype), np.ones((shape[b], 1), dtype=dtype))
    ref = B.astype(np.float64).sum(axis=(a, b))
    assert np.allclose(ones[:, 0], ref, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("dtype", DTYPES)
def test_modes_zero_extents_and_bad_arguments(oracle, dtype):
    B = np.zeros((2, 0, 3), dtype=dtype)
    assert np.array_equal(oracle.ttm_mode(1, B, np.zeros((0, 4), dtype=dtype)), np.zeros((2, 4, 3)))
    assert oracle.ttm_mode(0, B, np.zeros((2, 4), dtype=dtype)).shape == (4, 0, 3)
    out = oracle.mttkrp_mode(2, B, np.ones((2, 2), dtype=dtype), np.ones((0, 2), dtype=dtype))
    assert np.array_equal(out, np.zeros((3, 2)))
    with pytest.raises(ValueError):
        oracle.ttm_mode(3, np.zeros((2, 2, 2), dtype=dtype), np.zeros((2, 2), dtype=dtype))
    with pytest.raises(ValueError):
        oracle.ttm_mode(0, np.zeros((2, 3, 2), dtype=dtype), np.zeros((3, 2), dtype=dtype))
    with pytest.raises(ValueError):
        oracle.mttkrp_mode(1, np.zeros((2, 3, 4), dtype=dtype), np.zeros((3, 2), dtype=dtype),
                           np.zeros((4, 2), dtype=dtype))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_ttv_mode_brute_force(oracle, dtype, shape, mode):
    B, c = rnd(76, 0, shape, dtype), rnd(76, 1, (shape[mode],), dtype)
    out = oracle.ttv_mode(mode, B, c)
    keep = others(mode)
    assert out.shape == (shape[keep[0]], shape[keep[1]])
    for p, q in itertools.product(range(shape[keep[0]]), range(shape[keep[1]])):
        ex = Fraction(0)
        for x in range(shape[mode]):
            src = [0, 0, 0]
            src[mode], src[keep[0]], src[keep[1]] = x, p, q
            ex += F(B[tuple(src)]) * F(c[x])
        assert near(out[p, q], ex), (mode, p, q)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_ttv_mode_closed_forms(oracle, dtype, mode):
    shape = (5, 6, 7)
    B = rnd(77, 0, shape, dtype, inputs.SMALLINT)
    n = shape[mode]
    c = rnd(77, 1, (n,), dtype, inputs.SMALLINT)
    ref = np.einsum(EINSUM_TTV[mode], B.astype(np.int64), c.astype(np.int64))
    assert np.array_equal(oracle.ttv_mode(mode, B, c), ref.astype(np.float64))
    # all ones: the plain sum over the mode; a unit vector: the slice at that index
    assert np.array_equal(oracle.ttv_mode(mode, B, np.ones(n, dtype=dtype)), B.astype(np.float64).sum(axis=mode))
    e = np.zeros(n, dtype=dtype)
    e[n - 2] = 1
    assert np.array_equal(oracle.ttv_mode(mode, B, e), np.take(B, n - 2, axis=mode).astype(np.float64))
    # the last mode is the paper's statement; the others are it on a transposed copy, bit for bit
    Bf = rnd(77, 2, shape, dtype)
    cf = rnd(77, 3, (n,), dtype)
    if mode == 2:
        assert np.array_equal(oracle.ttv_mode(2, Bf, cf), oracle.ttv(Bf, cf))
    else:
        keep = others(mode)
        moved = np.ascontiguousarray(Bf.transpose(keep[0], keep[1], mode))
        assert np.array_equal(oracle.ttv_mode(mode, Bf, cf), oracle.ttv(moved, cf))
    # tensor times vector is tensor times a one-column matrix
    assert np.array_equal(oracle.ttv_mode(mode, Bf, cf),
                          np.squeeze(oracle.ttm_mode(mode, Bf, np.ascontiguousarray(cf[:, None])), axis=mode))
