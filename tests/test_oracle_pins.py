"""Pins for the CPU oracle: it is checked against things other than itself.

Exact rational brute force written out here from the index-notation statements
(paper: background section for TTV; evaluation list for innerprod, TTM,
MTTKRP; the introductory listing for the matrix multiply), closed forms,
numpy's exact int64 arithmetic on integer-valued tensors, cross-expression
identities, and the chunk orders of the paper's SUMMA / Cannon / Johnson
schedules.  None of these tests needs a GPU.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2203_08069_amd import inputs

DTYPES = [np.float32, np.float64]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def F(x):
    return Fraction(float(x))


def rnd(seed, ordinal, shape, dtype, kind=inputs.UNIFORM, r=3):
    return inputs.tensor(seed, ordinal, shape, dtype, kind, r)


def assert_rounds_exact(got, exact):
    """``got`` (binary64) is the correctly rounded value of the Fraction, or its neighbour."""
    got = float(got)
    ex = float(exact)  # Fraction -> float is correctly rounded
    if ex == 0.0:
        assert abs(got) <= 2.0 ** -60
    else:
        assert abs(got - ex) <= np.spacing(abs(ex)), (got, ex)


# ---------------------------------------------------------------- brute force

GEMM_SHAPES = [(1, 1, 1), (2, 3, 4), (4, 3, 2), (5, 1, 3), (1, 5, 2), (3, 4, 1), (3, 2, 5)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_brute_force(oracle, dtype, M, N, K):
    A, B = rnd(10, 0, (M, K), dtype), rnd(10, 1, (K, N), dtype)
    out = oracle.gemm(A, B)
    assert out.shape == (M, N) and out.dtype == np.float64
    for i in range(M):
        for j in range(N):
            ex = sum(F(A[i, k]) * F(B[k, j]) for k in range(K))
            assert_rounds_exact(out[i, j], ex)


@pytest.mark.parametrize("dtype", DTYPES)
def test_gemm_brute_force_strided_accumulate(oracle, dtype):
    # operands are sub-blocks of larger matrices, as a schedule's k-chunks are
    big_a, big_b, big_c = rnd(11, 0, (6, 9), dtype), rnd(11, 1, (8, 7), dtype), rnd(11, 2, (5, 6), dtype)
    A, B, C0 = big_a[1:4, 2:7], big_b[3:8, 1:5], big_c[2:5, 1:5]
    out = oracle.gemm(A, B, init=C0)
    for i in range(3):
        for j in range(4):
            ex = F(C0[i, j]) + sum(F(A[i, k]) * F(B[k, j]) for k in range(5))
            assert_rounds_exact(out[i, j], ex)


TENSOR_SHAPES = [(1, 1, 1), (2, 3, 4), (4, 2, 3), (3, 1, 5), (1, 4, 2), (2, 5, 1)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("I,J,K", TENSOR_SHAPES)
def test_ttv_brute_force(oracle, dtype, I, J, K):
    B, c = rnd(12, 0, (I, J, K), dtype), rnd(12, 1, (K,), dtype)
    out = oracle.ttv(B, c)
    assert out.shape == (I, J)
    for i, j in itertools.product(range(I), range(J)):
        assert_rounds_exact(out[i, j], sum(F(B[i, j, k]) * F(c[k]) for k in range(K)))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("I,J,K", TENSOR_SHAPES)
def test_innerprod_brute_force(oracle, dtype, I, J, K):
    B, C = rnd(13, 0, (I, J, K), dtype), rnd(13, 2, (I, J, K), dtype)
    ex = sum(F(B[i, j, k]) * F(C[i, j, k])
             for i, j, k in itertools.product(range(I), range(J), range(K)))
    assert_rounds_exact(oracle.innerprod(B, C), ex)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("I,J,K", TENSOR_SHAPES)
@pytest.mark.parametrize("L", [1, 3])
def test_ttm_brute_force(oracle, dtype, I, J, K, L):
    B, C = rnd(14, 0, (I, J, K), dtype), rnd(14, 1, (K, L), dtype)
    out = oracle.ttm(B, C)
    assert out.shape == (I, J, L)
    for i, j, l in itertools.product(range(I), range(J), range(L)):
        assert_rounds_exact(out[i, j, l], sum(F(B[i, j, k]) * F(C[k, l]) for k in range(K)))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("I,J,K", TENSOR_SHAPES)
@pytest.mark.parametrize("L", [1, 3])
def test_mttkrp_brute_force(oracle, dtype, I, J, K, L):
    B = rnd(15, 0, (I, J, K), dtype)
    C, D = rnd(15, 1, (J, L), dtype), rnd(15, 2, (K, L), dtype)
    out = oracle.mttkrp(B, C, D)
    assert out.shape == (I, L)
    for i, l in itertools.product(range(I), range(L)):
        ex = sum(F(B[i, j, k]) * F(C[j, l]) * F(D[k, l])
                 for j, k in itertools.product(range(J), range(K)))
        # binary64 triple products are rounded twice in the 64-bit significand
        got = out[i, l]
        assert abs(float(got) - float(ex)) <= 4 * np.spacing(max(abs(float(ex)), 2.0 ** -40))


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("dtype", DTYPES)
def test_gemm_identity(oracle, dtype):
    A = rnd(20, 0, (7, 5), dtype)
    assert np.array_equal(oracle.gemm(A, np.eye(5, dtype=dtype)), A.astype(np.float64))
    assert np.array_equal(oracle.gemm(np.eye(7, dtype=dtype), A), A.astype(np.float64))
    # a permutation matrix on the right permutes columns: catches a transposed operand
    P = np.ascontiguousarray(np.eye(5, dtype=dtype)[:, [2, 0, 4, 1, 3]])
    assert np.array_equal(oracle.gemm(A, P), A[:, [2, 0, 4, 1, 3]].astype(np.float64))


@pytest.mark.parametrize("dtype", DTYPES)
def test_ttv_closed_forms(oracle, dtype):
    B = rnd(21, 0, (4, 6, 9), dtype, inputs.SMALLINT)
    ones = np.ones(9, dtype=dtype)
    assert np.array_equal(oracle.ttv(B, ones), B.astype(np.float64).sum(axis=2))
    Bu = rnd(21, 0, (4, 6, 9), dtype)
    for m in (0, 4, 8):
        e = np.zeros(9, dtype=dtype)
        e[m] = 1
        assert np.array_equal(oracle.ttv(Bu, e), Bu[:, :, m].astype(np.float64))


@pytest.mark.parametrize("dtype", DTYPES)
def test_innerprod_closed_forms(oracle, dtype):
    B = rnd(22, 0, (5, 4, 7), dtype, inputs.SMALLINT)
    Bi = B.astype(np.int64)
    assert oracle.innerprod(B, B) == float((Bi * Bi).sum())
    assert oracle.innerprod(B, np.ones_like(B)) == float(Bi.sum())
    Bu, Cu = rnd(22, 0, (5, 4, 7), dtype), rnd(22, 2, (5, 4, 7), dtype)
    assert oracle.innerprod(Bu, Bu) > 0
    assert oracle.innerprod(Bu, Cu) == oracle.innerprod(Cu, Bu)


@pytest.mark.parametrize("dtype", DTYPES)
def test_innerprod_many_blocks(oracle, dtype):
    # spans several of the oracle's fixed summation blocks plus a ragged tail
    n = (3 << 20) + 12345
    B = rnd(23, 0, (1, 1, n), dtype, inputs.SMALLINT)
    C = rnd(23, 2, (1, 1, n), dtype, inputs.SMALLINT)
    exact = int((B.astype(np.int64) * C.astype(np.int64)).sum())
    assert oracle.innerprod(B, C) == float(exact)


@pytest.mark.parametrize("dtype", DTYPES)
def test_ttm_identity_and_gemm_view(oracle, dtype):
    B = rnd(24, 0, (3, 4, 6), dtype)
    assert np.array_equal(oracle.ttm(B, np.eye(6, dtype=dtype)), B.astype(np.float64))
    C = rnd(24, 1, (6, 5), dtype)
    # the paper casts TTM to matrix multiplies: B viewed as (I*J) x K
    assert np.array_equal(oracle.ttm(B, C).reshape(12, 5), oracle.gemm(B.reshape(12, 6), C))


@pytest.mark.parametrize("dtype", DTYPES)
def test_mttkrp_rank1_and_selection(oracle, dtype):
    B = rnd(25, 0, (4, 5, 6), dtype, inputs.SMALLINT)
    Bi = B.astype(np.int64)
    # rank-1 factors of ones: the outer sums
    out = oracle.mttkrp(B, np.ones((5, 1), dtype=dtype), np.ones((6, 1), dtype=dtype))
    assert np.array_equal(out[:, 0], Bi.sum(axis=(1, 2)).astype(np.float64))
    # rank-1 integer factors u, v: A(i) = sum_jk B(i,j,k) u_j v_k
    u = rnd(25, 1, (5, 1), dtype, inputs.SMALLINT)
    v = rnd(25, 2, (6, 1), dtype, inputs.SMALLINT)
    ex = np.einsum("ijk,j,k->i", Bi, u[:, 0].astype(np.int64), v[:, 0].astype(np.int64))
    assert np.array_equal(oracle.mttkrp(B, u, v)[:, 0], ex.astype(np.float64))
    # unit-vector columns select single entries: A(i,l) = B(i, p_l, q_l)
    Bu = rnd(25, 0, (4, 5, 6), dtype)
    ps, qs = [3, 0, 4], [1, 5, 2]
    C = np.zeros((5, 3), dtype=dtype)
    D = np.zeros((6, 3), dtype=dtype)
    for l, (p, q) in enumerate(zip(ps, qs)):
        C[p, l] = 1
        D[q, l] = 1
    out = oracle.mttkrp(Bu, C, D)
    for l, (p, q) in enumerate(zip(ps, qs)):
        assert np.array_equal(out[:, l], Bu[:, p, q].astype(np.float64))


# ------------------------------------------- exact integer arithmetic (numpy int64)

def structured(shape):
    """B(i,j,k) = ((i + 2j + 3k) mod 7) - 3, an integer tensor with no symmetry."""
    idx = np.indices(shape)
    return ((idx[0] + 2 * idx[1] + 3 * idx[2]) % 7) - 3


@pytest.mark.parametrize("dtype", DTYPES)
def test_all_ops_against_int64(oracle, dtype):
    I, J, K, L = 6, 9, 40, 5
    Bi = structured((I, J, K))
    B = Bi.astype(dtype)
    ci = np.arange(K) % 5 - 2
    Ci = (np.arange(K * L).reshape(K, L) * 7 % 11) - 5
    Cj = (np.arange(J * L).reshape(J, L) * 5 % 7) - 3
    B2i = structured((I, J, K))[::-1, :, ::-1] * 2 + 1
    assert np.array_equal(oracle.ttv(B, ci.astype(dtype)), np.einsum("ijk,k->ij", Bi, ci))
    assert oracle.innerprod(B, np.ascontiguousarray(B2i).astype(dtype)) == float((Bi * B2i).sum())
    assert np.array_equal(oracle.ttm(B, Ci.astype(dtype)), np.einsum("ijk,kl->ijl", Bi, Ci))
    assert np.array_equal(oracle.mttkrp(B, Cj.astype(dtype), Ci.astype(dtype)),
                          np.einsum("ijk,jl,kl->il", Bi, Cj, Ci))
    Ai = Bi.reshape(I * J, K)
    assert np.array_equal(oracle.gemm(Ai.astype(dtype), Ci.astype(dtype)), Ai @ Ci)


@pytest.mark.parametrize("dtype", DTYPES)
def test_structured_closed_form_sum(oracle, dtype):
    # over a full period of 7 in k the values -3..3 each occur once: the k-sum vanishes
    B = structured((3, 4, 7 * 6)).astype(dtype)
    assert np.array_equal(oracle.ttv(B, np.ones(42, dtype=dtype)), np.zeros((3, 4)))
    # sum of squares over one period is 28
    assert oracle.innerprod(B, B) == 28.0 * 6 * 12


# ---------------------------------------------------------------- cross-expression

@pytest.mark.parametrize("dtype", DTYPES)
def test_mttkrp_is_weighted_ttv(oracle, dtype):
    I, J, K, L = 3, 4, 5, 2
    B = rnd(30, 0, (I, J, K), dtype, inputs.SMALLINT)
    C = rnd(30, 1, (J, L), dtype, inputs.SMALLINT)
    D = rnd(30, 2, (K, L), dtype, inputs.SMALLINT)
    out = oracle.mttkrp(B, C, D)
    for l in range(L):
        t = oracle.ttv(B, np.ascontiguousarray(D[:, l]))       # (I, J)
        assert np.array_equal(out[:, l], (t * C[:, l].astype(np.float64)).sum(axis=1))


@pytest.mark.parametrize("dtype", DTYPES)
def test_ttv_is_rowwise_innerprod(oracle, dtype):
    B, c = rnd(31, 0, (2, 3, 11), dtype), rnd(31, 1, (11,), dtype)
    out = oracle.ttv(B, c)
    for i, j in itertools.product(range(2), range(3)):
        row = np.ascontiguousarray(B[i, j]).reshape(1, 1, 11)
        assert out[i, j] == oracle.innerprod(row, c.reshape(1, 1, 11))


@pytest.mark.parametrize("dtype", DTYPES)
def test_power_of_two_scaling(oracle, dtype):
    B, C = rnd(32, 0, (3, 4, 5), dtype), rnd(32, 1, (5, 2), dtype)
    assert np.array_equal(oracle.ttm(B * dtype(4), C), 4 * oracle.ttm(B, C))
    A, Bm = rnd(32, 0, (4, 6), dtype), rnd(32, 1, (6, 3), dtype)
    assert np.array_equal(oracle.gemm(A, Bm * dtype(0.5)), 0.5 * oracle.gemm(A, Bm))


# ------------------------------- the paper's schedules reproduce the one-shot product

def load_cannon_order():
    """kos(io, jo, ko) on the 3x3 grid of the paper's Cannon figure, from the fixture."""
    order = {}
    with open(os.path.join(GOLDEN, "cannon_rotation_3x3.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                io, jo, ko, kos = map(int, line)
                order[(io, jo, ko)] = kos
    return order


@pytest.mark.parametrize("dtype", DTYPES)
def test_summa_chunks_accumulate(oracle, dtype):
    """SUMMA pseudocode: step k in chunks, A += B_l x C_l each step."""
    M, N, K, chunk = 6, 5, 12, 4
    A, B = rnd(40, 0, (M, K), dtype, inputs.SMALLINT), rnd(40, 1, (K, N), dtype, inputs.SMALLINT)
    acc = np.zeros((M, N), dtype=dtype)
    for kc in range(0, K, chunk):
        acc = oracle.gemm(A[:, kc:kc + chunk], B[kc:kc + chunk, :], init=acc).astype(dtype)
    assert np.array_equal(acc.astype(np.float64), oracle.gemm(A, B))
    assert np.array_equal(acc.astype(np.int64), A.astype(np.int64) @ B.astype(np.int64))


@pytest.mark.parametrize("dtype", DTYPES)
def test_cannon_rotated_order(oracle, dtype):
    """Cannon on a 3x3 grid: processor (io,jo) takes k-tile kos=(ko+io+jo) mod 3 at step ko."""
    order = load_cannon_order()
    g, t = 3, 4
    n = g * t
    A, B = rnd(41, 0, (n, n), dtype, inputs.SMALLINT), rnd(41, 1, (n, n), dtype, inputs.SMALLINT)
    full = oracle.gemm(A, B)
    out = np.zeros((n, n))
    for io in range(g):
        for jo in range(g):
            seen = []
            acc = np.zeros((t, t), dtype=dtype)
            for ko in range(g):
                kos = order[(io, jo, ko)]
                assert kos == (ko + io + jo) % g
                seen.append(kos)
                acc = oracle.gemm(A[io * t:(io + 1) * t, kos * t:(kos + 1) * t],
                                  B[kos * t:(kos + 1) * t, jo * t:(jo + 1) * t], init=acc).astype(dtype)
            assert sorted(seen) == [0, 1, 2]
            out[io * t:(io + 1) * t, jo * t:(jo + 1) * t] = acc
    assert np.array_equal(out, full)


@pytest.mark.parametrize("dtype", DTYPES)
def test_johnson_partials_then_reduce(oracle, dtype):
    """Johnson: A_ijk = B_ik x C_kj computed independently, then summed over k."""
    g, t = 2, 3
    n = g * t
    A, B = rnd(42, 0, (n, n), dtype, inputs.SMALLINT), rnd(42, 1, (n, n), dtype, inputs.SMALLINT)
    total = np.zeros((n, n))
    for k in range(g):
        total += oracle.gemm(A[:, k * t:(k + 1) * t], B[k * t:(k + 1) * t, :])
    assert np.array_equal(total, oracle.gemm(A, B))


@pytest.mark.parametrize("dtype", DTYPES)
def test_pumma_and_solomonik_orders(oracle, dtype):
    """Algorithm table: PUMMA rotates the k-loop by io only (kos = (ko + io) mod gx); Solomonik's
    2.5D algorithm distributes k over c layers and runs Cannon's rotation (kio + io + jo) mod steps
    inside each layer, the layers being summed afterwards.  Both visit every k-tile exactly once per
    output tile, so integer inputs reproduce the one-shot product exactly."""
    g, t = 3, 4
    n = g * t
    A, B = rnd(24, 0, (n, n), dtype, inputs.SMALLINT), rnd(24, 1, (n, n), dtype, inputs.SMALLINT)
    ref = oracle.gemm(A, B)
    C = np.zeros((n, n), dtype=dtype)
    for io in range(g):
        for jo in range(g):
            seen = set()
            for ko in range(g):
                kos = (ko + io) % g
                seen.add(kos)
                C[io * t:(io + 1) * t, jo * t:(jo + 1) * t] = oracle.gemm(
                    A[io * t:(io + 1) * t, kos * t:(kos + 1) * t], B[kos * t:(kos + 1) * t, jo * t:(jo + 1) * t],
                    init=C[io * t:(io + 1) * t, jo * t:(jo + 1) * t]).astype(dtype)
            assert seen == set(range(g))
    assert np.array_equal(C.astype(np.float64), ref)
    # 2.5D: 2 x 2 x 2 grid over a 12 x 12 product, three rotated steps per layer
    g2, c, steps = 2, 2, 3
    tm, tk = n // g2, n // (c * steps)
    layers = [np.zeros((n, n), dtype=dtype) for _ in range(c)]
    for ko in range(c):
        for io in range(g2):
            for jo in range(g2):
                for kio in range(steps):
                    k0 = (ko * steps + (kio + io + jo) % steps) * tk
                    blk = (slice(io * tm, (io + 1) * tm), slice(jo * tm, (jo + 1) * tm))
                    layers[ko][blk] = oracle.gemm(A[blk[0], k0:k0 + tk], B[k0:k0 + tk, blk[1]],
                                                  init=layers[ko][blk]).astype(dtype)
    assert np.array_equal(sum(l.astype(np.float64) for l in layers), ref)


@pytest.mark.parametrize("dtype", DTYPES)
def test_chunked_float_matches_one_shot(oracle, dtype):
    M, N, K = 5, 4, 64
    A, B = rnd(43, 0, (M, K), dtype), rnd(43, 1, (K, N), dtype)
    acc = np.zeros((M, N), dtype=np.float64)
    for kc in range(0, K, 16):
        acc += oracle.gemm(A[:, kc:kc + 16], B[kc:kc + 16, :])
    np.testing.assert_allclose(acc, oracle.gemm(A, B), rtol=0, atol=1e-14)


# ---------------------------------------------------------------- edge cases

@pytest.mark.parametrize("dtype", DTYPES)
def test_zero_extents(oracle, dtype):
    z = np.zeros
    assert np.array_equal(oracle.gemm(z((3, 0), dtype), z((0, 4), dtype)), z((3, 4)))
    assert oracle.gemm(z((0, 2), dtype), z((2, 4), dtype)).shape == (0, 4)
    assert np.array_equal(oracle.ttv(z((2, 3, 0), dtype), z((0,), dtype)), z((2, 3)))
    assert oracle.innerprod(z((2, 0, 3), dtype), z((2, 0, 3), dtype)) == 0.0
    assert np.array_equal(oracle.ttm(z((2, 3, 0), dtype), z((0, 4), dtype)), z((2, 3, 4)))
    assert np.array_equal(oracle.mttkrp(z((2, 0, 3), dtype), z((0, 4), dtype), z((3, 4), dtype)), z((2, 4)))
    init = rnd(44, 2, (3, 4), dtype)
    assert np.array_equal(oracle.gemm(z((3, 0), dtype), z((0, 4), dtype), init=init), init.astype(np.float64))


def test_rejects_bad_arguments(oracle):
    with pytest.raises((TypeError, ValueError)):
        oracle.gemm(np.zeros((2, 3)), np.zeros((4, 2)))
    with pytest.raises(TypeError):
        oracle.gemm(np.zeros((2, 3), np.float32), np.zeros((3, 2), np.float64))
    with pytest.raises(TypeError):
        oracle.ttv(np.zeros((2, 3, 4), np.int32), np.zeros(4, np.int32))


def test_thread_count_independent(oracle):
    """One thread sums one output start to finish: 1 and 3 OpenMP threads agree bit for bit."""
    import subprocess
    import sys
    root = os.path.dirname(GOLDEN.rstrip("/")).rsplit("/tests", 1)[0]
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import numpy as np, oracle\n"
        "from paper_2203_08069_amd import inputs\n"
        "B = inputs.tensor(45, 0, (8, 9, 50), np.float64); C = inputs.tensor(45, 1, (50, 6), np.float64)\n"
        "n = (2 << 20) + 77\n"
        "X = inputs.tensor(45, 0, (1, 1, n), np.float32); Y = inputs.tensor(45, 2, (1, 1, n), np.float32)\n"
        "print(oracle.ttm(B, C).tobytes().hex()[:4000], oracle.innerprod(X, Y).hex())\n" % root)
    outs = []
    for nt in ("1", "3"):
        env = dict(os.environ, OMP_NUM_THREADS=nt)
        outs.append(subprocess.check_output([sys.executable, "-c", code], env=env))
    assert outs[0] == outs[1]


def test_stored_oracle_outputs(oracle):
    """Regression fixture written by tests/golden/make_oracle_golden.py (oracle only)."""
    path = os.path.join(GOLDEN, "oracle_small_cases.txt")
    cases = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                cases[line[0]] = [float.fromhex(x) for x in line[1:]]
    import importlib.util
    spec = importlib.util.spec_from_file_location(
        "make_oracle_golden", os.path.join(GOLDEN, "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    fresh = mod.compute_cases()
    assert set(fresh) == set(cases)
    for name, vals in fresh.items():
        assert [float(v) for v in vals] == cases[name], name
