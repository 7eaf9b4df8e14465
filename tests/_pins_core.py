"""A compact set of oracle pins in one function, so that it can be pointed at the real
oracle (must pass) and at copies of it with a planted mistake (must fail)."""
import itertools
from fractions import Fraction

import numpy as np

from paper_2203_08069_amd import inputs


def F(x):
    return Fraction(float(x))


def near(got, exact, ulps=1):
    ex = float(exact)
    return abs(float(got) - ex) <= ulps * np.spacing(max(abs(ex), 2.0 ** -60))


def run(o):
    for dtype in (np.float32, np.float64):
        t = lambda seed, ordinal, shape, kind=inputs.UNIFORM: inputs.tensor(seed, ordinal, shape, dtype, kind)
        # gemm: brute force, strided accumulate, permutation
        A, B = t(60, 0, (3, 5)), t(60, 1, (5, 4))
        out = o.gemm(A, B)
        for i, j in itertools.product(range(3), range(4)):
            assert near(out[i, j], sum(F(A[i, k]) * F(B[k, j]) for k in range(5)))
        bigc = t(60, 2, (5, 6))
        C0 = bigc[1:4, 1:5]
        out = o.gemm(A, B, init=C0)
        for i, j in itertools.product(range(3), range(4)):
            assert near(out[i, j], F(C0[i, j]) + sum(F(A[i, k]) * F(B[k, j]) for k in range(5)))
        # operands that are sub-blocks of larger matrices (leading dimension > row length)
        As, Bs = t(60, 3, (4, 9))[1:4, 2:7], t(60, 4, (7, 8))[1:6, 3:7]
        out = o.gemm(As, Bs)
        for i, j in itertools.product(range(3), range(4)):
            assert near(out[i, j], sum(F(As[i, k]) * F(Bs[k, j]) for k in range(5)))
        P = np.ascontiguousarray(np.eye(5, dtype=dtype)[:, [2, 0, 4, 1, 3]])
        assert np.array_equal(o.gemm(A, P), A[:, [2, 0, 4, 1, 3]].astype(np.float64))
        # ttv
        T, c = t(61, 0, (2, 3, 6)), t(61, 1, (6,))
        out = o.ttv(T, c)
        for i, j in itertools.product(range(2), range(3)):
            assert near(out[i, j], sum(F(T[i, j, k]) * F(c[k]) for k in range(6)))
        # innerprod: small, and across the fixed summation blocks
        T2 = t(61, 2, (2, 3, 6))
        ex = sum(F(T[i, j, k]) * F(T2[i, j, k]) for i, j, k in itertools.product(range(2), range(3), range(6)))
        assert near(o.innerprod(T, T2), ex)
        n = (2 << 20) + 321
        X, Y = t(62, 0, (1, 1, n), inputs.SMALLINT), t(62, 2, (1, 1, n), inputs.SMALLINT)
        assert o.innerprod(X, Y) == float((X.astype(np.int64) * Y.astype(np.int64)).sum())
        # ttm
        Cm = t(63, 1, (6, 4))
        out = o.ttm(T, Cm)
        for i, j, l in itertools.product(range(2), range(3), range(4)):
            assert near(out[i, j, l], sum(F(T[i, j, k]) * F(Cm[k, l]) for k in range(6)))
        # mttkrp
        Cf, Df = t(64, 1, (3, 4)), t(64, 2, (6, 4))
        out = o.mttkrp(T, Cf, Df)
        for i, l in itertools.product(range(2), range(4)):
            ex = sum(F(T[i, j, k]) * F(Cf[j, l]) * F(Df[k, l]) for j, k in itertools.product(range(3), range(6)))
            assert near(out[i, l], ex, ulps=4)
        # the same two contractions along every mode of the tensor
        for mode in (0, 1, 2):
            shape = T.shape
            a, b = [m for m in (0, 1, 2) if m != mode]
            Cn = t(65, 1, (shape[mode], 4))
            out = o.ttm_mode(mode, T, Cn)
            oshape = list(shape)
            oshape[mode] = 4
            assert out.shape == tuple(oshape)
            for idx in itertools.product(*(range(n) for n in oshape)):
                ex = Fraction(0)
                for x in range(shape[mode]):
                    src = list(idx)
                    src[mode] = x
                    ex += F(T[tuple(src)]) * F(Cn[x, idx[mode]])
                assert near(out[idx], ex)
            cn = t(65, 2, (shape[mode],))
            out = o.ttv_mode(mode, T, cn)
            for p_, q_ in itertools.product(range(shape[a]), range(shape[b])):
                ex = Fraction(0)
                for x in range(shape[mode]):
                    src = [0, 0, 0]
                    src[mode], src[a], src[b] = x, p_, q_
                    ex += F(T[tuple(src)]) * F(cn[x])
                assert near(out[p_, q_], ex)
            Ca, Db = t(66, 1, (shape[a], 3)), t(66, 2, (shape[b], 3))
            out = o.mttkrp_mode(mode, T, Ca, Db)
            for x, l in itertools.product(range(shape[mode]), range(3)):
                ex = Fraction(0)
                for p_, q_ in itertools.product(range(shape[a]), range(shape[b])):
                    src = [0, 0, 0]
                    src[mode], src[a], src[b] = x, p_, q_
                    ex += F(T[tuple(src)]) * F(Ca[p_, l]) * F(Db[q_, l])
                assert near(out[x, l], ex, ulps=4)
    # binary64 sums must be carried wider than binary64: a cancelling sum only a 64-bit
    # significand gets right (1 + 2^-60 - 1 keeps the small term)
    a = np.array([[1.0, 2.0 ** -60, -1.0]])
    b = np.ones((3, 1))
    assert o.gemm(a, b)[0, 0] == 2.0 ** -60
