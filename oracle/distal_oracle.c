/*
 * CPU oracle for the five dense leaf expressions of the DISTAL paper.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It is independent of the GPU code: it
 * includes none of its headers, calls no BLAS and no torch, and the product
 * never calls it.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may load it.
 *
 * Every expression here is a finite sum of products, so the method reaches
 * exactly (up to rounding order) a result with a plain definition; each
 * function below is that definition written out as nested loops in the index
 * order of the paper's statement:
 *
 *   gemm       A(i,j)   = sum_k   B(i,k) * C(k,j)            (paper: the matrix
 *              multiply of the introductory schedule listing; the leaf update
 *              "A += B_l x C_l" of the SUMMA, Cannon and Johnson pseudocode)
 *   ttv        A(i,j)   = sum_k   B(i,j,k) * c(k)            (background section
 *              on tensor index notation; evaluation, higher-order kernels)
 *   innerprod  a        = sum_ijk B(i,j,k) * C(i,j,k)        (evaluation list)
 *   ttm        A(i,j,l) = sum_k   B(i,j,k) * C(k,l)          (evaluation list)
 *   mttkrp     A(i,l)   = sum_jk  B(i,j,k) * C(j,l) * D(k,l) (evaluation list)
 *
 * and the higher-order contractions with a vector or a matrix taken along the other modes of B
 * (the evaluation section names TTM and MTTKRP as the building blocks of Tucker
 * and canonical polyadic decompositions, which apply them along every mode):
 *
 *   ttv_mode     0: A(j,k)   = sum_i B(i,j,k) * c(i)
 *                1: A(i,k)   = sum_j B(i,j,k) * c(j)
 *                2: A(i,j)   = sum_k B(i,j,k) * c(k)              (= ttv)
 *   ttm_mode     0: A(r,j,k) = sum_i B(i,j,k) * C(i,r)
 *                1: A(i,r,k) = sum_j B(i,j,k) * C(j,r)
 *                2: A(i,j,r) = sum_k B(i,j,k) * C(k,r)            (= ttm)
 *   mttkrp_mode  0: A(i,l)   = sum_jk B(i,j,k) * C(j,l) * D(k,l)  (= mttkrp)
 *                1: A(j,l)   = sum_ik B(i,j,k) * C(i,l) * D(k,l)
 *                2: A(k,l)   = sum_ij B(i,j,k) * C(i,l) * D(j,l)
 *
 * An index variable that occurs only on the right-hand side is summed over its
 * whole domain (background section, tensor index notation): every sum below
 * runs over the full extent of such an index.
 *
 * Layout: dense row-major, last index fastest (evaluation section: inputs are
 * laid out row-major).  gemm alone takes leading dimensions (in elements), as
 * the schedules hand it column/row slices of a tile.
 *
 * Arithmetic: operands (binary32 or binary64) are widened exactly to
 * long double (x87 80-bit, 64-bit significand, on x86-64); products and sums
 * are taken in long double, in increasing index order, and the sum is rounded
 * ONCE to binary64: that is "the oracle's fp64 result".  A product of two
 * binary32 values (48 bits) is exact in this type; a product of two binary64
 * values carries a relative error of at most 2^-64.  The paper fixes no
 * precision beyond using double tensors, and says nothing on summation order.
 *
 * Parallelism: OpenMP over output elements only.  One thread sums one output
 * element start to finish, so results do not depend on the thread count.
 * innerprod (a single output) sums fixed blocks of 2^20 consecutive elements,
 * then the block sums in block order; the blocking is a constant of this file,
 * not of the machine.
 *
 * Pins (tests/test_oracle_pins.py): exact rational brute force on tiny shapes,
 * identity/selection/all-ones closed forms, structured integer tensors with
 * closed-form sums, cross-expression identities, power-of-two scaling, and the
 * SUMMA/Cannon/Johnson chunk schedules of the paper reproducing the one-shot
 * product.  Random floating-point inputs are pinned only to within the
 * difference between long double and exact arithmetic (far below tolerance).
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_F64 1

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1

typedef long double acc_t;

static inline acc_t ld_elem(const void *p, int dt, int64_t n)
{
    return dt == ORACLE_F64 ? (acc_t)((const double *)p)[n]
                            : (acc_t)((const float *)p)[n];
}

int oracle_version(void) { return 1; }

int oracle_long_double_digits(void) { return __LDBL_MANT_DIG__; }

/* Number of OpenMP threads the loops below will use (1 when built without OpenMP). */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * out(i,j) = [init(i,j) +] sum_k A(i,k) * B(k,j)     (operand names as in the
 * C-ABI of the GPU library: out = A x B; the paper writes A = B x C.)
 * A is MxK with leading dimension lda, B is KxN with ldb, init (dtype dt, may
 * be NULL when accumulate == 0) is MxN with ldinit; out is binary64 MxN, dense.
 * accumulate != 0 models the leaf update "A += B_l x C_l" of the SUMMA and
 * Cannon pseudocode: the k-sum is formed first and then added to init.
 */
int oracle_gemm(int dt, int64_t M, int64_t N, int64_t K,
                const void *A, int64_t lda, const void *B, int64_t ldb,
                const void *init, int64_t ldinit, int accumulate, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (M < 0 || N < 0 || K < 0 || lda < K || ldb < N) return ORACLE_BAD_ARG;
    if (accumulate && (!init || ldinit < N)) return ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            acc_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += ld_elem(A, dt, i * lda + k) * ld_elem(B, dt, k * ldb + j);
            if (accumulate) s = ld_elem(init, dt, i * ldinit + j) + s;
            out[i * N + j] = (double)s;
        }
    }
    return ORACLE_OK;
}

/* A(i,j) = sum_k B(i,j,k) * c(k);  B is IxJxK, c has K entries, out is IxJ. */
int oracle_ttv(int dt, int64_t I, int64_t J, int64_t K,
               const void *B, const void *c, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0) return ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < I; ++i) {
        for (int64_t j = 0; j < J; ++j) {
            acc_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(c, dt, k);
            out[i * J + j] = (double)s;
        }
    }
    return ORACLE_OK;
}

/* a = sum_{i,j,k} B(i,j,k) * C(i,j,k);  B, C are IxJxK; out is one binary64. */
#define INNERPROD_BLOCK ((int64_t)1 << 20)
int oracle_innerprod(int dt, int64_t I, int64_t J, int64_t K,
                     const void *B, const void *C, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0) return ORACLE_BAD_ARG;
    const int64_t n = I * J * K; /* row-major: (i,j,k) -> (i*J+j)*K+k covers 0..n-1 */
    const int64_t nblocks = (n + INNERPROD_BLOCK - 1) / INNERPROD_BLOCK;
    acc_t total = 0;
    /* block sums are formed independently, then added in block order */
    enum { GROUP = 256 };
    acc_t part[GROUP];
    for (int64_t g = 0; g < nblocks; g += GROUP) {
        const int64_t gcount = nblocks - g < GROUP ? nblocks - g : GROUP;
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < gcount; ++b) {
            const int64_t lo = (g + b) * INNERPROD_BLOCK;
            const int64_t hi = lo + INNERPROD_BLOCK < n ? lo + INNERPROD_BLOCK : n;
            acc_t s = 0;
            for (int64_t m = lo; m < hi; ++m)
                s += ld_elem(B, dt, m) * ld_elem(C, dt, m);
            part[b] = s;
        }
        for (int64_t b = 0; b < gcount; ++b) total += part[b];
    }
    *out = (double)total;
    return ORACLE_OK;
}

/* A(i,j,l) = sum_k B(i,j,k) * C(k,l);  B is IxJxK, C is KxL, out is IxJxL. */
int oracle_ttm(int dt, int64_t I, int64_t J, int64_t K, int64_t L,
               const void *B, const void *C, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0 || L < 0) return ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < I; ++i) {
        for (int64_t j = 0; j < J; ++j) {
            for (int64_t l = 0; l < L; ++l) {
                acc_t s = 0;
                for (int64_t k = 0; k < K; ++k)
                    s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, k * L + l);
                out[(i * J + j) * L + l] = (double)s;
            }
        }
    }
    return ORACLE_OK;
}

/*
 * A(i,l) = sum_j sum_k B(i,j,k) * C(j,l) * D(k,l);
 * B is IxJxK, C is JxL, D is KxL, out is IxL.  The literal triple product is
 * summed; no factorisation into matrix products is used here.
 */
int oracle_mttkrp(int dt, int64_t I, int64_t J, int64_t K, int64_t L,
                  const void *B, const void *C, const void *D, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0 || L < 0) return ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < I; ++i) {
        for (int64_t l = 0; l < L; ++l) {
            acc_t s = 0;
            for (int64_t j = 0; j < J; ++j)
                for (int64_t k = 0; k < K; ++k)
                    s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, j * L + l)
                         * ld_elem(D, dt, k * L + l);
            out[i * L + l] = (double)s;
        }
    }
    return ORACLE_OK;
}

/*
 * Tensor times matrix along mode `mode` of B (IxJxK).  C has one row per index
 * of the contracted mode and R columns; the output has that mode replaced by R:
 *   mode 0: out(r,j,k) = sum_i B(i,j,k) * C(i,r)     C is IxR, out is RxJxK
 *   mode 1: out(i,r,k) = sum_j B(i,j,k) * C(j,r)     C is JxR, out is IxRxK
 *   mode 2: out(i,j,r) = sum_k B(i,j,k) * C(k,r)     C is KxR, out is IxJxR
 * Each case is its own loop nest, written out.
 */
int oracle_ttm_mode(int dt, int mode, int64_t I, int64_t J, int64_t K, int64_t R,
                    const void *B, const void *C, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0 || R < 0 || mode < 0 || mode > 2) return ORACLE_BAD_ARG;
    if (mode == 0) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t r = 0; r < R; ++r)
            for (int64_t j = 0; j < J; ++j)
                for (int64_t k = 0; k < K; ++k) {
                    acc_t s = 0;
                    for (int64_t i = 0; i < I; ++i)
                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, i * R + r);
                    out[(r * J + j) * K + k] = (double)s;
                }
    } else if (mode == 1) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = 0; i < I; ++i)
            for (int64_t r = 0; r < R; ++r)
                for (int64_t k = 0; k < K; ++k) {
                    acc_t s = 0;
                    for (int64_t j = 0; j < J; ++j)
                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, j * R + r);
                    out[(i * R + r) * K + k] = (double)s;
                }
    } else {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = 0; i < I; ++i)
            for (int64_t j = 0; j < J; ++j)
                for (int64_t r = 0; r < R; ++r) {
                    acc_t s = 0;
                    for (int64_t k = 0; k < K; ++k)
                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, k * R + r);
                    out[(i * J + j) * R + r] = (double)s;
                }
    }
    return ORACLE_OK;
}

/*
 * MTTKRP along mode `mode` of B (IxJxK): the output has one row per index of that
 * mode; C and D are the factor matrices of the two other modes, in mode order:
 *   mode 0: out(i,l) = sum_j sum_k B(i,j,k) * C(j,l) * D(k,l)    C JxL, D KxL
 *   mode 1: out(j,l) = sum_i sum_k B(i,j,k) * C(i,l) * D(k,l)    C IxL, D KxL
 *   mode 2: out(k,l) = sum_i sum_j B(i,j,k) * C(i,l) * D(j,l)    C IxL, D JxL
 * The literal triple product is summed, earlier mode outermost.
 */
int oracle_mttkrp_mode(int dt, int mode, int64_t I, int64_t J, int64_t K, int64_t L,
                       const void *B, const void *C, const void *D, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0 || L < 0 || mode < 0 || mode > 2) return ORACLE_BAD_ARG;
    if (mode == 0) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = 0; i < I; ++i)
            for (int64_t l = 0; l < L; ++l) {
                acc_t s = 0;
                for (int64_t j = 0; j < J; ++j)
                    for (int64_t k = 0; k < K; ++k)
                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, j * L + l)
                             * ld_elem(D, dt, k * L + l);
                out[i * L + l] = (double)s;
            }
    } else if (mode == 1) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t j = 0; j < J; ++j)
            for (int64_t l = 0; l < L; ++l) {
                acc_t s = 0;
                for (int64_t i = 0; i < I; ++i)
                    for (int64_t k = 0; k < K; ++k)
                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, i * L + l)
                             * ld_elem(D, dt, k * L + l);
                out[j * L + l] = (double)s;
            }
    } else {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t k = 0; k < K; ++k)
            for (int64_t l = 0; l < L; ++l) {
                acc_t s = 0;
                for (int64_t i = 0; i < I; ++i)
                    for (int64_t j = 0; j < J; ++j)
                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, i * L + l)
                             * ld_elem(D, dt, j * L + l);
                out[k * L + l] = (double)s;
            }
    }
    return ORACLE_OK;
}

/*
 * Tensor times vector along mode `mode` of B (IxJxK): c has one entry per index of
 * the contracted mode, the output keeps the two other modes in order:
 *   mode 0: out(j,k) = sum_i B(i,j,k) * c(i)     out is JxK
 *   mode 1: out(i,k) = sum_j B(i,j,k) * c(j)     out is IxK
 *   mode 2: out(i,j) = sum_k B(i,j,k) * c(k)     out is IxJ
 */
int oracle_ttv_mode(int dt, int mode, int64_t I, int64_t J, int64_t K,
                    const void *B, const void *c, double *out)
{
    if (dt != ORACLE_F32 && dt != ORACLE_F64) return ORACLE_BAD_ARG;
    if (I < 0 || J < 0 || K < 0 || mode < 0 || mode > 2) return ORACLE_BAD_ARG;
    if (mode == 0) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t j = 0; j < J; ++j)
            for (int64_t k = 0; k < K; ++k) {
                acc_t s = 0;
                for (int64_t i = 0; i < I; ++i)
                    s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(c, dt, i);
                out[j * K + k] = (double)s;
            }
    } else if (mode == 1) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = 0; i < I; ++i)
            for (int64_t k = 0; k < K; ++k) {
                acc_t s = 0;
                for (int64_t j = 0; j < J; ++j)
                    s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(c, dt, j);
                out[i * K + k] = (double)s;
            }
    } else {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = 0; i < I; ++i)
            for (int64_t j = 0; j < J; ++j) {
                acc_t s = 0;
                for (int64_t k = 0; k < K; ++k)
                    s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(c, dt, k);
                out[i * J + j] = (double)s;
            }
    }
    return ORACLE_OK;
}
