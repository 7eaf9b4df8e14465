/*
 * Runs the CPU oracle (oracle/distal_oracle.c, compiled into this program with
 * -fsanitize=address,undefined) on cases read from a file, every operand in a heap buffer of
 * exactly its size, so that an out-of-bounds read or write, a misaligned access or an integer
 * overflow inside the oracle ends the program.  The binary64 results are written to a second
 * file; tests/test_host_sanitizers.py compares them bit for bit with the ordinary build.
 *
 * Case record: 11 int64 {op, dt, mode, I, J, K, L, lda, ldb, ldinit, accumulate}, then the
 * operands as raw little-endian arrays of dt in the order the oracle function takes them.
 *   op 0 gemm (I=M, J=N)  1 ttv  2 innerprod  3 ttm  4 mttkrp  5 ttm_mode  6 mttkrp_mode  7 ttv_mode
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_gemm(int, int64_t, int64_t, int64_t, const void *, int64_t, const void *, int64_t, const void *, int64_t, int, double *);
int oracle_ttv(int, int64_t, int64_t, int64_t, const void *, const void *, double *);
int oracle_innerprod(int, int64_t, int64_t, int64_t, const void *, const void *, double *);
int oracle_ttm(int, int64_t, int64_t, int64_t, int64_t, const void *, const void *, double *);
int oracle_mttkrp(int, int64_t, int64_t, int64_t, int64_t, const void *, const void *, const void *, double *);
int oracle_ttm_mode(int, int, int64_t, int64_t, int64_t, int64_t, const void *, const void *, double *);
int oracle_mttkrp_mode(int, int, int64_t, int64_t, int64_t, int64_t, const void *, const void *, const void *, double *);
int oracle_ttv_mode(int, int, int64_t, int64_t, int64_t, const void *, const void *, double *);

static void *read_exact(FILE *f, int64_t elems, size_t esz) {
    /* malloc(0) may return NULL: keep a one-byte block then, never dereferenced for zero elements */
    void *p = malloc(elems > 0 ? (size_t)elems * esz : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
    if (elems > 0 && fread(p, esz, (size_t)elems, f) != (size_t)elems) { fprintf(stderr, "short case file\n"); exit(3); }
    return p;
}

static int64_t strided(int64_t rows, int64_t cols, int64_t ld) { return (rows > 0 && cols > 0) ? (rows - 1) * ld + cols : 0; }

int main(int argc, char **argv) {
    if (argc != 3) { fprintf(stderr, "usage: %s cases.bin results.bin\n", argv[0]); return 2; }
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) { fprintf(stderr, "cannot open files\n"); return 2; }
    int64_t h[11];
    int ncases = 0;
    while (fread(h, sizeof(int64_t), 11, in) == 11) {
        const int op = (int)h[0], dt = (int)h[1], mode = (int)h[2], acc = (int)h[10];
        const int64_t I = h[3], J = h[4], K = h[5], L = h[6], lda = h[7], ldb = h[8], ldi = h[9];
        const size_t esz = dt == 1 ? 8 : 4;
        const int64_t dim[3] = {I, J, K};
        void *a = NULL, *b = NULL, *c = NULL;
        double *res = NULL;
        int64_t nres = 0;
        int rc = -1;
        switch (op) {
        case 0:
            a = read_exact(in, strided(I, K, lda), esz);
            b = read_exact(in, strided(K, J, ldb), esz);
            c = read_exact(in, acc ? strided(I, J, ldi) : 0, esz);
            nres = I * J; res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_gemm(dt, I, J, K, a, lda, b, ldb, acc ? c : NULL, ldi, acc, res);
            break;
        case 1:
            a = read_exact(in, I * J * K, esz); b = read_exact(in, K, esz);
            nres = I * J; res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_ttv(dt, I, J, K, a, b, res);
            break;
        case 2:
            a = read_exact(in, I * J * K, esz); b = read_exact(in, I * J * K, esz);
            nres = 1; res = malloc(8);
            rc = oracle_innerprod(dt, I, J, K, a, b, res);
            break;
        case 3:
            a = read_exact(in, I * J * K, esz); b = read_exact(in, K * L, esz);
            nres = I * J * L; res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_ttm(dt, I, J, K, L, a, b, res);
            break;
        case 4:
            a = read_exact(in, I * J * K, esz); b = read_exact(in, J * L, esz); c = read_exact(in, K * L, esz);
            nres = I * L; res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_mttkrp(dt, I, J, K, L, a, b, c, res);
            break;
        case 5:
            a = read_exact(in, I * J * K, esz); b = read_exact(in, dim[mode] * L, esz);
            nres = I * J * K / (dim[mode] ? dim[mode] : 1) * L; res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_ttm_mode(dt, mode, I, J, K, L, a, b, res);
            break;
        case 6:
            a = read_exact(in, I * J * K, esz);
            b = read_exact(in, (mode == 0 ? J : I) * L, esz);
            c = read_exact(in, (mode == 2 ? J : K) * L, esz);
            nres = dim[mode] * L; res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_mttkrp_mode(dt, mode, I, J, K, L, a, b, c, res);
            break;
        case 7:
            a = read_exact(in, I * J * K, esz); b = read_exact(in, dim[mode], esz);
            nres = I * J * K / (dim[mode] ? dim[mode] : 1); res = malloc(nres > 0 ? (size_t)nres * 8 : 1);
            rc = oracle_ttv_mode(dt, mode, I, J, K, a, b, res);
            break;
        default:
            fprintf(stderr, "unknown op %d\n", op); return 3;
        }
        if (rc != 0) { fprintf(stderr, "case %d (op %d): oracle returned %d\n", ncases, op, rc); return 4; }
        if (nres > 0 && fwrite(res, 8, (size_t)nres, out) != (size_t)nres) { fprintf(stderr, "write failed\n"); return 3; }
        free(a); free(b); free(c); free(res);
        ++ncases;
    }
    fclose(in);
    fclose(out);
    printf("oracle_asan_driver: %d cases ok\n", ncases);
    return 0;
}
