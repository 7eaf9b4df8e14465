/*
 * distal.h - C ABI of the MI355X (gfx950) leaf-kernel library for the dense
 * tensor-algebra expressions of DISTAL (Yadav, Aiken, Kjolstad, PLDI 2022).
 *
 * A distributed schedule in the paper ends in a leaf: the code one processor
 * runs on the tiles it holds, either generated loops or a substituted
 * optimised kernel (the `substitute` command of the introductory SUMMA
 * listing).  This library is that leaf for five expressions, each stated in the
 * paper's tensor index notation, where an index that appears only on the
 * right-hand side is summed over its whole extent (background section).
 *
 * Common rules for every call
 *   - All tensor pointers are DEVICE pointers (HBM of the current HIP device)
 *     to dense row-major data, last index fastest (evaluation section: inputs
 *     are laid out row-major).  Element type is given by `dt`.
 *   - The caller owns every buffer, including workspaces.  The library never
 *     allocates, frees or synchronises inside these calls.  Inputs are only read.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *     Calls are asynchronous: outputs are valid once the stream reaches the
 *     point of the call.  A call enqueues kernels only (no memset or copy
 *     nodes), so sequences of calls can be recorded under HIP stream capture
 *     and replayed as a graph, provided the same call (same dtype and
 *     extents) has run once outside the capture on that device: the first
 *     launch of a kernel raises its LDS limit, which is not a stream operation.
 *   - Return value: DISTAL_OK (0) or a distal_status error code.  All argument
 *     checks happen on the host before anything is launched, so a call that
 *     returns an argument error has touched no device memory.
 *   - Extents are int64_t.  An extent of zero in a summed index gives a zero
 *     output (or leaves C unchanged under `accumulate`); an extent of zero in an
 *     output index is a successful no-op.  Negative extents are an error.
 *   - An output that starts at the same address as an input is rejected
 *     (DISTAL_ERR_ALIAS); partial overlaps are not detected and are undefined.
 *   - Arithmetic: binary64 expressions multiply and accumulate in binary64;
 *     binary32 expressions multiply and accumulate in binary32 or wider.  No
 *     reduced-precision emulation.  Summation order is fixed for a given call
 *     signature (dtype, extents, leading dimensions, flags and the 16-byte
 *     alignment of the operands), so results are bitwise reproducible run to run.
 */
#ifndef DISTAL_H
#define DISTAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DISTAL_F32 = 0, DISTAL_F64 = 1 } distal_dtype;

typedef enum {
    DISTAL_OK = 0,
    DISTAL_ERR_NULL = 1,      /* a required pointer is NULL                      */
    DISTAL_ERR_SHAPE = 2,     /* negative extent, or extents whose product overflows */
    DISTAL_ERR_DTYPE = 3,     /* dt is not DISTAL_F32 / DISTAL_F64               */
    DISTAL_ERR_STRIDE = 4,    /* a leading dimension is smaller than its row     */
    DISTAL_ERR_ALIAS = 5,     /* output pointer equals an input pointer          */
    DISTAL_ERR_WORKSPACE = 6, /* workspace missing, misaligned or too small      */
    DISTAL_ERR_LAUNCH = 7,    /* the HIP runtime refused a kernel launch         */
    DISTAL_ERR_MODE = 8       /* mode is not 0, 1 or 2                           */
} distal_status;

/*
 * Matrix-multiply tile step:  C(i,j) = [C(i,j) +] sum_k A(i,k) * B(k,j).
 * This is the local update every matrix-multiplication schedule of the paper
 * issues once per k-step ("A += B_l x C_l" in the SUMMA pseudocode, the tile
 * product of the Cannon and Johnson pseudocode; the paper names the output A
 * and the inputs B and C).
 *   A: M x K, row i starts at A + i*lda.   B: K x N, row k at B + k*ldb.
 *   C: M x N, row i at C + i*ldc.  lda >= K, ldb >= N, ldc >= N, in elements,
 *   so operands may be sub-blocks (k-chunks, tiles) of larger matrices.
 *   accumulate == 0: C is overwritten (its old contents are not read).
 *   accumulate != 0: the k-sum is added to the old C (SUMMA / Cannon k-steps).
 */
int distal_gemm(distal_dtype dt, int64_t M, int64_t N, int64_t K,
                const void *A, int64_t lda, const void *B, int64_t ldb,
                void *C, int64_t ldc, int accumulate, void *stream);

/*
 * Tensor times matrix:  A(i,j,l) = sum_k B(i,j,k) * C(k,l)
 * (evaluation section, list of higher-order expressions).
 *   B: I x J x K, C: K x L, A: I x J x L, all dense.  A is overwritten.
 * It is the matrix product of the (I*J) x K view of B with C and runs on the tiles
 * distal_gemm_plan reports for M = I*J, N = L - except for a rank-sized factor on a long tensor,
 * which has a kernel of its own (distal_ttm_slices_per_wave says when).
 */
int distal_ttm(distal_dtype dt, int64_t I, int64_t J, int64_t K, int64_t L,
               const void *B, const void *C, void *A, void *stream);

/*
 * Tensor times matrix along any mode of B (I x J x K).  C has one row per index
 * of the contracted mode and R columns; A is B with that mode's extent replaced
 * by R.  The evaluation section names TTM as a building block of the Tucker
 * decomposition, which applies it along every mode; its list states mode 2.
 *   mode 0: A(r,j,k) = sum_i B(i,j,k) * C(i,r)     C: I x R, A: R x J x K
 *   mode 1: A(i,r,k) = sum_j B(i,j,k) * C(j,r)     C: J x R, A: I x R x K
 *   mode 2: A(i,j,r) = sum_k B(i,j,k) * C(k,r)     C: K x R, A: I x J x R  (= distal_ttm)
 * All dense; A is overwritten.  B is read in place (no transposed copy is made).
 */
int distal_ttm_mode(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K, int64_t R,
                    const void *B, const void *C, void *A, void *stream);

/*
 * Matricized tensor times Khatri-Rao product:
 *   A(i,l) = sum_j sum_k B(i,j,k) * C(j,l) * D(k,l)
 * (evaluation section, list of higher-order expressions).
 *   B: I x J x K, C: J x L, D: K x L, A: I x L, all dense.  A is overwritten.
 *   workspace: device scratch of at least distal_mttkrp_workspace_bytes(...)
 *   bytes, 256-byte aligned; may be NULL when that size is 0.  Its contents on
 *   entry are ignored and on exit are unspecified.
 */
int distal_mttkrp(distal_dtype dt, int64_t I, int64_t J, int64_t K, int64_t L,
                  const void *B, const void *C, const void *D, void *A,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * MTTKRP along any mode of B (I x J x K): A has one row per index of that mode,
 * C and D are the factor matrices of the two other modes, in mode order.  The
 * evaluation section names MTTKRP as a building block of the canonical polyadic
 * decomposition, whose alternating sweep needs it along every mode; its list
 * states mode 0.
 *   mode 0: A(i,l) = sum_j sum_k B(i,j,k) * C(j,l) * D(k,l)   C: J x L, D: K x L  (= distal_mttkrp)
 *   mode 1: A(j,l) = sum_i sum_k B(i,j,k) * C(i,l) * D(k,l)   C: I x L, D: K x L
 *   mode 2: A(k,l) = sum_i sum_j B(i,j,k) * C(i,l) * D(j,l)   C: I x L, D: J x L
 * All dense; A is overwritten; B is read once, in place (no transposed copy).
 *   workspace: device scratch of at least distal_mttkrp_mode_workspace_bytes(...)
 *   bytes, 256-byte aligned; may be NULL when that size is 0.
 */
int distal_mttkrp_mode(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K, int64_t L,
                       const void *B, const void *C, const void *D, void *A,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Tensor times vector:  A(i,j) = sum_k B(i,j,k) * c(k)
 * (background section on tensor index notation; evaluation list).
 *   B: I x J x K, c: K, A: I x J, all dense.  A is overwritten.
 */
int distal_ttv(distal_dtype dt, int64_t I, int64_t J, int64_t K,
               const void *B, const void *c, void *A, void *stream);

/*
 * Tensor times vector along any mode of B (I x J x K).  c has one entry per index
 * of the contracted mode; A keeps the two other modes, in order.  (The background
 * section's statement contracts the last mode; the decompositions the evaluation
 * section names apply such products along every mode.)
 *   mode 0: A(j,k) = sum_i B(i,j,k) * c(i)     A: J x K
 *   mode 1: A(i,k) = sum_j B(i,j,k) * c(j)     A: I x K
 *   mode 2: A(i,j) = sum_k B(i,j,k) * c(k)     A: I x J   (= distal_ttv)
 * All dense; A is overwritten; B is read once, in place.
 */
int distal_ttv_mode(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K,
                    const void *B, const void *c, void *A, void *stream);

/*
 * Tensor inner product:  a = sum_i sum_j sum_k B(i,j,k) * C(i,j,k)
 * (evaluation list).  B, C: I x J x K dense.  `a` is a DEVICE pointer to one
 * element of type dt, overwritten.  Products are summed in binary64 for both
 * dtypes (per-block partial sums, then one fixed-order final pass - the
 * on-device part of the paper's node-level reduction), and rounded once to dt.
 *   workspace: device scratch of at least distal_innerprod_workspace_bytes(...)
 *   bytes, 256-byte aligned.
 */
int distal_innerprod(distal_dtype dt, int64_t I, int64_t J, int64_t K,
                     const void *B, const void *C, void *a,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * distal_innerprod for callers that cannot allocate or hand over device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result, bit
 * for bit, as distal_innerprod; the partial sums live in an array the library's code object
 * holds on every device (16 KiB, there until the process ends), so no workspace is passed and
 * nothing is allocated, freed or synchronised.  Every shape distal_innerprod accepts fits; a
 * shape whose partial sums would not fit returns DISTAL_ERR_WORKSPACE, and a runtime that
 * cannot give the array's address DISTAL_ERR_LAUNCH.  All calls on one device share the one
 * array: calls that may overlap in time on one device (different streams, different host
 * threads) race and must be ordered by the caller; calls on one stream are safe.
 */
int distal_innerprod_noalloc(distal_dtype dt, int64_t I, int64_t J, int64_t K,
                             const void *B, const void *C, void *a, void *stream);

/*
 * distal_gemm with the tile of the output chosen by the caller instead of by distal_gemm_plan:
 * for schedules that fix their leaf tile themselves, for tuning, and for tests that must reach
 * one particular kernel.  bm x bn is one of the tile shapes the dtype has kernels for (the BM x
 * BN pairs distal_gemm_plan can report for it: 256x256 and 128x256 [binary32], 256x128, 128x128,
 * 128x64, 64x128, 64x64, 128x32, 32x256, and 256x64, 64x256 [binary32]; into how many wavefronts a
 * tile is cut is the library's choice and does not change a result); anything else returns
 * DISTAL_ERR_SHAPE.  The whole product runs as one launch of that tile (plus the peeled
 * trailing columns and rows described under distal_gemm_plan); K < 16 takes the bounds-checked
 * kernel whatever the tile.  transposed_left != 0: the left operand is stored K x M (lda >= M)
 * and C = [C +] A^T * B (the product a tensor-times-matrix contraction over a non-last mode
 * consists of).  Other arguments, ownership and errors as distal_gemm.  It is the same
 * operation as distal_gemm (the local update of the matrix-multiplication schedules, whose
 * scheduling language lets the schedule divide loops down to a leaf tile of its own choosing);
 * which tile is fastest for given extents is what distal_gemm_plan estimates.
 */
int distal_gemm_tiled(distal_dtype dt, int transposed_left, int bm, int bn, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc,
                      int accumulate, void *stream);

/*
 * distal_gemm with scratch memory from the caller, for products whose output is small and whose
 * contracted index is long: such a product has fewer tiles than the part has compute units,
 * whatever the tile.  It is cut along k into parts - the way the three-dimensional schedules of
 * the matrix-multiplication case study (Johnson's algorithm, the 2.5D and COSMA schedules) cut
 * the k loop over processors and reduce - which run as one batch into M x N slabs of the
 * workspace; a second kernel adds the slabs in the order of k and then onto C, so the result is
 * a function of the extents only (it differs in rounding from distal_gemm's, which sums each
 * output in one run of k).
 *   distal_gemm_workspace_bytes(dt, M, N, K): bytes of workspace distal_gemm_ws needs for these
 *   extents; 0 where the product is not cut (at least 128 tiles, or K < 2048, or invalid
 *   arguments): distal_gemm_ws then is distal_gemm and ignores the workspace.
 *   workspace: DEVICE pointer, 256-byte aligned, at least that many bytes, distinct from the
 *   operands; its contents on entry do not matter, on return they are unspecified.
 * Other arguments, ownership and errors as distal_gemm; DISTAL_ERR_WORKSPACE for a missing, small
 * or misaligned workspace when one is needed.
 */
int distal_gemm_ws(distal_dtype dt, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                   const void *B, int64_t ldb, void *C, int64_t ldc, int accumulate,
                   void *workspace, size_t workspace_bytes, void *stream);
size_t distal_gemm_workspace_bytes(distal_dtype dt, int64_t M, int64_t N, int64_t K);

/*
 * Host-only query (no device work): how the library runs C = A * B with these extents (K >= 16).
 * Bases and leading dimensions need no alignment.  What the plan covers is the output without
 * the columns and rows the library peels off: the last distal_gemm_peeled_columns(...) columns
 * (a streaming matrix-vector kernel) and, with a transposed left operand, the last
 * M % (16 / sizeof dt) rows (bounds-checked kernel); pass the extents of that part.
 * K < 16 takes the bounds-checked 128 x 128 kernel.  TTM is such a
 * product: mode 2 is M = I*J, N = L; mode 0 is transposed_left with M = R, N = J*K, K = I;
 * mode 1 the same with batch = I, N = K, K = J.  accumulate as in distal_gemm: a product added
 * onto an old C takes its largest tiles from deeper K on (the tensor calls overwrite: 0).
 *   tile      = {BM, BN, BK}: tile and slab depth of the (first) launch
 *   split     = 0: one launch.  1: rows [0, cut) of C with `tile`, rows [cut, M) in a second
 *               launch with rest_tile.  2: the same along columns, [0, cut) and [cut, N).
 *               A product whose tiles would end in a thin last round of the compute units is
 *               split so that the first launch is whole rounds and the rest runs on small tiles.
 *   rest_tile = {BM, BN, BK} of the second launch, zeros when split == 0.
 * The plan is a function of the arguments only, never of the device.  Returns a status.
 */
int distal_gemm_plan(distal_dtype dt, int transposed_left, int64_t M, int64_t N, int64_t K, int64_t batch,
                     int accumulate, int tile[3], int *split, int64_t *cut, int rest_tile[3]);

/*
 * Host-only query: how many trailing columns of C = A * B the library computes apart from the
 * tiled launches.  0 when N is a multiple of 16 / sizeof dt.  Otherwise rows of B end inside a
 * 16-byte piece, and the library either takes them as they are inside the tiled kernels (0:
 * narrow outputs, where a second pass over the left operand would double the time) or peels
 * N % (16 / sizeof dt) columns off to a streaming kernel that reads the left operand once more
 * (wide outputs, where that pass costs a percent and the rest then runs on whole pieces); N
 * itself when N is narrower than one piece.  A function of the arguments only; -1 for invalid
 * arguments.  Results do not depend on it beyond rounding order in binary32.
 */
int64_t distal_gemm_peeled_columns(distal_dtype dt, int transposed_left, int64_t M, int64_t N, int64_t K,
                                   int64_t batch, int accumulate);

/*
 * Host-only query: which kernel distal_ttm (and distal_ttm_mode along mode 2) runs for a tensor of
 * `rows` = I*J rows of K elements and a K x L factor whose base is 16-byte aligned.  0: the tiled
 * matrix product on the (I*J) x K view.  1 ... 4: a rank-sized factor (L <= 32) on a long tensor
 * (at least 65536 rows) whose rows are at most 32 slices of 256 bytes - the factor then stays in
 * the registers of each workgroup, that many slices per wavefront, while the tensor streams by
 * once (evaluation section: TTM's leaves are matrix products; this is the one a factorisation's
 * shapes give).  The two kernels sum the terms of an output in different orders: results agree
 * within rounding, not bit for bit.  A function of the arguments only; 0 for invalid arguments.
 */
int distal_ttm_slices_per_wave(distal_dtype dt, int64_t rows, int64_t K, int64_t L);

/* Scratch sizes for the calls that take a workspace (0 for invalid arguments). */
size_t distal_mttkrp_workspace_bytes(distal_dtype dt, int64_t I, int64_t J, int64_t K, int64_t L);
size_t distal_mttkrp_mode_workspace_bytes(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K,
                                          int64_t L);
size_t distal_innerprod_workspace_bytes(distal_dtype dt, int64_t I, int64_t J, int64_t K);

/* Static, human-readable text for a distal_status value. */
const char *distal_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int distal_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DISTAL_H */
