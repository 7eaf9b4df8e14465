// C ABI of the leaf-kernel library: argument checks on the host, then launches.
// Nothing here allocates, frees or synchronises; see include/distal.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>
#include <algorithm>
#include <cstdint>
#include <limits>

#include "../../include/distal.h"
#include "host_plan.hpp"
#include "gemm_kernel.hpp"
#include "mttkrp_kernel.hpp"
#include "ttm_kernel.hpp"
#include "stream_kernels.hpp"

using namespace distal;

namespace {

constexpr int kMaxDevices = 64;
constexpr size_t kWorkspaceAlign = 256;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int current_device() {
    int d = 0;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) d = 0;
    return d;
}

// Opt in, once per device and kernel, to dynamic LDS beyond the default limit.
template <typename Kern>
bool allow_lds(Kern kern, int bytes, std::atomic<bool> (&done)[kMaxDevices]) {
    if (bytes <= 48 * 1024) return true;
    const int d = current_device();
    if (done[d].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    done[d].store(true, std::memory_order_release);
    return true;
}

constexpr int64_t kMaxGridY = 65535;

// One launch of one form of the straight-line kernel (each form raises its LDS limit once per device).
template <typename T, int BM, int BN, int BK, int WM, int WN, bool TA, int EDGE, bool INIT, bool FINE, bool SHIFT>
bool launch_fast_form(const dim3 &grid, const ContractArgs<T> &a, hipStream_t stream) {
    typedef ContractCfg<T, BM, BN, BK, WM, WN, TA, FINE> Cfg;
    static std::atomic<bool> done[kMaxDevices];
    auto kern = contract_fast_kernel<T, BM, BN, BK, WM, WN, TA, EDGE, INIT, FINE, SHIFT>;
    if (!allow_lds(kern, Cfg::LDS_BYTES, done)) return false;
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::NT), Cfg::LDS_BYTES, stream, a);
    return true;
}

// One launch per run of at most kMaxGridY problems of the batch (blockIdx.y picks the problem).
// KIND: the guarded kernel, the straight-line kernel on whole tiles, or its edge-clamping form.
enum { kGuarded = 0, kWhole = 1, kEdge = 2, kEdgeK = 3 };
template <typename T, int BM, int BN, int BK, int WM, int WN, int KIND, bool TA, bool FINE = false>
int launch_contract(ContractArgs<T> a, int64_t batch, hipStream_t stream) {
    typedef ContractCfg<T, BM, BN, BK, WM, WN, TA, FINE> Cfg;
    a.tiles_m = (int)((a.M + BM - 1) / BM);
    a.tiles_n = (int)((a.N + BN - 1) / BN);
    const int64_t nblocks = (int64_t)a.tiles_m * a.tiles_n;
    static std::atomic<bool> done[kMaxDevices];
    for (int64_t first = 0; first < batch; first += kMaxGridY) {
        const int64_t count = batch - first < kMaxGridY ? batch - first : kMaxGridY;
        const dim3 grid((unsigned)nblocks, (unsigned)count);
        if constexpr (KIND == kGuarded) {
            auto kern = contract_kernel<T, BM, BN, BK, WM, WN, TA>;
            if (!allow_lds(kern, Cfg::LDS_BYTES, done)) return DISTAL_ERR_LAUNCH;
            hipLaunchKernelGGL(kern, grid, dim3(Cfg::NT), Cfg::LDS_BYTES, stream, a);
        } else {
            constexpr int EDGE = KIND == kEdgeK ? 2 : (KIND == kEdge ? 1 : 0);
            // binary32, tiles up to 128 x 128, at most 256 terms: the old C goes into the accumulators up
            // front, so the short k-loop is not followed by a read-modify-write (8192 x 8192 x 128 on
            // 64 x 128 tiles: 59 -> 63 % of peak).  Deeper products and larger tiles add in the epilogue:
            // there the up-front form measured 1..4 % slower at every depth.
            constexpr bool kInitForm = sizeof(T) == 4 && BM * BN <= 128 * 128;
            // rows of B that end inside a 16-byte piece take the edge forms that shift the last piece
            const bool shift = EDGE != 0 && a.N % (16 / (int)sizeof(T)) != 0;
            const bool init = kInitForm && a.accumulate && a.K <= 256;
            // (a form the tile has no use for collapses onto the plain one at compile time)
            auto form = [&](auto init_c, auto shift_c) {
                constexpr bool I = decltype(init_c)::value && kInitForm, S = decltype(shift_c)::value && EDGE != 0;
                return launch_fast_form<T, BM, BN, BK, WM, WN, TA, EDGE, I, FINE, S>(grid, a, stream);
            };
            const std::true_type yes{};
            const std::false_type no{};
            const bool ok = init ? (shift ? form(yes, yes) : form(yes, no)) : (shift ? form(no, yes) : form(no, no));
            if (!ok) return DISTAL_ERR_LAUNCH;
        }
        if (hipGetLastError() != hipSuccess) return DISTAL_ERR_LAUNCH;
        a.A += count * a.batch_a;
        a.B += count * a.batch_b;
        a.C += count * a.batch_c;
    }
    return DISTAL_OK;
}

// The straight-line kernel with BM x BN x BK tiles on operands whose 16-byte pieces never
// straddle an edge (K >= BK): whole tiles as they are, ragged M or N through the edge-clamping
// form, K % BK trailing terms as that form's extra slab - or, where pieces of A would straddle
// the end of K (no TA, K not a multiple of the vector), by a second, guarded pass over C.
template <typename T, int BM, int BN, int BK, int WM, int WN, bool TA, bool FINE = false>
int launch_tiles(ContractArgs<T> a, int64_t batch, hipStream_t stream) {
    constexpr int VEC = 16 / (int)sizeof(T);
    if (a.K < BK) return launch_contract<T, 128, 128, 16, 2, 2, kGuarded, TA>(a, batch, stream);   // no whole slab
    // leading dimensions so large that a slab's rows lie more than 4 GiB apart: the straight-line
    // kernel's 32-bit offsets do not reach, the bounds-checked kernel addresses with pointers
    if (!slab_offsets_fit((int64_t)sizeof(T), TA, BM, BN, BK, a.lda, a.ldb)) return launch_contract<T, 128, 128, 16, 2, 2, kGuarded, TA>(a, batch, stream);
    // a row of B that ends inside a piece is fetched from column N - VEC: that column must exist
    if (a.N % VEC != 0 && a.N + a.n_before < VEC) return launch_contract<T, 128, 128, 16, 2, 2, kGuarded, TA>(a, batch, stream);
    const int64_t k_main = a.K / BK * BK, k_tail = a.K - k_main;
    if (k_tail == 0)
        return (a.M % BM == 0 && a.N % BN == 0) ? launch_contract<T, BM, BN, BK, WM, WN, kWhole, TA, FINE>(a, batch, stream)
                                                : launch_contract<T, BM, BN, BK, WM, WN, kEdge, TA, FINE>(a, batch, stream);
    if (TA || a.K % VEC == 0) return launch_contract<T, BM, BN, BK, WM, WN, kEdgeK, TA, FINE>(a, batch, stream);
    ContractArgs<T> m = a;
    m.K = k_main;
    const int rc = launch_contract<T, BM, BN, BK, WM, WN, kEdge, TA, FINE>(m, batch, stream);
    if (rc != DISTAL_OK) return rc;
    ContractArgs<T> t = a;                       // k_main is a multiple of 16: alignment is unchanged
    t.A += k_main;
    t.B += k_main * a.ldb;
    t.K = k_tail;
    t.accumulate = 1;
    return launch_contract<T, 128, 128, 16, 2, 2, kGuarded, TA>(t, batch, stream);
}

template <typename T>
int launch_fill(T *out, int64_t rows, int64_t cols, int64_t ld, hipStream_t stream) {
    const int64_t n = rows * cols;
    if (n == 0) return DISTAL_OK;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, stream, out, rows, cols, ld, T(0));
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

// ---- matrix multiply ------------------------------------------------------
// Tile choice depends on the shape only.  What matters most is four wavefronts per SIMD (at most
// 128 registers each) and at least two workgroups per compute unit, so that one's prologue and
// epilogue run under the other's k-loop: the tile large grids run on is 128 x 128 in both types,
// eight wavefronts of 32 x 64 (2 x 4 blocks of the 16 x 16 x 4 instruction); binary32 also has
// 128 x 256 and 256 x 128 on eight wavefronts of 64 x 64 and 256 x 256 on sixteen (32 x 32 x 2
// blocks, 32-deep slabs), binary64 256 x 128 on sixteen - they win where a compute unit gets one or
// two tiles; 128 x 64, 64 x 128 and 64 x 64 tiles serve problems too small to fill the part with
// those.  Among the shapes a product is deep enough for, the one with the
// least estimated time wins: tiles per compute unit, a partly filled last round counted in
// full, x tile area / the efficiency measured for that tile at that many tiles per compute
// unit (tile_candidates() holds the table).  A rank-sized output side (N <= 64, or M <= 64 as
// the transposed forms of a tensor-times-matrix have it) adds tiles with a 64- or 32-wide short
// side, which read the large operand once instead of padding the narrow one to 64.  Whole
// tiles take the straight-line kernels as they are, ragged M and N their edge-clamping
// form (the padding is paid for through the tile count), with one more zero-filled slab for
// K % BK trailing terms.  Alignment does not matter; columns (and, transposed, rows) whose
// 16-byte pieces would straddle an edge are peeled off first (see gemm_t).  A grid that would
// end in a thin last round is cut into two launches (plan_product).

// The launch for a tile id of tile_candidates().  How many wavefronts share a tile is chosen here,
// not by the caller: the result does not depend on it (every output sums its terms in the same
// order whichever wavefront owns it), only the speed does.  A grid that gives a compute unit one
// tile or two leaves its SIMDs with one wavefront each unless the tile is cut into more of them:
// binary64 128 x 128 on sixteen wavefronts of 32 x 32 instead of eight of 32 x 64 measures 92.3
// against 88.8 % of peak at 256 tiles (sixteen of 16 x 64: 90.8), 91.2 against 93.6 at 512; binary64 64 x 64 on eight instead of four 74.2 against 64.1
// at 1024^3 (256 tiles), level from 600 tiles on.  The binary64 128 x 64 and 64 x 128 tiles run on
// eight wavefronts of 32 x 32 at every grid size (4096^2 x 2048: 93.5 against 88.8 and 94.9
// against 92.4 on four).  In binary32 a wavefront of 32 x 32 would own a single block of the
// 32 x 32 x 2 instruction and measured 1 to 5 points slower; the binary32 tiles up to 128 x 128
// therefore use the 16 x 16 x 4 instruction (FINE), eight wavefronts of 2 x 2 blocks (2 x 4 on
// 128 x 128, 1 x 2 on 64 x 64), at every grid size - a different instruction sums in a different
// order, so a tile name stands for one of the two and never both: 64 x 64 x 32 at 4096^2 x 2048
// 87.9 -> 91.2 % of peak, at 3000^3 82.4 -> 86.2; 128 x 64 at 256 tiles 68.4 -> 81.3; 128 x 128
// at 8192^3 93.3 -> 96.2.
template <typename T, bool TA>
int launch_by_id(int id, const ContractArgs<T> &a, int64_t batch, hipStream_t stream) {
    auto tiles = [&](int bm, int bn) { return ((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * batch; };
    switch (id) {
    case 1:
        // a transposed left operand is staged in rows of 256 either way: 16-deep slabs measure 1 % faster
        if constexpr (sizeof(T) == 4) {
            if constexpr (TA) return launch_tiles<T, 256, 256, 16, 4, 4, TA>(a, batch, stream);
            else return launch_tiles<T, 256, 256, 32, 4, 4, TA>(a, batch, stream);
        }
        break;
    case 2:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 256, 128, 16, 4, 2, TA>(a, batch, stream);
        else return launch_tiles<T, 256, 128, 16, 8, 2, TA>(a, batch, stream);
    case 3:
        if constexpr (sizeof(T) == 4) {
            return launch_tiles<T, 128, 128, 16, 4, 2, TA, true>(a, batch, stream);
        } else {
            if (tiles(128, 128) <= 256) return launch_tiles<T, 128, 128, 16, 4, 4, TA>(a, batch, stream);
            return launch_tiles<T, 128, 128, 16, 4, 2, TA>(a, batch, stream);
        }
    case 5:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 256, 64, 16, 4, 1, TA>(a, batch, stream);
        else return launch_tiles<T, 128, 64, 16, 4, 2, TA>(a, batch, stream);
    case 6:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 128, 32, 32, 4, 1, TA>(a, batch, stream);
        else return launch_tiles<T, 128, 32, 16, 4, 1, TA>(a, batch, stream);
    case 7:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 64, 256, 16, 1, 4, TA>(a, batch, stream);
        else return launch_tiles<T, 64, 128, 16, 4, 2, TA>(a, batch, stream);
    case 8:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 32, 256, 32, 1, 4, TA>(a, batch, stream);
        else return launch_tiles<T, 32, 256, 16, 1, 4, TA>(a, batch, stream);
    case 9:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 128, 64, 32, 4, 2, TA, true>(a, batch, stream);
        break;
    case 10:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 64, 128, 32, 4, 2, TA, true>(a, batch, stream);
        break;
    case 11:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 64, 64, 32, 4, 2, TA, true>(a, batch, stream);
        break;
    case 12:
        if constexpr (sizeof(T) == 4) return launch_tiles<T, 128, 256, 16, 2, 4, TA>(a, batch, stream);
        break;
    default: break;
    }
    // too few larger tiles to give every CU one: quarter-size tiles, four times the workgroups
    if constexpr (sizeof(T) == 8)
        if (tiles(64, 64) <= 512) return launch_tiles<T, 64, 64, 16, 4, 2, TA>(a, batch, stream);
    return launch_tiles<T, 64, 64, 16, 2, 2, TA>(a, batch, stream);
}

// TA = false: C = [C +] A * B with A stored M x K.  TA = true: the left operand is stored
// K x M (C = [C +] At^T * B), the form a contraction over a non-last tensor mode takes.
// `batch` independent problems, operand p of problem n at p + n * stride_p (elements).
template <typename T, bool TA = false>
int gemm_t(int64_t M, int64_t N, int64_t K, const T *A, int64_t lda, const T *B, int64_t ldb,
           T *C, int64_t ldc, int accumulate, hipStream_t stream, int64_t batch = 1,
           int64_t stride_a = 0, int64_t stride_b = 0, int64_t stride_c = 0, int force_id = 0) {
    constexpr int VEC = 16 / (int)sizeof(T);
    if (M == 0 || N == 0 || batch == 0) return DISTAL_OK;
    if (K == 0) {
        if (accumulate) return DISTAL_OK;
        for (int64_t n = 0; n < batch; ++n) {
            const int rc = launch_fill<T>(C + n * stride_c, M, N, ldc, stream);
            if (rc != DISTAL_OK) return rc;
        }
        return DISTAL_OK;
    }
    const int64_t tm = (M + 127) / 128, tn = (N + 127) / 128;
    int64_t nblocks;
    if (!mul_ok(tm, tn, &nblocks) || nblocks > std::numeric_limits<int>::max()) return DISTAL_ERR_SHAPE;
    ContractArgs<T> a{};
    a.A = A; a.B = B; a.C = C;
    a.M = M; a.N = N; a.K = K;
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.batch_a = stride_a; a.batch_b = stride_b; a.batch_c = stride_c;
    a.accumulate = accumulate ? 1 : 0;
    a.a_vec_ok = aligned16(A) && lda % VEC == 0 && stride_a % VEC == 0;
    a.b_vec_ok = aligned16(B) && ldb % VEC == 0 && stride_b % VEC == 0;
    a.c_vec_ok = aligned16(C) && ldc % VEC == 0 && stride_c % VEC == 0;
    if (K < 16) return launch_contract<T, 128, 128, 16, 2, 2, kGuarded, TA>(a, batch, stream);
    // The straight-line kernels move 16-byte pieces (alignment does not matter: their global accesses
    // are only element-aligned).  A row of B that does not end on a piece is either handled inside
    // them (the last piece is fetched VEC columns before the end, which takes N >= VEC) or its
    // trailing N % VEC columns go to a streaming kernel, whichever peeled_columns estimates cheaper.
    // Pieces of a transposed left operand must not straddle its last column: there the trailing
    // M % VEC rows of C are peeled off to the guarded kernel.
    const int64_t nfr = peeled_columns(sizeof(T) == 8, TA, M, N, K, batch, accumulate != 0), mfr = TA ? M % VEC : 0;
    const int64_t Nm = N - nfr, Mm = M - mfr;
    if (nfr > 0) {
        int64_t blocks = TA ? (M + 255) / 256 : (M + 31) / 32;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        for (int64_t first = 0; first < batch; first += kMaxGridY) {
            const int64_t count = batch - first < kMaxGridY ? batch - first : kMaxGridY;
            const dim3 grid((unsigned)blocks, (unsigned)count);
            const T *Af = A + first * stride_a, *Bf = B + first * stride_b + Nm;
            T *Cf = C + first * stride_c + Nm;
            if constexpr (TA)
                hipLaunchKernelGGL(gemm_fringe_cols_ta_kernel<T>, grid, dim3(256), 0, stream, Af, lda, Bf, ldb, Cf, ldc,
                                   M, K, (int)nfr, a.accumulate, stride_a, stride_b, stride_c);
            else
                hipLaunchKernelGGL(gemm_fringe_cols_kernel<T>, grid, dim3(256), 0, stream, Af, lda, Bf, ldb, Cf, ldc,
                                   M, K, (int)nfr, a.accumulate, stride_a, stride_b, stride_c);
            if (hipGetLastError() != hipSuccess) return DISTAL_ERR_LAUNCH;
        }
        if (Nm == 0) return DISTAL_OK;
    }
    if (mfr > 0) {
        ContractArgs<T> r = a;                   // rows [Mm, M) x columns [0, Nm)
        r.A += Mm;
        r.C += Mm * ldc;
        r.M = mfr;
        r.N = Nm;
        r.a_vec_ok = r.c_vec_ok = 0;
        const int rc = launch_contract<T, 128, 128, 16, 2, 2, kGuarded, TA>(r, batch, stream);
        if (rc != DISTAL_OK || Mm == 0) return rc;
    }
    a.M = Mm;
    a.N = Nm;
    if (force_id != 0) return launch_by_id<T, TA>(force_id, a, batch, stream);   // the caller's tile
    const ProductPlan plan = plan_product(sizeof(T) == 8, TA, Mm, Nm, K, batch, a.accumulate != 0);
    if (plan.split == 0) return launch_by_id<T, TA>(plan.main.id, a, batch, stream);
    ContractArgs<T> first = a, second = a;
    if (plan.split == 1) {
        first.M = plan.cut;
        second.M = Mm - plan.cut;
        second.A += TA ? plan.cut : plan.cut * lda;
        second.C += plan.cut * ldc;
    } else {
        first.N = plan.cut;
        second.N = Nm - plan.cut;
        second.B += plan.cut;
        second.C += plan.cut;
        second.n_before = plan.cut;
    }
    const int rc = launch_by_id<T, TA>(plan.main.id, first, batch, stream);
    return rc != DISTAL_OK ? rc : launch_by_id<T, TA>(plan.rest.id, second, batch, stream);
}

// The product cut along k (plan_split_k): parts of kchunk terms as one batch into the slabs of
// the scratch W, a shorter last part on its own, then the sum of the slabs onto C.
template <typename T>
int gemm_splitk_t(int64_t M, int64_t N, int64_t K, const T *A, int64_t lda, const T *B, int64_t ldb, T *C,
                  int64_t ldc, int accumulate, T *W, const SplitKPlan &p, hipStream_t stream) {
    const int64_t slab = M * N, whole = K / p.kchunk, rest = K - whole * p.kchunk;   // whole parts, and a shorter last one
    int rc = gemm_t<T>(M, N, p.kchunk, A, lda, B, ldb, W, N, 0, stream, whole, p.kchunk, p.kchunk * ldb, slab);
    if (rc != DISTAL_OK) return rc;
    if (rest > 0) {
        rc = gemm_t<T>(M, N, rest, A + whole * p.kchunk, lda, B + whole * p.kchunk * ldb, ldb, W + whole * slab, N, 0, stream);
        if (rc != DISTAL_OK) return rc;
    }
    int64_t blocks = (slab + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(splitk_sum_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, stream, (const T *)W, (int)p.parts, M, N, C,
                       ldc, accumulate ? 1 : 0);
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

// TTM over the last mode with the factor held in registers (ttm_slices_per_wave says where).
template <typename T, int NS, bool RAGGED>
int launch_ttm_slices_form(const TtmSlicesArgs<T> &a, hipStream_t stream) {
    typedef TtmSlicesCfg<T, NS> Cfg;
    static std::atomic<bool> done[kMaxDevices];
    auto kern = ttm_slices_kernel<T, NS, RAGGED>;
    if (!allow_lds(kern, Cfg::LDS_BYTES, done)) return DISTAL_ERR_LAUNCH;
    const int64_t grid = a.rblocks < kComputeUnits ? a.rblocks : kComputeUnits;      // one workgroup per compute unit
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Cfg::NT), Cfg::LDS_BYTES, stream, a);
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

template <typename T>
int ttm_slices_t(int ns, int64_t R, int64_t K, int64_t L, const T *B, const T *C, T *A, hipStream_t stream) {
    const bool kwhole = K == (int64_t)8 * ns * MttkrpCfg<T>::SL;
    // whole slices: the straight-line form on the whole blocks of 32 rows, the last R % 32 rows as a
    // small tiled product; a short last slice: the ragged form on all rows
    const int64_t Rk = kwhole ? R - R % 32 : R;
    TtmSlicesArgs<T> a{B, C, A, Rk, K, L, (Rk + 31) / 32};
    int rc;
    switch (ns) {
    case 1: rc = kwhole ? launch_ttm_slices_form<T, 1, false>(a, stream) : launch_ttm_slices_form<T, 1, true>(a, stream); break;
    case 2: rc = kwhole ? launch_ttm_slices_form<T, 2, false>(a, stream) : launch_ttm_slices_form<T, 2, true>(a, stream); break;
    case 3: rc = kwhole ? launch_ttm_slices_form<T, 3, false>(a, stream) : DISTAL_ERR_SHAPE; break;   // never planned: the ragged forms spill
    case 4: rc = kwhole ? launch_ttm_slices_form<T, 4, false>(a, stream) : DISTAL_ERR_SHAPE; break;
    default: rc = DISTAL_ERR_SHAPE;
    }
    if (rc != DISTAL_OK || Rk == R) return rc;
    return gemm_t<T>(R - Rk, L, K, B + Rk * K, K, C, L, A + Rk * L, L, 0, stream);
}

int check_dtype(int dt) { return (dt == DISTAL_F32 || dt == DISTAL_F64) ? DISTAL_OK : DISTAL_ERR_DTYPE; }

size_t elem_size(int dt) { return dt == DISTAL_F64 ? 8 : 4; }

// ---- MTTKRP ---------------------------------------------------------------
// Every workgroup gets a fixed piece of the output rows and of one summed index, and a
// contiguous range of the other summed index (j for mode 0, i for modes 1 and 2).  The number
// of ranges is a function of the shape only (enough workgroups for three per CU of a 256-CU
// part), never of the device, so the summation order is reproducible across devices.
// Workspace: one partial row of L values per (output row, range, piece), none when that is
// one row per output row.
// vec: whole aligned k-slices (vector loads); full: every block of output rows and columns is whole
template <typename T, int LT>
int launch_walk(const MttkrpWalkArgs<T> &a, unsigned nblocks, bool vec, bool full, hipStream_t stream) {
    typedef MttkrpCfg<T> Cfg;
    constexpr int lds = Cfg::LDS_BYTES;
    static std::atomic<bool> done[3][kMaxDevices];
    if (full) {
        auto kern = mttkrp_walk_kernel<T, false, false, LT>;
        if (!allow_lds(kern, lds, done[0])) return DISTAL_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(nblocks), dim3(Cfg::NT), lds, stream, a);
    } else if (vec) {
        auto kern = mttkrp_walk_kernel<T, false, true, LT>;
        if (!allow_lds(kern, lds, done[1])) return DISTAL_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(nblocks), dim3(Cfg::NT), lds, stream, a);
    } else {
        auto kern = mttkrp_walk_kernel<T, true, true, LT>;
        if (!allow_lds(kern, lds, done[2])) return DISTAL_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(nblocks), dim3(Cfg::NT), lds, stream, a);
    }
    return DISTAL_OK;
}

template <typename T, int LT>
void launch_mode2(const MttkrpMode2Args<T> &a, unsigned nblocks, bool aligned, hipStream_t stream) {
    typedef MttkrpMode2Cfg<T, LT> Cfg;
    const dim3 grid(nblocks), block(Cfg::NT);
    const bool vec = aligned && a.K % Cfg::VEC == 0;
    if (vec && a.K % Cfg::KW == 0 && a.J % Cfg::JB == 0 && a.L % Cfg::BN == 0)
        hipLaunchKernelGGL((mttkrp_mode2_kernel<T, false, false, LT>), grid, block, Cfg::LDS_BYTES, stream, a);
    else if (vec)
        hipLaunchKernelGGL((mttkrp_mode2_kernel<T, false, true, LT>), grid, block, Cfg::LDS_BYTES, stream, a);
    else
        hipLaunchKernelGGL((mttkrp_mode2_kernel<T, true, true, LT>), grid, block, Cfg::LDS_BYTES, stream, a);
}

template <typename T>
int mttkrp_mode_t(int mode, int64_t I, int64_t J, int64_t K, int64_t L, const T *B, const T *C, const T *D,
                  T *A, void *workspace, hipStream_t stream) {
    const int64_t out_rows = mode == 0 ? I : (mode == 1 ? J : K);
    if (out_rows == 0 || L == 0) return DISTAL_OK;
    if (I == 0 || J == 0 || K == 0) return launch_fill<T>(A, out_rows, L, L, stream);
    const MttkrpModePlan plan = mttkrp_mode_plan(sizeof(T) == 8 ? DISTAL_F64 : DISTAL_F32, mode, I, J, K, L);
    if (!plan.ok) return DISTAL_ERR_SHAPE;
    T *partial = plan.nparts == 1 ? A : static_cast<T *>(workspace);
    const unsigned nblocks = (unsigned)(plan.tasks * plan.nsplit);
    // the vector kernels need 16-byte aligned rows of B (an aligned base, K a multiple of the vector);
    // everything else may be ragged
    const bool aligned = aligned16(B);
    if (mode != 2) {
        typedef MttkrpCfg<T> Cfg;
        MttkrpWalkArgs<T> a{};
        a.B = B; a.F = C; a.D = D; a.partial = partial;
        a.K = K; a.L = L;
        int64_t jk;
        if (!mul_ok(J, K, &jk)) return DISTAL_ERR_SHAPE;
        if (mode == 0) { a.R = I; a.W = J; a.row_stride = jk; a.walk_stride = K; }
        else           { a.R = J; a.W = I; a.row_stride = K;  a.walk_stride = jk; }
        a.wsplit = plan.isplit; a.nsplit = (int)plan.nsplit;
        a.nslices = (int)plan.nslices; a.spw = (int)plan.spw; a.kgroups = (int)plan.kgroups;
        a.tiles_n = (int)plan.tiles_n; a.rblocks = (int)plan.rblocks; a.rgroups = (int)plan.rgroups;
        const bool vec = aligned && K % Cfg::VEC == 0, whole = vec && K % Cfg::SL == 0 && a.R % Cfg::RB == 0;
        const int rc = L > 32 ? launch_walk<T, 2>(a, nblocks, vec, whole && L % (2 * Cfg::BN) == 0, stream)
                              : launch_walk<T, 1>(a, nblocks, vec, whole && L % Cfg::BN == 0, stream);
        if (rc != DISTAL_OK) return rc;
    } else {
        MttkrpMode2Args<T> a{};
        a.B = B; a.C = C; a.D = D; a.partial = partial;
        a.I = I; a.J = J; a.K = K; a.L = L;
        a.isplit = plan.isplit; a.nsplit = (int)plan.nsplit;
        a.jgroups = (int)plan.jgroups; a.kblocks = (int)plan.kblocks; a.tiles_n = (int)plan.tiles_n;
        if (L > 32) launch_mode2<T, 2>(a, nblocks, aligned, stream);
        else launch_mode2<T, 1>(a, nblocks, aligned, stream);
    }
    if (hipGetLastError() != hipSuccess) return DISTAL_ERR_LAUNCH;
    if (plan.nparts == 1) return DISTAL_OK;
    const int64_t blocks = out_rows < 4096 ? out_rows : 4096;
    hipLaunchKernelGGL(mttkrp_reduce_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<const T *>(partial), A, out_rows, L, (int)plan.nparts);
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

// ---- TTV ------------------------------------------------------------------
// ttv_row_kernel with RW * PU = 8 loads per lane in flight and a contiguous range of rows per
// workgroup; K / VEC must be a multiple of 64 * PU.
template <typename T, int RW, int PU>
int launch_ttv_rows(int64_t rows, int64_t K, const T *B, const T *c, T *A, hipStream_t stream) {
    constexpr int VEC = 16 / (int)sizeof(T);
    if (K % VEC != 0 || (K / VEC) % (64 * PU) != 0) return DISTAL_ERR_SHAPE;   // the kernel reads whole steps only
    const RangeSplit r = split_ranges(rows, kStreamBlocks, 1, 4 * RW);   // four wavefronts of RW rows per step
    hipLaunchKernelGGL((ttv_row_kernel<T, RW, PU>), dim3((unsigned)r.blocks), dim3(256), 0, stream, B, c, A, rows, K, r.per);
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

template <typename T>
int ttv_t(int64_t rows, int64_t K, const T *B, const T *c, T *A, hipStream_t stream) {
    constexpr int VEC = 16 / (int)sizeof(T);
    if (rows == 0) return DISTAL_OK;
    if (K == 0) return launch_fill<T>(A, rows, 1, 1, stream);
    // one 16-row group per workgroup; very large grids fall back to the grid-stride loop
    int64_t blocks = (rows + 15) / 16;
    if (blocks > (1 << 22)) blocks = 1 << 22;
    const bool vec = aligned16(B) && aligned16(c) && K % VEC == 0;
    if (!vec) {
        // odd K or operands off a 16-byte boundary: rows of at least 16 pieces take the vector kernel
        // with element-aligned loads, shorter ones the element-wise kernel
        if (K >= 16 * VEC)
            hipLaunchKernelGGL((ttv_vec_kernel<T, 8, false, true>), dim3((unsigned)blocks), dim3(256), 0, stream, B, c, A, rows, K);
        else
            hipLaunchKernelGGL(ttv_generic_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, stream, B, c, A, rows, K);
    } else if (K / VEC <= 16) {
        // short rows: eight rows per 16-lane group and trip, so a workgroup streams 128 rows
        int64_t b8 = (rows + 127) / 128;
        if (b8 > (1 << 22)) b8 = 1 << 22;
        hipLaunchKernelGGL((ttv_short_kernel<T, 8>), dim3((unsigned)b8), dim3(256), 0, stream, B, c, A, rows, K);
    } else if (rows >= 8192 && (K / VEC) % 256 == 0) {
        // many rows of whole 4 KiB runs: whole rows per wavefront, a contiguous range of rows per
        // workgroup and one workgroup per compute unit (1 to 16 % faster than the grid below)
        // 8 KiB rows: one row per wavefront and step; others (4 KiB; 12 KiB and longer): two rows of
        // four pieces (16 KiB rows: 6.98 TB/s against 6.37 with one row of eight)
        if (K / VEC == 512) return launch_ttv_rows<T, 1, 8>(rows, K, B, c, A, stream);
        return launch_ttv_rows<T, 2, 4>(rows, K, B, c, A, stream);
    } else if (sizeof(T) == 4 && rows >= 8192 && (K / VEC) % 128 == 0 && K * (int64_t)sizeof(T) <= 16 * 1024) {
        // binary32 rows of whole 2 KiB runs: the same with four rows per wavefront (+5 %; binary64
        // rows of 2 KiB lose 5 % and stay with the grid below)
        return launch_ttv_rows<T, 4, 2>(rows, K, B, c, A, stream);
    } else if (rows >= 1024 && rows < 8192 && (K / VEC) % 512 == 0 && K * (int64_t)sizeof(T) >= 64 * 1024) {
        // a thousand or more long rows: one whole row per wavefront at a time, four rows per workgroup
        return launch_ttv_rows<T, 1, 8>(rows, K, B, c, A, stream);
    } else if (rows < 8192 && K * (int64_t)sizeof(T) >= 64 * 1024) {
        // too few rows to fill the chip with 16 per workgroup: one workgroup per row
        hipLaunchKernelGGL((ttv_wide_kernel<T, 8>), dim3((unsigned)rows), dim3(256), 0, stream, B, c, A, rows, K);
    } else if (K * (int64_t)sizeof(T) <= 32 * 1024) {
        // trips of 16 pieces per lane where rows are made of such trips, else of 8 (less of a row is
        // then left to the short predicated trips)
        if ((K / VEC) % 256 == 0)
            hipLaunchKernelGGL((ttv_vec_kernel<T, 16, true>), dim3((unsigned)blocks), dim3(256),
                               (size_t)K * sizeof(T), stream, B, c, A, rows, K);
        else
            hipLaunchKernelGGL((ttv_vec_kernel<T, 8, true>), dim3((unsigned)blocks), dim3(256),
                               (size_t)K * sizeof(T), stream, B, c, A, rows, K);
    } else {
        hipLaunchKernelGGL((ttv_vec_kernel<T, 8, false>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           B, c, A, rows, K);
    }
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

// out(b, n) = sum_r c(r) * B(b, r, n): TTV along mode 0 (batch 1, r = i, n = (j,k)) or 1 (b = i, r = j, n = k)
template <typename T>
int ttv_left_t(int64_t batch, int64_t R, int64_t N, const T *B, const T *c, T *A, hipStream_t stream) {
    constexpr int VEC = 16 / (int)sizeof(T);
    int64_t total;
    if (!mul_ok(batch, N, &total)) return DISTAL_ERR_SHAPE;
    if (total == 0) return DISTAL_OK;
    if (R == 0) return launch_fill<T>(A, 1, total, total, stream);
    // 16-byte pieces of the output row: aligned ones, or - any N >= VEC, any alignment - the same
    // accesses typed as element-aligned with a last piece that overlaps its neighbour
    const bool al = aligned16(B) && aligned16(A) && N % VEC == 0;
    const bool vec = al || N >= VEC;
    const int64_t np = vec ? (N + VEC - 1) / VEC : N;
    int64_t work;
    if (!mul_ok(batch, np, &work)) return DISTAL_ERR_SHAPE;
    int64_t blocks = (work + 255) / 256;
    if (blocks > (1 << 22)) blocks = 1 << 22;
    // Rows far apart (a whole slice per step of r) stream best when a workgroup reads 16 KiB
    // of each row in one go; needs that many whole spans to give every compute unit one.
    constexpr int64_t kWideSpan = 4 * 256 * VEC;
    const int64_t wide_groups = (al && N % kWideSpan == 0) ? total / kWideSpan : 0;
    const dim3 wg(256);
    if (blocks < kComputeUnits && R >= 64) {
        // fewer outputs than give every compute unit a workgroup, many rows to add: the rows are split
        // inside a workgroup.  16 lanes per 256-byte run of a row and 16 row groups where that gives
        // every compute unit a workgroup, else 8 lanes and 32 groups (4 lanes and 64-byte runs
        // measured slower than leaving compute units idle)
        const int64_t g16 = batch * ((np + 15) / 16), g8 = batch * ((np + 7) / 8), g32 = batch * ((np + 31) / 32);
        const int64_t cap = 1 << 20;
        const dim3 d16((unsigned)(g16 < cap ? g16 : cap)), d8((unsigned)(g8 < cap ? g8 : cap)), d32((unsigned)(g32 < cap ? g32 : cap));
        if (vec && g16 >= kComputeUnits) {
            if (al) hipLaunchKernelGGL((ttv_left_split_kernel<T, VEC, 16, 4>), d16, wg, 0, stream, B, c, A, batch, R, N);
            else hipLaunchKernelGGL((ttv_left_split_kernel<T, VEC, 16, 4, true>), d16, wg, 0, stream, B, c, A, batch, R, N);
        } else if (vec) {
            if (al) hipLaunchKernelGGL((ttv_left_split_kernel<T, VEC, 8, 4>), d8, wg, 0, stream, B, c, A, batch, R, N);
            else hipLaunchKernelGGL((ttv_left_split_kernel<T, VEC, 8, 4, true>), d8, wg, 0, stream, B, c, A, batch, R, N);
        } else {
            hipLaunchKernelGGL((ttv_left_split_kernel<T, 1, 32, 4>), d32, wg, 0, stream, B, c, A, batch, R, N);
        }
    } else if (wide_groups >= 256) {
        hipLaunchKernelGGL((ttv_left_wide_kernel<T, 4, 4>),
                           dim3((unsigned)(wide_groups < (1 << 22) ? wide_groups : (1 << 22))), wg, 0,
                           stream, B, c, A, batch, R, N);
    } else if (vec) {
        // long walks over many output pieces: one workgroup per compute unit, each taking several
        // 4 KiB column strips in turn (1024^3 along mode 1: +1 % in binary32, +4 % in binary64)
        if (blocks >= 4 * kStreamBlocks && R >= 256) blocks = kStreamBlocks;
        if (al) hipLaunchKernelGGL((ttv_left_vec_kernel<T, 8>), dim3((unsigned)blocks), wg, 0, stream, B, c, A, batch, R, N);
        else hipLaunchKernelGGL((ttv_left_vec_kernel<T, 8, true>), dim3((unsigned)blocks), wg, 0, stream, B, c, A, batch, R, N);
    } else {
        hipLaunchKernelGGL(ttv_left_generic_kernel<T>, dim3((unsigned)blocks), wg, 0, stream, B, c, A, batch, R, N);
    }
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

// ---- innerprod ------------------------------------------------------------
template <typename T>
int innerprod_t(int64_t n, const T *B, const T *C, T *out, double *partial, hipStream_t stream) {
    constexpr int VEC = 16 / (int)sizeof(T);
    int nparts = 0;
    int64_t tail_lo = 0;
    if (n > 0) {
        // 16-byte pieces counted from each operand's own start; operands that do not start on a
        // 16-byte boundary (views) take the same loads typed as element-aligned
        const int64_t nvec = n / VEC;
        if (nvec > 0) {
            const RangeSplit r = split_ranges(nvec, kStreamBlocks, 256, 256);
            if (aligned16(B) && aligned16(C))
                hipLaunchKernelGGL((innerprod_pass1_kernel<T, 4>), dim3((unsigned)r.blocks), dim3(256), 0, stream,
                                   B, C, partial, nvec, r.per);
            else
                hipLaunchKernelGGL((innerprod_pass1_kernel<T, 4, true>), dim3((unsigned)r.blocks), dim3(256), 0, stream,
                                   B, C, partial, nvec, r.per);
            if (hipGetLastError() != hipSuccess) return DISTAL_ERR_LAUNCH;
            nparts = (int)r.blocks;
        }
        tail_lo = nvec * VEC;
    }
    hipLaunchKernelGGL(innerprod_pass2_kernel<T>, dim3(1), dim3(256), 0, stream,
                       (const double *)partial, nparts, B, C, tail_lo, n, out);
    return hipGetLastError() == hipSuccess ? DISTAL_OK : DISTAL_ERR_LAUNCH;
}

// ---- library-owned scratch for the entry point that allocates nothing ------
// One array per device, inside the code object: the partial sums of distal_innerprod_noalloc.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels and every
// other device-side use take the address that call returns, looked up once per device.
constexpr size_t kScratchBytes = (size_t)kInnerprodMaxBlocks * sizeof(double);
}  // namespace
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
namespace {
std::atomic<void *> scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (NULL if the runtime refuses).
void *scratch_of_current_device() {
    int d = -1;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
    void *p = scratch_ptr[d].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
    scratch_ptr[d].store(p, std::memory_order_release);   // every thread finds the same address
    return p;
}

bool tensor_elems(int64_t I, int64_t J, int64_t K, int64_t *n) {
    int64_t ij;
    // keep byte offsets inside int64 as well
    return mul_ok(I, J, &ij) && mul_ok(ij, K, n) && *n <= std::numeric_limits<int64_t>::max() / 8;
}

}  // namespace

extern "C" {

int distal_version(void) { return 600; }   // 0.6.0

const char *distal_status_string(int status) {
    switch (status) {
        case DISTAL_OK: return "ok";
        case DISTAL_ERR_NULL: return "a required pointer is NULL";
        case DISTAL_ERR_SHAPE: return "negative or overflowing extent";
        case DISTAL_ERR_DTYPE: return "unknown dtype";
        case DISTAL_ERR_STRIDE: return "leading dimension smaller than the row length";
        case DISTAL_ERR_ALIAS: return "output aliases an input";
        case DISTAL_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case DISTAL_ERR_LAUNCH: return "kernel launch failed";
        case DISTAL_ERR_MODE: return "mode is not 0, 1 or 2";
        default: return "unknown status";
    }
}

int distal_gemm(distal_dtype dt, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                const void *B, int64_t ldb, void *C, int64_t ldc, int accumulate, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (M < 0 || N < 0 || K < 0) return DISTAL_ERR_SHAPE;
    int64_t t;
    if (!mul_ok(M, N, &t) || !mul_ok(M, K, &t) || !mul_ok(K, N, &t)) return DISTAL_ERR_SHAPE;
    if (lda < K || ldb < N || ldc < N) return DISTAL_ERR_STRIDE;
    if ((M > 1 && (!mul_ok(M, lda, &t) || !mul_ok(M, ldc, &t) || t > INT64_MAX / 8)) ||
        (K > 1 && (!mul_ok(K, ldb, &t) || t > INT64_MAX / 8)))
        return DISTAL_ERR_SHAPE;
    const bool need_a = M > 0 && K > 0 && N > 0, need_b = need_a, need_c = M > 0 && N > 0;
    if ((need_a && !A) || (need_b && !B) || (need_c && !C)) return DISTAL_ERR_NULL;
    if (need_c && (C == A || C == B)) return DISTAL_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == DISTAL_F64)
        return gemm_t<double>(M, N, K, (const double *)A, lda, (const double *)B, ldb, (double *)C, ldc,
                              accumulate, s);
    return gemm_t<float>(M, N, K, (const float *)A, lda, (const float *)B, ldb, (float *)C, ldc,
                         accumulate, s);
}

size_t distal_gemm_workspace_bytes(distal_dtype dt, int64_t M, int64_t N, int64_t K) {
    int64_t t;
    if (check_dtype(dt) != DISTAL_OK || M <= 0 || N <= 0 || K <= 0 || !mul_ok(M, N, &t)) return 0;
    const SplitKPlan p = plan_split_k(dt == DISTAL_F64, M, N, K);
    if (p.parts < 2 || !mul_ok(t, p.parts, &t) || t > (int64_t)(SIZE_MAX / 16)) return 0;
    return (size_t)t * elem_size(dt);
}

int distal_gemm_ws(distal_dtype dt, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                   int64_t ldb, void *C, int64_t ldc, int accumulate, void *workspace, size_t workspace_bytes,
                   void *stream) {
    const size_t need = distal_gemm_workspace_bytes(dt, M, N, K);
    if (need == 0) return distal_gemm(dt, M, N, K, A, lda, B, ldb, C, ldc, accumulate, stream);
    // need > 0: the extents are positive and their products fit; the other checks of distal_gemm
    if (lda < K || ldb < N || ldc < N) return DISTAL_ERR_STRIDE;
    int64_t t;
    if ((M > 1 && (!mul_ok(M, lda, &t) || !mul_ok(M, ldc, &t) || t > INT64_MAX / 8)) ||
        (K > 1 && (!mul_ok(K, ldb, &t) || t > INT64_MAX / 8)))
        return DISTAL_ERR_SHAPE;
    if (!A || !B || !C) return DISTAL_ERR_NULL;
    if (C == A || C == B) return DISTAL_ERR_ALIAS;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) % kWorkspaceAlign) != 0)
        return DISTAL_ERR_WORKSPACE;
    if (workspace == A || workspace == B || workspace == C) return DISTAL_ERR_ALIAS;
    const SplitKPlan p = plan_split_k(dt == DISTAL_F64, M, N, K);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == DISTAL_F64)
        return gemm_splitk_t<double>(M, N, K, (const double *)A, lda, (const double *)B, ldb, (double *)C, ldc, accumulate,
                                     (double *)workspace, p, s);
    return gemm_splitk_t<float>(M, N, K, (const float *)A, lda, (const float *)B, ldb, (float *)C, ldc, accumulate,
                                (float *)workspace, p, s);
}

int distal_gemm_tiled(distal_dtype dt, int transposed_left, int bm, int bn, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc,
                      int accumulate, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (M < 0 || N < 0 || K < 0) return DISTAL_ERR_SHAPE;
    // the tile must be one the dtype has kernels for, whatever the extents make eligible
    TileCandidate cand[kMaxTileCandidates];
    const int n = tile_candidates(dt == DISTAL_F64, transposed_left != 0, 1, 1, K, cand);
    int id = 0;
    for (int i = 0; i < n; ++i)            // of two slab depths of one tile, the one this K is deep enough for
        if (cand[i].bm == bm && cand[i].bn == bn && (id == 0 || cand[i].eligible)) id = cand[i].id;
    if (id == 0) return DISTAL_ERR_SHAPE;
    int64_t t;
    if (!mul_ok(M, N, &t) || !mul_ok(M, K, &t) || !mul_ok(K, N, &t)) return DISTAL_ERR_SHAPE;
    const int64_t a_rows = transposed_left ? K : M, a_cols = transposed_left ? M : K;
    if (lda < a_cols || ldb < N || ldc < N) return DISTAL_ERR_STRIDE;
    if ((a_rows > 1 && (!mul_ok(a_rows, lda, &t) || t > INT64_MAX / 8)) ||
        (M > 1 && (!mul_ok(M, ldc, &t) || t > INT64_MAX / 8)) ||
        (K > 1 && (!mul_ok(K, ldb, &t) || t > INT64_MAX / 8)))
        return DISTAL_ERR_SHAPE;
    const bool need_in = M > 0 && K > 0 && N > 0, need_c = M > 0 && N > 0;
    if ((need_in && (!A || !B)) || (need_c && !C)) return DISTAL_ERR_NULL;
    if (need_c && (C == A || C == B)) return DISTAL_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == DISTAL_F64) {
        if (transposed_left)
            return gemm_t<double, true>(M, N, K, (const double *)A, lda, (const double *)B, ldb, (double *)C, ldc,
                                        accumulate, s, 1, 0, 0, 0, id);
        return gemm_t<double>(M, N, K, (const double *)A, lda, (const double *)B, ldb, (double *)C, ldc,
                              accumulate, s, 1, 0, 0, 0, id);
    }
    if (transposed_left)
        return gemm_t<float, true>(M, N, K, (const float *)A, lda, (const float *)B, ldb, (float *)C, ldc,
                                   accumulate, s, 1, 0, 0, 0, id);
    return gemm_t<float>(M, N, K, (const float *)A, lda, (const float *)B, ldb, (float *)C, ldc,
                         accumulate, s, 1, 0, 0, 0, id);
}

int distal_ttm(distal_dtype dt, int64_t I, int64_t J, int64_t K, int64_t L, const void *B,
               const void *C, void *A, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (I < 0 || J < 0 || K < 0 || L < 0) return DISTAL_ERR_SHAPE;
    int64_t nb, na, ij, t;
    if (!tensor_elems(I, J, K, &nb) || !tensor_elems(I, J, L, &na) || !mul_ok(K, L, &t) ||
        !mul_ok(I, J, &ij))
        return DISTAL_ERR_SHAPE;
    if ((nb > 0 && L > 0 && !B) || (t > 0 && ij > 0 && !C) || (na > 0 && !A)) return DISTAL_ERR_NULL;
    if (na > 0 && (A == B || A == C)) return DISTAL_ERR_ALIAS;
    // The contraction over the last mode is one matrix product on the (I*J) x K view.
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t ldk = K > 0 ? K : 1, ldl = L > 0 ? L : 1;
    // a rank-sized factor on a long tensor: the factor stays in registers, the tensor streams by
    const int ns = aligned16(B) ? ttm_slices_per_wave(dt == DISTAL_F64, ij, K, L) : 0;
    if (ns != 0) {
        if (dt == DISTAL_F64) return ttm_slices_t<double>(ns, ij, K, L, (const double *)B, (const double *)C, (double *)A, s);
        return ttm_slices_t<float>(ns, ij, K, L, (const float *)B, (const float *)C, (float *)A, s);
    }
    if (dt == DISTAL_F64)
        return gemm_t<double>(ij, L, K, (const double *)B, ldk, (const double *)C, ldl, (double *)A, ldl, 0, s);
    return gemm_t<float>(ij, L, K, (const float *)B, ldk, (const float *)C, ldl, (float *)A, ldl, 0, s);
}

int distal_ttm_mode(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K, int64_t R, const void *B,
                    const void *C, void *A, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (mode < 0 || mode > 2) return DISTAL_ERR_MODE;
    if (mode == 2) return distal_ttm(dt, I, J, K, R, B, C, A, stream);
    if (I < 0 || J < 0 || K < 0 || R < 0) return DISTAL_ERR_SHAPE;
    const int64_t X = mode == 0 ? I : J;                    // the contracted extent
    int64_t nb, na, nc, jk;
    if (!tensor_elems(I, J, K, &nb) || !mul_ok(J, K, &jk) || !mul_ok(X, R, &nc) ||
        !tensor_elems(mode == 0 ? R : I, mode == 0 ? J : R, K, &na))
        return DISTAL_ERR_SHAPE;
    if ((nb > 0 && R > 0 && !B) || (nc > 0 && na > 0 && !C) || (na > 0 && !A)) return DISTAL_ERR_NULL;
    if (na > 0 && (A == B || A == C)) return DISTAL_ERR_ALIAS;
    if (na == 0) return DISTAL_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f64 = dt == DISTAL_F64;
    if (X == 0)   // empty sum: the whole (contiguous) output is zero
        return f64 ? launch_fill<double>((double *)A, 1, na, na, s) : launch_fill<float>((float *)A, 1, na, na, s);
    const int64_t ldr = R > 0 ? R : 1;
    if (mode == 0) {
        // A(r, jk) = sum_i C(i, r) * B(i, jk): one product with the left operand stored I x R
        if (f64)
            return gemm_t<double, true>(R, jk, I, (const double *)C, ldr, (const double *)B, jk, (double *)A, jk, 0, s);
        return gemm_t<float, true>(R, jk, I, (const float *)C, ldr, (const float *)B, jk, (float *)A, jk, 0, s);
    }
    // mode 1: for every i, A_i(r, k) = sum_j C(j, r) * B_i(j, k): a batch of I products sharing C
    int64_t rk;
    if (!mul_ok(R, K, &rk)) return DISTAL_ERR_SHAPE;
    if (f64)
        return gemm_t<double, true>(R, K, J, (const double *)C, ldr, (const double *)B, K, (double *)A, K, 0, s,
                                    I, 0, jk, rk);
    return gemm_t<float, true>(R, K, J, (const float *)C, ldr, (const float *)B, K, (float *)A, K, 0, s,
                               I, 0, jk, rk);
}

size_t distal_mttkrp_mode_workspace_bytes(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K,
                                          int64_t L) {
    if (check_dtype(dt) != DISTAL_OK || mode < 0 || mode > 2 || I < 0 || J < 0 || K < 0 || L < 0) return 0;
    if (I == 0 || J == 0 || K == 0 || L == 0) return 0;
    const MttkrpModePlan p = mttkrp_mode_plan(dt, mode, I, J, K, L);
    if (!p.ok) return 0;
    return (size_t)p.partial_elems * elem_size(dt);
}

int distal_mttkrp_mode(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K, int64_t L,
                       const void *B, const void *C, const void *D, void *A, void *workspace,
                       size_t workspace_bytes, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (mode < 0 || mode > 2) return DISTAL_ERR_MODE;
    if (I < 0 || J < 0 || K < 0 || L < 0) return DISTAL_ERR_SHAPE;
    // factor extents: C belongs to mode i, D to k (mode 1) or j (mode 2); the output to the mode itself
    const int64_t crows = mode == 0 ? J : I, drows = mode == 2 ? J : K;
    const int64_t arows = mode == 0 ? I : (mode == 1 ? J : K);
    int64_t nb, nc, nd, na;
    if (!tensor_elems(I, J, K, &nb) || !mul_ok(crows, L, &nc) || !mul_ok(drows, L, &nd) || !mul_ok(arows, L, &na))
        return DISTAL_ERR_SHAPE;
    const bool work = nb > 0 && L > 0;
    if (work && !mttkrp_mode_plan(dt, mode, I, J, K, L).ok) return DISTAL_ERR_SHAPE;
    if ((work && (!B || !C || !D)) || (na > 0 && !A)) return DISTAL_ERR_NULL;
    if (na > 0 && (A == B || A == C || A == D)) return DISTAL_ERR_ALIAS;
    const size_t need = work ? distal_mttkrp_mode_workspace_bytes(dt, mode, I, J, K, L) : 0;
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) % kWorkspaceAlign) != 0))
        return DISTAL_ERR_WORKSPACE;
    if (need > 0 && (workspace == A || workspace == B || workspace == C || workspace == D))
        return DISTAL_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == DISTAL_F64)
        return mttkrp_mode_t<double>(mode, I, J, K, L, (const double *)B, (const double *)C, (const double *)D,
                                     (double *)A, workspace, s);
    return mttkrp_mode_t<float>(mode, I, J, K, L, (const float *)B, (const float *)C, (const float *)D,
                                (float *)A, workspace, s);
}

size_t distal_mttkrp_workspace_bytes(distal_dtype dt, int64_t I, int64_t J, int64_t K, int64_t L) {
    return distal_mttkrp_mode_workspace_bytes(dt, 0, I, J, K, L);
}

int distal_mttkrp(distal_dtype dt, int64_t I, int64_t J, int64_t K, int64_t L, const void *B,
                  const void *C, const void *D, void *A, void *workspace, size_t workspace_bytes,
                  void *stream) {
    return distal_mttkrp_mode(dt, 0, I, J, K, L, B, C, D, A, workspace, workspace_bytes, stream);
}

int distal_ttv(distal_dtype dt, int64_t I, int64_t J, int64_t K, const void *B, const void *c,
               void *A, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (I < 0 || J < 0 || K < 0) return DISTAL_ERR_SHAPE;
    int64_t nb, rows;
    if (!tensor_elems(I, J, K, &nb) || !mul_ok(I, J, &rows)) return DISTAL_ERR_SHAPE;
    if ((nb > 0 && (!B || !c)) || (rows > 0 && !A)) return DISTAL_ERR_NULL;
    if (rows > 0 && (A == B || A == c)) return DISTAL_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == DISTAL_F64) return ttv_t<double>(rows, K, (const double *)B, (const double *)c, (double *)A, s);
    return ttv_t<float>(rows, K, (const float *)B, (const float *)c, (float *)A, s);
}

int distal_gemm_plan(distal_dtype dt, int transposed_left, int64_t M, int64_t N, int64_t K, int64_t batch, int accumulate,
                     int tile[3], int *split, int64_t *cut, int rest_tile[3]) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (M <= 0 || N <= 0 || K <= 0 || batch <= 0) return DISTAL_ERR_SHAPE;
    if (!tile || !split || !cut || !rest_tile) return DISTAL_ERR_NULL;
    int64_t tiles;
    if (!mul_ok((M + 127) / 128, (N + 127) / 128, &tiles) || tiles > std::numeric_limits<int>::max())
        return DISTAL_ERR_SHAPE;
    const ProductPlan p = plan_product(dt == DISTAL_F64, transposed_left != 0, M, N, K, batch, accumulate != 0);
    tile[0] = p.main.bm; tile[1] = p.main.bn; tile[2] = p.main.bk;
    *split = p.split;
    *cut = p.cut;
    rest_tile[0] = p.rest.bm; rest_tile[1] = p.rest.bn; rest_tile[2] = p.rest.bk;
    return DISTAL_OK;
}

int distal_ttm_slices_per_wave(distal_dtype dt, int64_t rows, int64_t K, int64_t L) {
    if (check_dtype(dt) != DISTAL_OK || rows < 0 || K < 0 || L < 0) return 0;
    return ttm_slices_per_wave(dt == DISTAL_F64, rows, K, L);
}

int64_t distal_gemm_peeled_columns(distal_dtype dt, int transposed_left, int64_t M, int64_t N, int64_t K, int64_t batch,
                                   int accumulate) {
    if (check_dtype(dt) != DISTAL_OK || M <= 0 || N <= 0 || K <= 0 || batch <= 0) return -1;
    int64_t tiles;
    if (!mul_ok((M + 127) / 128, (N + 127) / 128, &tiles) || tiles > std::numeric_limits<int>::max()) return -1;
    return peeled_columns(dt == DISTAL_F64, transposed_left != 0, M, N, K, batch, accumulate != 0);
}

size_t distal_innerprod_workspace_bytes(distal_dtype dt, int64_t I, int64_t J, int64_t K) {
    int64_t n;
    if (check_dtype(dt) != DISTAL_OK || I < 0 || J < 0 || K < 0 || !tensor_elems(I, J, K, &n)) return 0;
    return (size_t)kInnerprodMaxBlocks * sizeof(double);
}

int distal_ttv_mode(distal_dtype dt, int mode, int64_t I, int64_t J, int64_t K, const void *B, const void *c,
                    void *A, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (mode < 0 || mode > 2) return DISTAL_ERR_MODE;
    if (mode == 2) return distal_ttv(dt, I, J, K, B, c, A, stream);
    if (I < 0 || J < 0 || K < 0) return DISTAL_ERR_SHAPE;
    int64_t nb, na, jk;
    if (!tensor_elems(I, J, K, &nb) || !mul_ok(J, K, &jk) || !mul_ok(mode == 0 ? J : I, K, &na)) return DISTAL_ERR_SHAPE;
    const int64_t X = mode == 0 ? I : J;                    // the contracted extent
    if ((nb > 0 && !B) || (X > 0 && na > 0 && !c) || (na > 0 && !A)) return DISTAL_ERR_NULL;
    if (na > 0 && (A == B || A == c)) return DISTAL_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t batch = mode == 0 ? 1 : I, N = mode == 0 ? jk : K;
    if (dt == DISTAL_F64)
        return ttv_left_t<double>(batch, X, N, (const double *)B, (const double *)c, (double *)A, s);
    return ttv_left_t<float>(batch, X, N, (const float *)B, (const float *)c, (float *)A, s);
}

int distal_innerprod(distal_dtype dt, int64_t I, int64_t J, int64_t K, const void *B, const void *C,
                     void *a, void *workspace, size_t workspace_bytes, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (I < 0 || J < 0 || K < 0) return DISTAL_ERR_SHAPE;
    int64_t n;
    if (!tensor_elems(I, J, K, &n)) return DISTAL_ERR_SHAPE;
    if (!a || (n > 0 && (!B || !C))) return DISTAL_ERR_NULL;
    if (a == B || a == C) return DISTAL_ERR_ALIAS;
    const size_t need = distal_innerprod_workspace_bytes(dt, I, J, K);
    if (!workspace || workspace_bytes < need ||
        (reinterpret_cast<uintptr_t>(workspace) % kWorkspaceAlign) != 0)
        return DISTAL_ERR_WORKSPACE;
    if (workspace == a || workspace == B || workspace == C) return DISTAL_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == DISTAL_F64)
        return innerprod_t<double>(n, (const double *)B, (const double *)C, (double *)a, (double *)workspace, s);
    return innerprod_t<float>(n, (const float *)B, (const float *)C, (float *)a, (double *)workspace, s);
}

int distal_innerprod_noalloc(distal_dtype dt, int64_t I, int64_t J, int64_t K, const void *B, const void *C,
                             void *a, void *stream) {
    if (check_dtype(dt) != DISTAL_OK) return DISTAL_ERR_DTYPE;
    if (I < 0 || J < 0 || K < 0) return DISTAL_ERR_SHAPE;
    int64_t n;
    if (!tensor_elems(I, J, K, &n)) return DISTAL_ERR_SHAPE;
    if (!a || (n > 0 && (!B || !C))) return DISTAL_ERR_NULL;
    if (a == B || a == C) return DISTAL_ERR_ALIAS;
    // the partial sums of this shape must fit the library's array
    if (distal_innerprod_workspace_bytes(dt, I, J, K) > kScratchBytes) return DISTAL_ERR_WORKSPACE;
    void *ws = scratch_of_current_device();
    if (!ws) return DISTAL_ERR_LAUNCH;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // pass 1 writes every partial that pass 2 reads, so nothing of an earlier call is seen
    if (dt == DISTAL_F64)
        return innerprod_t<double>(n, (const double *)B, (const double *)C, (double *)a, (double *)ws, s);
    return innerprod_t<float>(n, (const float *)B, (const float *)C, (float *)a, (double *)ws, s);
}

}  // extern "C"
