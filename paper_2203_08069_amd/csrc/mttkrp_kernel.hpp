// MTTKRP for gfx950 along every mode of the tensor, in one pass over B:
//   mode 0: A(i,l) = sum_j sum_k B(i,j,k) * C(j,l) * D(k,l)
//   mode 1: A(j,l) = sum_i sum_k B(i,j,k) * C(i,l) * D(k,l)
//   mode 2: A(k,l) = sum_i sum_j B(i,j,k) * C(i,l) * D(j,l)
//
// The paper's leaf casts MTTKRP to matrix multiplications followed by an
// element-wise reduction (evaluation section, leaf kernels).  Here the second
// factor matrix is folded INTO one operand of the matrix products (each k-slice of
// D, or each row of D, is scaled by the other factor's entry before it is fed to
// the MFMAs), so the products of all values of the summed non-contiguous index
// accumulate in place in the matrix pipe and no separate reduction pass over an
// intermediate exists.  B is read from HBM exactly once, by fully coalesced
// 16-byte loads (the address unit, not HBM or the matrix pipe, is the first thing
// lane-scattered loads exhaust here).  Every wavefront is an independent stream;
// nothing is atomic and the work split depends on the shape only, so results are
// bitwise reproducible, also across devices.
//
//   mttkrp_walk_kernel   modes 0 and 1 (the MFMA contracts the contiguous index k)
//   mttkrp_mode2_kernel  mode 2 (the output rows are the contiguous index)
//   mttkrp_reduce_kernel adds the partial rows of each output row in a fixed order
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace distal {

template <typename T>
struct MttkrpCfg {
    typedef Mfma<T> MF;
    static constexpr int NT = 256, NW = 4, BN = 32, RB = 32;
    static constexpr int VEC = 16 / (int)sizeof(T);
    static constexpr int SL = 256 / (int)sizeof(T);       // k values per slice
    static constexpr int KV = VEC, KG = MF::KS * KV, NKG = SL / KG;
    static constexpr int MI = RB / MF::NB;                // j blocks (MFMA columns)
    static constexpr int LB = BN / MF::MB;                // l blocks (MFMA rows): 1 (f32) or 2 (f64)
    static constexpr int CPR = SL / VEC;                  // 16-byte pieces per patch row (16)
    static constexpr int RPI = 64 / CPR;                  // rows covered by one wavefront load (4)
    static constexpr int PER_T = RB / RPI;                // loads per lane per block (8)
    static constexpr int LDW = SL + VEC;                  // patch row stride (elements): +16 B
    static constexpr int PATCH = RB * LDW;                // elements per wavefront patch
    static constexpr int LDS_BYTES = NW * PATCH * (int)sizeof(T);
    static_assert(SL % KG == 0 && RB % MF::NB == 0 && LB <= 2 && 64 % CPR == 0, "tile shape");
};

// ---- pieces shared by the kernels of this file --------------------------------------------

// Orders this wavefront's own LDS writes and reads (a patch has one owner).
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Where a lane's 16-byte pieces of a row block sit: piece p is row prow + p*RPI, elements
// pcol .. pcol+VEC-1 of the k-slice.  lane_off is the element offset of piece 0 from the
// block's first element for a tensor whose rows are `row_stride` elements apart; the step
// from piece to piece (RPI rows) is the same for every lane.
template <typename T>
struct MttkrpPieces {
    typedef MttkrpCfg<T> Cfg;
    int prow, pcol;
    int64_t lane_off;
    __device__ __forceinline__ MttkrpPieces(int lane, int64_t row_stride) {
        prow = lane / Cfg::CPR;
        pcol = (lane % Cfg::CPR) * Cfg::VEC;
        lane_off = (int64_t)prow * row_stride + pcol;
    }
};

// RB rows x SL k-values starting at `base` (rows `row_stride` elements apart) -> rs.
// Unguarded: 16-byte vector loads from an aligned base; without RAGGED every block must be full
// (k_valid >= SL, rows_valid >= RB); with it rows past rows_valid re-read the last valid row and
// a last k-slice may be short by whole 16-byte pieces.
// GUARD: rows >= rows_valid and k >= k_valid read as zero, element loads (any alignment).
template <typename T, bool GUARD, bool RAGGED>
__device__ __forceinline__ void mttkrp_load_block(
    const T *base, int64_t row_stride, int64_t rows_valid, int64_t k_valid, const MttkrpPieces<T> &pc,
    typename VecOf<T, MttkrpCfg<T>::VEC>::type (&rs)[MttkrpCfg<T>::PER_T]) {
    typedef MttkrpCfg<T> Cfg;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    if constexpr (!GUARD) {
        if (!RAGGED || (rows_valid >= Cfg::RB && k_valid >= Cfg::SL)) {    // wavefront-uniform: a full block
#pragma unroll
            for (int p = 0; p < Cfg::PER_T; ++p)  // base + p*RPI rows is wavefront-uniform
                rs[p] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(
                    base + (int64_t)(p * Cfg::RPI) * row_stride + pc.lane_off));
        } else {
            // a ragged block: rows past the end re-read the last valid row (what they produce
            // lands in accumulator columns that are never stored); pieces past the end of a
            // short last k-slice (k_valid is a multiple of VEC) are zero
#pragma unroll
            for (int p = 0; p < Cfg::PER_T; ++p) {
                int64_t jr = pc.prow + p * Cfg::RPI;
                if (jr >= rows_valid) jr = rows_valid - 1;
                rs[p] = pc.pcol < k_valid
                            ? __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(base + jr * row_stride + pc.pcol))
                            : vec_t(T(0));
            }
        }
    } else {
#pragma unroll
        for (int p = 0; p < Cfg::PER_T; ++p) {
            const int64_t jr = pc.prow + p * Cfg::RPI;                          // row within the block
#pragma unroll
            for (int e = 0; e < Cfg::VEC; ++e)
                rs[p][e] = (jr < rows_valid && pc.pcol + e < k_valid) ? base[jr * row_stride + pc.pcol + e] : T(0);
        }
    }
}

// registers -> the wavefront's private patch (row-major, k contiguous)
template <typename T>
__device__ __forceinline__ void mttkrp_patch_store(
    T *patch, const MttkrpPieces<T> &pc, const typename VecOf<T, MttkrpCfg<T>::VEC>::type (&rs)[MttkrpCfg<T>::PER_T]) {
    typedef MttkrpCfg<T> Cfg;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
#pragma unroll
    for (int p = 0; p < Cfg::PER_T; ++p)
        *reinterpret_cast<vec_t *>(patch + (pc.prow + p * Cfg::RPI) * Cfg::LDW + pc.pcol) = rs[p];
}

// acc[lt](l, j) += sum over the slice of f[lt](l) * d[lt](l, k) * patch(j, k): the transposed
// product of one block with LT column tiles of 32, the D slice scaled by the walked index's
// factor on the way into the matrix pipe (KV multiplies per MFMA group; no scaled copy is kept).
template <typename T, int LT>
__device__ __forceinline__ void mttkrp_patch_mfma(
    const T *patch, int li, int ls,
    const typename VecOf<T, MttkrpCfg<T>::VEC>::type (&d)[LT][MttkrpCfg<T>::LB][MttkrpCfg<T>::NKG],
    const T (&f)[LT][MttkrpCfg<T>::LB],
    typename Mfma<T>::acc_t (&acc)[LT][MttkrpCfg<T>::LB][MttkrpCfg<T>::MI]) {
    typedef MttkrpCfg<T> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
#pragma unroll
    for (int g = 0; g < Cfg::NKG; ++g) {
        vec_t b[Cfg::MI];
#pragma unroll
        for (int mi = 0; mi < Cfg::MI; ++mi)
            b[mi] = *reinterpret_cast<const vec_t *>(patch + (mi * MF::NB + li) * Cfg::LDW
                                                     + g * Cfg::KG + ls * Cfg::KV);
#pragma unroll
        for (int lt = 0; lt < LT; ++lt)
#pragma unroll
            for (int lb = 0; lb < Cfg::LB; ++lb) {
                const vec_t ds = d[lt][lb][g] * f[lt][lb];
#pragma unroll
                for (int t = 0; t < Cfg::KV; ++t)
#pragma unroll
                    for (int mi = 0; mi < Cfg::MI; ++mi)
                        acc[lt][lb][mi] = MF::run(ds[t], b[mi][t], acc[lt][lb][mi]);
            }
    }
}

// The D operand of one k-slice, transposed into registers: d[lb][g][t] = D(k, l) for
// k = k0 + g*KG + ls*KV + t and l = n0 + li (binary32) or n0 + 2*li + lb (binary64); zero
// for l >= L (RAGGED), and for k >= K (GUARD).  Lanes with neighbouring li read neighbouring l.
template <typename T, bool GUARD, bool RAGGED>
__device__ __forceinline__ void mttkrp_load_d(
    const T *D, int64_t K, int64_t L, int64_t k0, int64_t n0, int li, int ls,
    typename VecOf<T, MttkrpCfg<T>::VEC>::type (&d)[MttkrpCfg<T>::LB][MttkrpCfg<T>::NKG]) {
    typedef MttkrpCfg<T> Cfg;
#pragma unroll
    for (int lb = 0; lb < Cfg::LB; ++lb) {
        const int64_t l = n0 + (Cfg::LB == 1 ? li : 2 * li + lb);
#pragma unroll
        for (int g = 0; g < Cfg::NKG; ++g)
#pragma unroll
            for (int t = 0; t < Cfg::KV; ++t) {
                const int64_t k = k0 + g * Cfg::KG + ls * Cfg::KV + t;
                d[lb][g][t] = ((!RAGGED || l < L) && ((!GUARD && !RAGGED) || k < K)) ? D[k * L + l] : T(0);
            }
    }
}

// A(i, l) = sum of the per_i partial rows of i, in row order.  One workgroup per i:
// thread (r, l) adds rows r, r+8, ..., then the eight strands are added in order.
template <typename T>
__global__ void __launch_bounds__(256)
mttkrp_reduce_kernel(const T *__restrict__ partial, T *__restrict__ A, int64_t I, int64_t L, int per_i) {
    __shared__ T strand[8][32];
    const int r = threadIdx.x >> 5, lx = threadIdx.x & 31;
    for (int64_t i = blockIdx.x; i < I; i += gridDim.x) {
        for (int64_t l0 = 0; l0 < L; l0 += 32) {
            const int64_t l = l0 + lx;
            T s = T(0);
            if (l < L)
                for (int t = r; t < per_i; t += 8) s += partial[(i * per_i + t) * L + l];
            __syncthreads();
            strand[r][lx] = s;
            __syncthreads();
            if (r == 0 && l < L) {
                T tot = strand[0][lx];
#pragma unroll
                for (int q = 1; q < 8; ++q) tot += strand[q][lx];
                A[i * L + l] = tot;
            }
        }
    }
}

// l (0..31 within the column tile) of accumulator element v of l-block lb.  binary64
// interleaves its two l-blocks (block lb owns l = 2*r + lb for MFMA row r), so that a
// lane's two blocks own neighbouring l.
template <typename T>
__device__ __forceinline__ int mttkrp_l_of(int v, int lb, int lane) {
    if (sizeof(T) == 4) return Mfma<T>::out_row(v, lane);
    return 2 * Mfma<T>::out_row(v, lane) + lb;
}

// ---------------------------------------------------------------------------
// MTTKRP along mode 0 or 1, as one sum over a WALKED index w of scaled matrix products:
//   A(r,l) = sum_w F(w,l) * ( sum_k B[r, w, k] * D(k,l) )
// where r is the kept index (the output row), w the other index that is not contracted by
// the MFMA, and B[r, w, k] = B + r*row_stride + w*walk_stride + k:
//   mode 0: r = i, w = j, F = C (J x L)      mode 1: r = j, w = i, F = C (I x L).
//
// The contracted index k is the contiguous one, while the MFMA wants the lanes of an operand
// spread over rows.  A block of B (RB = 32 values of r, one k-slice of SL = 256 bytes) therefore
// goes global -> registers by coalesced loads (a wavefront load covers 4 rows x 256 B; the next
// block's loads are in flight during the multiply) -> a wavefront-private LDS patch -> back in
// MFMA operand layout.  Only the wavefront that wrote a patch reads it, so ordering inside the
// wavefront suffices.  The MFMAs form the TRANSPOSED product Tt(l,r) = sum_k D(k,l) B[r,w,k].
// A wavefront keeps ONE block of r and one k-slice for its whole life (the D values of the
// slice stay in registers, already transposed) and walks a range of w.  For each w it scales
// its D slice by F(w,l) (32 multiplies) and lets the MFMAs add straight into one accumulator
// that lives as long as the wavefront: no per-block reduction, no lane reduction, no barrier
// anywhere.  The four wavefronts of a workgroup take neighbouring slices of the same rows
// (1 KiB contiguous per row).  At the end a wavefront writes its 32 x 32 partial block; the
// row-sum kernel adds the partial rows of each r in order.
// ---------------------------------------------------------------------------
template <typename T>
struct MttkrpWalkArgs {
    const T *B;        // I x J x K
    const T *F;        // W x L: the factor of the walked index
    const T *D;        // K x L
    T *partial;        // (R * nparts) x L: row r * nparts + (split * nslices + slice);
                       // the output itself when nparts == 1
    int64_t R, W, K, L;
    int64_t row_stride, walk_stride;   // elements between consecutive r resp. w in B
    int64_t wsplit;    // w per range
    int nsplit;        // ranges of w: ceil(W / wsplit), none empty
    int nslices;       // ceil(K / SL)
    int spw;           // k-slices per workgroup: 4, or 2 or 1 when K has no more; the workgroup's
                       // other wavefronts then take the next blocks of r (4 / spw blocks per workgroup)
    int kgroups;       // ceil(nslices / spw)
    int tiles_n;       // ceil(L / (32 * LT))
    int rblocks;       // ceil(R / 32)
    int rgroups;       // ceil(rblocks / (4 / spw))
};

// GUARD = false: rows of B are 16-byte aligned (aligned base, K a multiple of the vector):
// vector loads only.  RAGGED = true then allows any R and L and a short last k-slice (the last
// block of r re-reads its last row, columns l >= L carry zero factors, neither is stored; pieces
// and D rows past K are zero); RAGGED = false needs K % SL == 0, R % 32 == 0 and L % 32 == 0
// and keeps the register count at four wavefronts per SIMD.
// GUARD = true (with RAGGED): any shape and alignment, element loads with bounds checks.
// LT = column tiles of 32 per wavefront (1 or 2): with two, a rank above 32 reads B once per 64
// columns instead of once per 32.
template <typename T, bool GUARD, bool RAGGED, int LT>
__global__ void __launch_bounds__(256, GUARD ? 1 : (sizeof(T) == 4 ? 3 : 2))
mttkrp_walk_kernel(const MttkrpWalkArgs<T> args) {
    typedef MttkrpCfg<T> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    constexpr int NKG = Cfg::NKG, MI = Cfg::MI, LB = Cfg::LB;
    constexpr int SL = Cfg::SL, BN = Cfg::BN * LT, RB = Cfg::RB;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane % MF::MB, ls = lane / MF::MB;
    T *patch = reinterpret_cast<T *>(lds_raw) + wave * Cfg::PATCH;

    int bid = blockIdx.x;
    const int tn = bid % args.tiles_n;     bid /= args.tiles_n;
    const int kgp = bid % args.kgroups;    bid /= args.kgroups;
    const int rgrp = bid % args.rgroups;   bid /= args.rgroups;
    const int split = bid;
    const int64_t R = args.R, W = args.W, K = args.K, L = args.L;
    const int spw_log2 = args.spw >> 1;                          // spw is 1, 2 or 4
    const int slice = (kgp << spw_log2) + (wave & (args.spw - 1));
    const int rblk = (rgrp << (2 - spw_log2)) + (wave >> spw_log2);
    const int64_t n0 = (int64_t)tn * BN, r0 = (int64_t)rblk * RB;
    const int64_t k0 = (int64_t)slice * SL;
    if (k0 >= K || rblk >= args.rblocks) return;   // wavefront-uniform; this kernel has no barrier
    const int64_t w_lo = (int64_t)split * args.wsplit;
    const int64_t w_hi = (w_lo + args.wsplit < W) ? w_lo + args.wsplit : W;      // w_lo < w_hi by the plan

    vec_t d[LT][LB][NKG];
#pragma unroll
    for (int lt = 0; lt < LT; ++lt) mttkrp_load_d<T, GUARD, RAGGED>(args.D, K, L, k0, n0 + lt * Cfg::BN, li, ls, d[lt]);

    typename MF::acc_t acc[LT][LB][MI];
#pragma unroll
    for (int lt = 0; lt < LT; ++lt)
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) acc[lt][lb][mi][v] = T(0);

    vec_t rs[Cfg::PER_T];
    T fnext[LT][LB];                       // F(w, l) of the block in flight, l as in d
    const MttkrpPieces<T> pc(lane, args.row_stride);
    const T *block0 = args.B + r0 * args.row_stride + k0;                        // wavefront-uniform
    auto fetch = [&](int64_t w) {
        mttkrp_load_block<T, GUARD, RAGGED>(block0 + w * args.walk_stride, args.row_stride, R - r0, K - k0, pc, rs);
#pragma unroll
        for (int lt = 0; lt < LT; ++lt)
#pragma unroll
            for (int lb = 0; lb < LB; ++lb) {
                const int64_t l = n0 + lt * Cfg::BN + (LB == 1 ? li : 2 * li + lb);
                fnext[lt][lb] = (!RAGGED || l < L) ? args.F[w * L + l] : T(0);
            }
    };

    fetch(w_lo);
    for (int64_t w = w_lo; w < w_hi; ++w) {
        T f[LT][LB];
#pragma unroll
        for (int lt = 0; lt < LT; ++lt)
#pragma unroll
            for (int lb = 0; lb < LB; ++lb) f[lt][lb] = fnext[lt][lb];
        mttkrp_patch_store<T>(patch, pc, rs);
        fetch(w + 1 < w_hi ? w + 1 : w);   // past the end: a redundant, in-bounds reload
        wave_lds_fence();
        mttkrp_patch_mfma<T, LT>(patch, li, ls, d, f, acc);
        wave_lds_fence();
    }

    const int nparts = args.nsplit * args.nslices;
    const int part = split * args.nslices + slice;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int64_t r = r0 + mi * MF::NB + li;
        if (RAGGED && r >= R) continue;
        T *row = args.partial + (r * nparts + part) * L + n0;
#pragma unroll
        for (int lt = 0; lt < LT; ++lt)
#pragma unroll
            for (int lb = 0; lb < LB; ++lb)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) {
                    const int l = lt * Cfg::BN + mttkrp_l_of<T>(v, lb, lane);
                    if (!RAGGED || n0 + l < L) row[l] = acc[lt][lb][mi][v];
                }
    }
}

// ---------------------------------------------------------------------------
// MTTKRP along mode 2:  A(k,l) = sum_i sum_j B(i,j,k) * C(i,l) * D(j,l).
//
// The output rows are indexed by the CONTIGUOUS index of B, so B's rows are already in
// MFMA operand layout: the lane that owns output row k reads B(i,j,k) itself, with
// coalesced 16-byte loads and no LDS.  A lane's VEC neighbouring values belong to VEC
// interleaved row blocks (block e owns k = ... + li*VEC + e).  The other operand is the
// Khatri-Rao row W((i,j), l) = C(i,l) * D(j,l), formed in registers: a wavefront keeps 16
// rows of j (their D values stay in registers), walks a range of i, and for each i
// multiplies by C(i,l).  The accumulators (KW output rows x 32 columns per wavefront)
// live as long as the wavefront, and so does the single register set that holds a block
// of B: each piece is reloaded with the next slice's values right after its MFMAs issue.  The four wavefronts of a workgroup take neighbouring
// j-blocks of the same k-range; at the end they are added through LDS in wavefront order
// and the workgroup writes one partial block; the row-sum kernel finishes.
// ---------------------------------------------------------------------------
template <typename T, int LT>
struct MttkrpMode2Cfg {
    typedef Mfma<T> MF;
    static constexpr int NT = 256, NW = 4, BN = 32 * LT;    // LT column tiles of 32 per wavefront
    static constexpr int VEC = 16 / (int)sizeof(T);
    static constexpr int KW = 512 / (int)sizeof(T);        // output rows (k) per workgroup
    static constexpr int NP = KW / (MF::MB * VEC);         // 16-byte loads per lane per r-group
    static constexpr int RBK = NP * VEC;                   // row blocks per wavefront
    static constexpr int LB = BN / MF::NB;                 // column blocks
    static constexpr int JB = 16;                          // rows of j per wavefront
    static constexpr int NG = JB / MF::KS;                 // MFMA steps (groups of KS rows) per block
    static constexpr int PER_T = NG * NP;                  // loads per lane per block
    static constexpr int NACC = RBK * LB * MF::NACC;       // accumulator values per lane
    static constexpr int LDS_BYTES = NACC * 64 * (int)sizeof(T);
    static_assert(KW % (MF::MB * VEC) == 0 && JB % MF::KS == 0, "tile shape");
};

template <typename T>
struct MttkrpMode2Args {
    const T *B;        // I x J x K
    const T *C;        // I x L
    const T *D;        // J x L
    T *partial;        // (K * nparts) x L: row k * nparts + (split * jgroups + jgroup);
                       // the output itself when nparts == 1
    int64_t I, J, K, L;
    int64_t isplit;    // i per range
    int nsplit;        // ranges of i, none empty
    int jgroups;       // ceil(J / (4 * JB))
    int kblocks;       // ceil(K / KW)
    int tiles_n;       // ceil(L / (32 * LT))
};

// GUARD / RAGGED / LT as for the kernel above: without GUARD an aligned base and K % VEC == 0 are
// needed; RAGGED = true allows any J and L and such K, RAGGED = false needs K % KW == 0,
// J % 16 == 0 and L % (32 * LT) == 0.
template <typename T, bool GUARD, bool RAGGED, int LT>
__global__ void __launch_bounds__(256, GUARD ? 1 : (LT == 1 ? 3 : 2))
mttkrp_mode2_kernel(const MttkrpMode2Args<T> args) {
    typedef MttkrpMode2Cfg<T, LT> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    constexpr int VEC = Cfg::VEC, NP = Cfg::NP, RBK = Cfg::RBK, LB = Cfg::LB, NG = Cfg::NG;
    constexpr int PER_T = Cfg::PER_T, JB = Cfg::JB;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T *red = reinterpret_cast<T *>(lds_raw);          // [NACC][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane % MF::MB, ls = lane / MF::MB;

    int bid = blockIdx.x;
    const int tn = bid % args.tiles_n;     bid /= args.tiles_n;
    const int kblk = bid % args.kblocks;   bid /= args.kblocks;
    const int jgroup = bid % args.jgroups; bid /= args.jgroups;
    const int split = bid;
    const int64_t I = args.I, J = args.J, K = args.K, L = args.L;
    const int64_t n0 = (int64_t)tn * Cfg::BN, k0 = (int64_t)kblk * Cfg::KW;
    const int64_t j0 = ((int64_t)jgroup * Cfg::NW + wave) * JB;
    const bool active = j0 < J;                       // wavefront-uniform
    const int64_t i_lo = (int64_t)split * args.isplit;
    const int64_t i_hi = (i_lo + args.isplit < I) ? i_lo + args.isplit : I;

    typename MF::acc_t acc[RBK][LB];
#pragma unroll
    for (int rb = 0; rb < RBK; ++rb)
#pragma unroll
        for (int cb = 0; cb < LB; ++cb)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) acc[rb][cb][v] = T(0);

    if (active) {
        // D(j, l) of this wavefront's rows: dj[g][cb] for j = j0 + g*KS + ls, l = n0 + cb*NB + li
        T dj[NG][LB];
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int cb = 0; cb < LB; ++cb) {
                const int64_t j = j0 + g * MF::KS + ls, l = n0 + cb * MF::NB + li;
                dj[g][cb] = (!RAGGED || (j < J && l < L)) ? args.D[j * L + l] : T(0);
            }
        // The lane's piece (g, p) of the block of slice i: row j0 + g*KS + ls, elements
        // k0 + p*MB*VEC + li*VEC ...  The row-group part of the address is wavefront-uniform.
        const int64_t lane_off = (int64_t)ls * K + li * VEC;
        const bool full_rows = j0 + JB <= J && k0 + Cfg::KW <= K;   // wavefront-uniform: a full block
        auto piece = [&](int64_t i, int g, int p) -> vec_t {
            const T *base = args.B + ((i * J + j0 + g * MF::KS) * K + k0 + p * MF::MB * VEC);   // uniform
            if constexpr (!GUARD) {
                if (!RAGGED || full_rows) return __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(base + lane_off));
                // a ragged block: rows of j past the end re-read row J-1 (their D factor is zero);
                // pieces past the end of a row re-read its last piece (K is a multiple of VEC) and
                // feed output rows k >= K, which are not stored
                int64_t j = j0 + g * MF::KS + ls, k = k0 + p * MF::MB * VEC + li * VEC;
                if (j >= J) j = J - 1;
                if (k > K - VEC) k = K - VEC;
                return __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(args.B + (i * J + j) * K + k));
            } else {
                vec_t x;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int64_t jr = g * MF::KS + ls, kc = p * MF::MB * VEC + li * VEC + e;
                    x[e] = (j0 + jr < J && k0 + kc < K) ? base[lane_off + e] : T(0);
                }
                return x;
            }
        };
        auto factor = [&](int64_t i, T (&c)[LB]) {
#pragma unroll
            for (int cb = 0; cb < LB; ++cb) {
                const int64_t l = n0 + cb * MF::NB + li;
                c[cb] = (!RAGGED || l < L) ? args.C[i * L + l] : T(0);
            }
        };

        // One register set, refilled piece by piece: as soon as the MFMAs of a row group have
        // been issued its registers are reloaded with the same group of the next slice, so
        // every piece has a whole block's multiply time to arrive.
        vec_t rs[PER_T];
        T c[LB], cn[LB];
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int p = 0; p < NP; ++p) rs[g * NP + p] = piece(i_lo, g, p);
        factor(i_lo, c);
        for (int64_t i = i_lo; i < i_hi; ++i) {
            const int64_t inext = i + 1 < i_hi ? i + 1 : i;      // past the end: a redundant, in-bounds reload
            factor(inext, cn);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                T w[LB];
#pragma unroll
                for (int cb = 0; cb < LB; ++cb) w[cb] = c[cb] * dj[g][cb];
#pragma unroll
                for (int p = 0; p < NP; ++p)
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
#pragma unroll
                        for (int cb = 0; cb < LB; ++cb)
                            acc[p * VEC + e][cb] = MF::run(rs[g * NP + p][e], w[cb], acc[p * VEC + e][cb]);
#pragma unroll
                for (int p = 0; p < NP; ++p) rs[g * NP + p] = piece(inext, g, p);
                __builtin_amdgcn_sched_barrier(0);     // keep each refill next to the MFMAs that freed it
            }
#pragma unroll
            for (int cb = 0; cb < LB; ++cb) c[cb] = cn[cb];
        }
    }

    // add the four wavefronts in wavefront order (inactive ones hold zeros)
#pragma unroll 1
    for (int w = 0; w < Cfg::NW; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rb = 0; rb < RBK; ++rb)
#pragma unroll
                for (int cb = 0; cb < LB; ++cb)
#pragma unroll
                    for (int v = 0; v < MF::NACC; ++v) {
                        T *slot = red + ((rb * LB + cb) * MF::NACC + v) * 64 + lane;
                        *slot = (w == 0) ? acc[rb][cb][v] : *slot + acc[rb][cb][v];
                    }
        }
        __syncthreads();
    }
    // the workgroup's partial block: row block rb is written by wavefront rb % NW
    const int nparts = args.nsplit * args.jgroups;
    const int part = split * args.jgroups + jgroup;
#pragma unroll
    for (int rb = 0; rb < RBK; ++rb) {
        if (rb % Cfg::NW != wave) continue;
        const int p = rb / VEC, e = rb % VEC;
#pragma unroll
        for (int cb = 0; cb < LB; ++cb)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) {
                const int64_t k = k0 + p * MF::MB * VEC + MF::out_row(v, lane) * VEC + e;
                const int64_t l = n0 + cb * MF::NB + li;
                if ((!RAGGED || l < L) && ((!GUARD && !RAGGED) || k < K))
                    args.partial[(k * nparts + part) * L + l] = red[((rb * LB + cb) * MF::NACC + v) * 64 + lane];
            }
    }
}

}  // namespace distal
