// Tensor-times-matrix over the last mode with a rank-sized factor (L <= 32) and a contracted
// extent of at most a few KiB per tensor row:
//   A(r, l) = sum_k B(r, k) * C(k, l),   r = (i, j), rows of B K elements apart.
//
// Such a product moves 16 flop per byte of B: it is bound by HBM, and what decides its speed is
// that B streams through exactly once and that nothing else competes for the path from L2.  The
// tiled contraction kernel fetches the whole factor again for every 128 rows (a quarter on top of
// the tensor's own requests).  Here the factor never moves again after the first microsecond: the
// k-extent is cut into slices of 256 bytes, wavefront w of a workgroup keeps slices w, w + 8, ...
// of C in registers, already in the layout the matrix instruction wants (as the MTTKRP kernels keep
// their slice of D), and the workgroup walks down the rows of B, 32 at a time.  For a block of rows
// every wavefront loads its slices of those rows (coalesced 16-byte loads, the eight wavefronts
// together 2 KiB contiguous per row; the next slice is in flight during the multiply), turns them
// into operand layout through its private LDS patch, and multiplies them into one 32 x 32
// accumulator.  The eight partial blocks are then added through LDS in wavefront order - each
// wavefront adds and stores four of the 32 rows - so the result does not depend on timing.  Two
// workgroup barriers per block of rows, with the next block's loads in flight across them (a
// second set of partial blocks, which saves one of the barriers, measured no faster).
//
// Evaluation section of the paper: TTM is among the higher-order kernels whose leaves are cast to
// matrix products; this is that product for the shape a factorisation gives it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mttkrp_kernel.hpp"

namespace distal {

template <typename T, int NS>
struct TtmSlicesCfg {
    typedef MttkrpCfg<T> MC;
    typedef Mfma<T> MF;
    static constexpr int NW = 8, NT = 64 * NW;
    static constexpr int RB = MC::RB, SL = MC::SL;
    static constexpr int KMAX = NW * NS * SL;                     // deepest product the registers hold the factor for
    static constexpr int LDP = 32 + 1;                            // partial block: row stride (elements), r-major
    static constexpr int PART = RB * LDP;                         // elements per partial block
    static_assert(PART <= MC::PATCH, "a partial block lies in its wavefront's patch");
    static constexpr int LDS_BYTES = NW * MC::PATCH * (int)sizeof(T);
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

template <typename T>
struct TtmSlicesArgs {
    const T *B;        // R x K, rows K elements apart (the tensor as a matrix)
    const T *C;        // K x L
    T *A;              // R x L
    int64_t R, K, L;
    int64_t rblocks;   // ceil(R / 32)
};

// acc(l, r) += sum over the slice of d(l, k) * patch(r, k)
template <typename T>
__device__ __forceinline__ void ttm_patch_mfma(
    const T *patch, int li, int ls,
    const typename VecOf<T, MttkrpCfg<T>::VEC>::type (&d)[MttkrpCfg<T>::LB][MttkrpCfg<T>::NKG],
    typename Mfma<T>::acc_t (&acc)[MttkrpCfg<T>::LB][MttkrpCfg<T>::MI]) {
    typedef MttkrpCfg<T> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
#pragma unroll
    for (int g = 0; g < Cfg::NKG; ++g) {
        vec_t b[Cfg::MI];
#pragma unroll
        for (int mi = 0; mi < Cfg::MI; ++mi)
            b[mi] = *reinterpret_cast<const vec_t *>(patch + (mi * MF::NB + li) * Cfg::LDW + g * Cfg::KG + ls * Cfg::KV);
#pragma unroll
        for (int lb = 0; lb < Cfg::LB; ++lb)
#pragma unroll
            for (int t = 0; t < Cfg::KV; ++t)
#pragma unroll
                for (int mi = 0; mi < Cfg::MI; ++mi) acc[lb][mi] = MF::run(d[lb][g][t], b[mi][t], acc[lb][mi]);
    }
}

// NS = slices per wavefront: K <= 8 * NS * (256 / sizeof(T)).  Rows of B are 16-byte aligned
// (aligned base, K a multiple of the vector); L <= 32, columns l >= L carry zero factors and are
// not stored.  RAGGED = false needs R % 32 == 0 and K == 8 * NS * (256 / sizeof(T)); RAGGED = true
// allows any R and a shorter K with a short last slice (the last block re-reads its last row,
// which is not stored; a wavefront whose slice lies past K multiplies zeros).
// Every workgroup takes the blocks of rows blockIdx.x, blockIdx.x + gridDim.x, ...; every
// wavefront of it runs the same number of trips, so the barriers match.
template <typename T, int NS, bool RAGGED>
__global__ void __launch_bounds__(512, 1)
ttm_slices_kernel(const TtmSlicesArgs<T> args) {
    typedef TtmSlicesCfg<T, NS> Cfg;
    typedef MttkrpCfg<T> MC;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, MC::VEC>::type vec_t;
    constexpr int NW = Cfg::NW, SL = Cfg::SL, RB = Cfg::RB, LB = MC::LB, MI = MC::MI, LDP = Cfg::LDP;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane % MF::MB, ls = lane / MF::MB;
    T *patch = reinterpret_cast<T *>(lds_raw) + wave * MC::PATCH;
    T *parts = reinterpret_cast<T *>(lds_raw);       // a wavefront's partial block lies in its own patch, free by then
    const int64_t R = args.R, K = args.K, L = args.L;

    // this wavefront's slices of the factor, for its whole life
    vec_t d[NS][LB][MC::NKG];
#pragma unroll
    for (int q = 0; q < NS; ++q)
        mttkrp_load_d<T, false, true>(args.C, K, L, (int64_t)(q * NW + wave) * SL, 0, li, ls, d[q]);

    const MttkrpPieces<T> pc(lane, K);
    vec_t rs[MC::PER_T];
    // step t = (trip, q): slice q * NW + wave of the trip's block of rows
    auto fetch = [&](int64_t blk, int q) {
        const int64_t r0 = blk * RB, k0 = (int64_t)(q * NW + wave) * SL;
        mttkrp_load_block<T, false, RAGGED>(args.B + r0 * K + k0, K, R - r0, K - k0, pc, rs);
    };

    const int64_t first = blockIdx.x, stride = gridDim.x;
    if (first >= args.rblocks) return;                                   // workgroup-uniform
    fetch(first, 0);
    for (int64_t blk = first; blk < args.rblocks; blk += stride) {
        typename MF::acc_t acc[LB][MI];
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) acc[lb][mi][v] = T(0);
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            mttkrp_patch_store<T>(patch, pc, rs);
            // the next step's loads; past the last block: a redundant, in-bounds reload of this one
            if (q + 1 < NS) fetch(blk, q + 1);
            else fetch(blk + stride < args.rblocks ? blk + stride : blk, 0);
            wave_lds_fence();
            ttm_patch_mfma<T>(patch, li, ls, d[q], acc);
            wave_lds_fence();
        }
        // this wavefront's partial block, r-major
        T *mine = parts + wave * MC::PATCH;
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v)
                    mine[(mi * MF::NB + li) * LDP + mttkrp_l_of<T>(v, lb, lane)] = acc[lb][mi][v];
        __syncthreads();
        // rows 4 * wave ... + 3 of the block, added in wavefront order: lane -> column lane % 32 of
        // rows lane / 32 and lane / 32 + 2 (64 lanes store two neighbouring rows of A: 256 contiguous bytes)
        {
            const int l = lane & 31, ra = 4 * wave + (lane >> 5), rb = ra + 2;
            const T *src = parts + l;
            T s0 = src[ra * LDP], s1 = src[rb * LDP];
#pragma unroll
            for (int p = 1; p < NW; ++p) {
                s0 += src[p * MC::PATCH + ra * LDP];
                s1 += src[p * MC::PATCH + rb * LDP];
            }
            const int64_t row = blk * RB;
            if (l < L) {
                // (plain and non-temporal stores measure the same here)
                if (!RAGGED || row + ra < R) args.A[(row + ra) * L + l] = s0;
                if (!RAGGED || row + rb < R) args.A[(row + rb) * L + l] = s1;
            }
        }
        __syncthreads();                 // the patches are free again
    }
}

}  // namespace distal
