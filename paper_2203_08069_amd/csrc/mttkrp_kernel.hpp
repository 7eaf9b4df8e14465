// Fused MTTKRP for gfx950:  A(i,l) = sum_j C(j,l) * ( sum_k B(i,j,k) * D(k,l) ).
//
// The paper's leaf casts MTTKRP to matrix multiplications followed by an
// element-wise reduction (evaluation section, leaf kernels).  Here both happen
// in one pass over B, which is read from HBM exactly once.  After a one-time
// set-up every wavefront is an independent stream: there is no workgroup barrier
// in the streaming loop, and the only global loads in it are fully coalesced
// 16-byte loads of B (the address unit, not HBM or the matrix pipe, is the first
// thing lane-scattered loads exhaust here).
//
//   * The grid is persistent.  A workgroup is pinned to one chunk of j (CJ rows),
//     one group of four k-slices and one column tile, and walks a strided list of
//     i.  The factor rows C(chunk, tile) are copied to LDS once, at set-up.
//   * A wavefront owns ONE k-slice of SL = 256 bytes for its whole life.  The D
//     values of its slice (SL k x 32 l) are loaded into registers once, already in
//     the transposed MFMA operand layout, so D costs no further traffic.  The four wavefronts of a workgroup take neighbouring
//     slices of the same rows (1 KiB contiguous per row).
//   * The wavefront walks (i, block of RB = 32 rows).  A block's RB x SL piece of B
//     goes global -> registers (the next block's loads are in flight during the
//     multiply) -> a wavefront-private LDS patch -> back in MFMA operand layout.
//     Only the wavefront that wrote the patch reads it, so ordering inside the
//     wavefront suffices.
//   * MFMA forms the TRANSPOSED partial product Tt(l,j) = sum_{k in slice} D(k,l)
//     B(j,k): a lane owns one j and several l, so the factor values C(j, l..) it
//     needs are neighbours in the LDS copy.  The sums over j and over k-slices are
//     both linear: after every block the lane scales its accumulators by C(j,l) and
//     adds them to running sums, one per owned l.
//   * At the end of an (i, chunk) the lanes that own the same l are added with DPP
//     rotations in a fixed order and the wavefront writes its own partial row of 32
//     values to the workspace; a last small kernel adds the partial rows of each i
//     in order.  Nothing is atomic and no sum depends on the grid size: results are
//     bitwise reproducible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"
#include "stream_kernels.hpp"   // sum16 (DPP row rotations)

namespace distal {

template <typename T>
struct MttkrpArgs {
    const T *B;        // I x J x K
    const T *C;        // J x L
    const T *D;        // K x L
    T *partial;        // (I * nchunks * nslices) x L: row ((i * nchunks + chunk) * nslices + slice);
                       // the output itself when nchunks * nslices == 1
    int64_t I, J, K, L;
    int nchunks;       // ceil(J / CJ)
    int nslices;       // ceil(K / SL)
    int kgroups;       // ceil(nslices / 4): k-slices are handed out four per workgroup
    int tiles_n;       // ceil(L / 32)
    int igroups;       // gridDim.x / (tiles_n * kgroups * nchunks): workgroups sharing the list of i
};

template <typename T>
struct MttkrpCfg {
    typedef Mfma<T> MF;
    static constexpr int NT = 256, NW = 4, BN = 32, RB = 32;
    static constexpr int CJ = 128;                        // rows of j per chunk
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
    static constexpr int LDC = BN + VEC;                  // factor-copy row stride (elements): +16 B
    static constexpr int C_ELEMS = CJ * LDC;
    static constexpr int LDS_BYTES = (NW * PATCH + C_ELEMS) * (int)sizeof(T);
    static_assert(SL % KG == 0 && RB % MF::NB == 0 && LB <= 2 && 64 % CPR == 0 && CJ % RB == 0, "tile shape");
};

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

// GUARD = false: every row block and k-slice of B is full and 16-byte aligned
// (J % 32 == 0, K % SL == 0, L % 32 == 0, aligned bases) - vector loads only.
// GUARD = true: any shape and alignment, element loads with bounds checks, zero fill.
template <typename T, bool GUARD>
__global__ void __launch_bounds__(256, GUARD ? 1 : (sizeof(T) == 4 ? 3 : 2))
mttkrp_kernel(const MttkrpArgs<T> args) {
    typedef MttkrpCfg<T> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    constexpr int VEC = Cfg::VEC, KV = Cfg::KV, KG = Cfg::KG, NKG = Cfg::NKG, MI = Cfg::MI, LB = Cfg::LB;
    constexpr int SL = Cfg::SL, BN = Cfg::BN, RB = Cfg::RB, CJ = Cfg::CJ;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // the wavefront index is the same in all lanes: say so, and every address that depends on it
    // stays in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane % MF::MB, ls = lane / MF::MB;
    T *patch = lds + wave * Cfg::PATCH;
    T *cfac = lds + Cfg::NW * Cfg::PATCH;          // C(chunk rows, tile columns), row stride LDC

    int bid = blockIdx.x;
    const int tn = bid % args.tiles_n;    bid /= args.tiles_n;
    const int kgp = bid % args.kgroups;   bid /= args.kgroups;
    const int chunk = bid % args.nchunks; bid /= args.nchunks;
    const int ig = bid;                                         // first i of this workgroup
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t I = args.I, J = args.J, K = args.K, L = args.L;
    const int64_t jb = (int64_t)chunk * CJ;
    const int64_t je = (jb + CJ < J) ? jb + CJ : J;
    const int nrb = (int)((je - jb + RB - 1) / RB);

    // set-up: factor rows of this chunk and tile -> LDS, zero outside J x L
    for (int v = tid; v < CJ * (BN / VEC); v += Cfg::NT) {
        const int r = v / (BN / VEC), cv = (v % (BN / VEC)) * VEC;
        vec_t x;
        if (!GUARD) {
            x = vec_t(T(0));
            if (jb + r < J) x = *reinterpret_cast<const vec_t *>(args.C + (jb + r) * L + n0 + cv);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                x[e] = (jb + r < J && n0 + cv + e < L) ? args.C[(jb + r) * L + n0 + cv + e] : T(0);
        }
        *reinterpret_cast<vec_t *>(cfac + r * Cfg::LDC + cv) = x;
    }
    __syncthreads();                       // the only barrier of this kernel

    const int slice = kgp * Cfg::NW + wave;
    const int64_t k0 = (int64_t)slice * SL;                    // this wavefront's k-slice
    if (k0 >= K || ig >= I) return;       // wavefront-uniform

    // The D operand of this slice, transposed into registers once: d[lb][g][t] = D(k, l) for
    // k = k0 + g*KG + ls*KV + t and l = n0 + li (binary32) or n0 + 2*li + lb (binary64); zero
    // outside K x L.  Lanes with neighbouring li read neighbouring l.
    vec_t d[LB][NKG];
#pragma unroll
    for (int lb = 0; lb < LB; ++lb) {
        const int64_t l = n0 + (LB == 1 ? li : 2 * li + lb);
#pragma unroll
        for (int g = 0; g < NKG; ++g)
#pragma unroll
            for (int t = 0; t < KV; ++t) {
                const int64_t k = k0 + g * KG + ls * KV + t;
                d[lb][g][t] = (!GUARD || (k < K && l < L)) ? args.D[k * L + l] : T(0);
            }
    }

    T lsum[LB][MF::NACC];                 // running sum for l = mttkrp_l_of(v, lb, lane)
#pragma unroll
    for (int lb = 0; lb < LB; ++lb)
#pragma unroll
        for (int v = 0; v < MF::NACC; ++v) lsum[lb][v] = T(0);

    vec_t rs[Cfg::PER_T];
    const int prow = lane / Cfg::CPR, pcol = (lane % Cfg::CPR) * VEC;
    // Per-lane byte offsets inside a row block; the block base is wavefront-uniform.  The host
    // sends shapes whose block spans exceed 32-bit offsets to the guarded kernel.
    uint32_t boff[Cfg::PER_T];
#pragma unroll
    for (int p = 0; p < Cfg::PER_T; ++p)
        boff[p] = (uint32_t)(((int64_t)(prow + p * Cfg::RPI) * K + pcol) * (int64_t)sizeof(T));

    // rows [jb + rb*RB, +RB) of slice i, k in [k0, k0 + SL) -> rs
    auto load_rows = [&](int64_t i, int rb) {
        const T *base = args.B + (i * J + jb + (int64_t)rb * RB) * K + k0;      // wavefront-uniform
        if constexpr (!GUARD) {
#pragma unroll
            for (int p = 0; p < Cfg::PER_T; ++p)
                rs[p] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(
                    reinterpret_cast<const char *>(base) + boff[p]));
        } else {
#pragma unroll
            for (int p = 0; p < Cfg::PER_T; ++p) {
                const int64_t jr = prow + p * Cfg::RPI;                          // row within the block
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    rs[p][e] = (jb + (int64_t)rb * RB + jr < J && k0 + pcol + e < K)
                                   ? base[jr * K + pcol + e] : T(0);
            }
        }
    };

    // One 32-row block: patch -> MFMA -> fold.  `c` are the lane's factor pieces for this block.
    auto block = [&](int64_t i, int rb, const vec_t (&c)[MI][4]) {
        // what comes after this block: the next block of this i, or the first block of the next i
        const bool last_rb = (rb + 1 == nrb);
        const int64_t next_i = last_rb ? i + args.igroups : i;
        const int next_rb = last_rb ? 0 : rb + 1;
        const bool more = next_i < I;

        // registers -> private patch (row-major, k contiguous)
#pragma unroll
        for (int p = 0; p < Cfg::PER_T; ++p)
            *reinterpret_cast<vec_t *>(patch + (prow + p * Cfg::RPI) * Cfg::LDW + pcol) = rs[p];
        // past the end: a redundant reload of the current block, never out of bounds
        load_rows(more ? next_i : i, more ? next_rb : rb);

        // the patch is written and read by this wavefront only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        typename MF::acc_t acc[LB][MI];
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) acc[lb][mi][v] = T(0);
#pragma unroll
        for (int g = 0; g < NKG; ++g) {
            vec_t b[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                b[mi] = *reinterpret_cast<const vec_t *>(patch + (mi * MF::NB + li) * Cfg::LDW
                                                         + g * KG + ls * KV);
#pragma unroll
            for (int t = 0; t < KV; ++t)
#pragma unroll
                for (int lb = 0; lb < LB; ++lb)
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        acc[lb][mi] = MF::run(d[lb][g][t], b[mi][t], acc[lb][mi]);
        }
        // all reads of the patch are done before the next block overwrites it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // scale Tt(l, j) by C(j, l) and add into the lane's running sums
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v)
#pragma unroll
                for (int lb = 0; lb < LB; ++lb) {
                    T f;
                    if constexpr (sizeof(T) == 4) f = c[mi][v >> 2][v & 3];
                    else f = c[mi][v][lb];
                    lsum[lb][v] = fma_t(acc[lb][mi][v], f, lsum[lb][v]);
                }
    };

    // (i, chunk) done: add the lanes that own the same l (same k-slot ls, all li) in a fixed
    // order and write this wavefront's partial row
    auto flush = [&](int64_t i) {
        T *prow_out = args.partial + ((i * args.nchunks + chunk) * args.nslices + slice) * L + n0;
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) {
                T s = sum16(lsum[lb][v]);
                if (MF::MB == 32) s += __shfl_xor(s, 16);
                lsum[lb][v] = s;
            }
        if (li == 0) {
#pragma unroll
            for (int lb = 0; lb < LB; ++lb)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) {
                    const int l = mttkrp_l_of<T>(v, lb, lane);
                    if (!GUARD || n0 + l < L) prow_out[l] = lsum[lb][v];
                }
        }
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) lsum[lb][v] = T(0);
    };

    load_rows(ig, 0);
    for (int64_t i = ig; i < I; i += args.igroups) {
        for (int rb = 0; rb < nrb; ++rb) {
            // the lane's factor pieces for this block, from the LDS copy:
            // binary32: l = 8q + 4*ls + r (v = 4q + r); binary64: l = 2*(4q + ls) + lb (v = q)
            vec_t c[MI][4];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const T *crow = cfac + (rb * RB + mi * MF::NB + li) * Cfg::LDC
                                + (sizeof(T) == 4 ? 4 * ls : 2 * ls);
#pragma unroll
                for (int q = 0; q < 4; ++q) c[mi][q] = *reinterpret_cast<const vec_t *>(crow + 8 * q);
            }
            block(i, rb, c);
        }
        flush(i);
    }
}

}  // namespace distal
