// Fused MTTKRP for gfx950:  A(i,l) = sum_j C(j,l) * ( sum_k B(i,j,k) * D(k,l) ).
//
// The paper's leaf casts MTTKRP to matrix multiplications followed by an
// element-wise reduction (evaluation section, leaf kernels).  Here both happen
// in one pass over B, which is read from HBM exactly once:
//
//   * A small pre-kernel writes D transposed and zero-padded (Dt: 32*tiles_n rows
//     of Kpad values), so that k is the contiguous index of BOTH MFMA operands.
//   * A workgroup owns one i and a chunk of j.  It walks that chunk in tiles of
//     BM rows (j) and each tile in slabs of BK = 512 bytes of k, so every global
//     read of B is a 512-byte contiguous run - the run length at which HBM
//     streaming reaches its plateau on this part.
//   * A slab is (BM + 32) rows of BK values: BM rows of B and the 32 rows of Dt
//     for this column tile.  It goes global -> registers -> LDS (one LDS buffer;
//     the next slab's loads are in flight while the current one is multiplied).
//   * MFMA forms the TRANSPOSED product Tt(l,j) = sum_k Dt(l,k) B(j,k): a lane then
//     owns one j and several l, so the factor values C(j, l..) it needs are
//     contiguous in memory.  The four wavefronts split the slab's k range
//     ("split-k"), each holding a partial Tt_w.
//   * The reduction over j is linear, so no wavefront needs the others' partial
//     Tt: at the end of a tile each lane scales its own accumulators by C(j,l)
//     and folds them into running sums, one per owned l.  Only when the whole
//     chunk is done do the lane sums meet in LDS, in a fixed order.
//   * One partial row of L values per (i, chunk) goes to the workspace; a last
//     tiny kernel adds the chunks in order.  Nothing is atomic: results are
//     bitwise reproducible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace distal {

template <typename T>
struct MttkrpArgs {
    const T *B;        // I x J x K
    const T *C;        // J x L
    const T *Dt;       // (32 * tiles_n) x Kpad, transposed zero-padded D
    T *partial;        // (I * nchunks) x L, or the output itself when nchunks == 1
    int64_t I, J, K, L;
    int64_t Kpad;      // K rounded up to a multiple of BK
    int64_t jc;        // rows of j per chunk (a multiple of BM)
    int nchunks;       // ceil(J / jc)
    int tiles_n;       // ceil(L / 32)
};

template <typename T, int BM>
struct MttkrpCfg {
    typedef Mfma<T> MF;
    static constexpr int NT = 256, NW = 4, BN = 32;
    static constexpr int VEC = 16 / (int)sizeof(T);
    static constexpr int BK = 512 / (int)sizeof(T);
    static constexpr int KV = VEC, KG = MF::KS * KV;
    static constexpr int KG_PER_WAVE = BK / KG / NW;
    static constexpr int MI = BM / MF::NB;                // j blocks (MFMA columns)
    static constexpr int LB = BN / MF::MB;                // l blocks (MFMA rows): 1 (f32) or 2 (f64)
    static constexpr int NSUM = LB * MF::NACC;            // running sums per lane
    static constexpr int ROWS = BM + BN;                  // slab rows: B tile, then Dt tile
    static constexpr int LD_S = BK + VEC;                 // LDS row stride (elements): +16 B
    static constexpr int LDS_BYTES = ROWS * LD_S * (int)sizeof(T);
    static constexpr int VECS = ROWS * (BK / VEC);
    static constexpr int PER_T = VECS / NT;
    static constexpr int B_PER_T = BM * (BK / VEC) / NT;  // of which from B
    static_assert(BM % MF::NB == 0 && BK % (KG * NW) == 0 && LB <= 2, "tile shape");
    static_assert(VECS % NT == 0 && (BM * (BK / VEC)) % NT == 0, "slab vectors must divide over threads");
    static_assert(NT * NSUM * (int)sizeof(T) <= LDS_BYTES, "final reduction fits the slab buffer");
};

// Dt(l, k) = D(k, l), zero outside K x L.
template <typename T>
__global__ void __launch_bounds__(256)
mttkrp_transpose_kernel(const T *__restrict__ D, T *__restrict__ Dt, int64_t K, int64_t L,
                        int64_t Kpad, int64_t Lpad) {
    const int64_t n = Kpad * Lpad;
    for (int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x; m < n; m += (int64_t)gridDim.x * 256) {
        const int64_t l = m / Kpad, k = m % Kpad;
        Dt[m] = (l < L && k < K) ? D[k * L + l] : T(0);
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

// GUARD = false: every tile and slab of B is full and 16-byte aligned (J % BM == 0,
// K % BK == 0, L % 32 == 0, aligned bases) - vector loads only.  GUARD = true: any
// shape and alignment, element loads with bounds checks and zero fill.
template <typename T, int BM, bool GUARD>
__global__ void __launch_bounds__(256, GUARD ? 1 : (sizeof(T) == 4 ? 3 : 2))
mttkrp_kernel(const MttkrpArgs<T> args) {
    typedef MttkrpCfg<T, BM> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    constexpr int VEC = Cfg::VEC, KV = Cfg::KV, KG = Cfg::KG, MI = Cfg::MI, LB = Cfg::LB;
    constexpr int NT = Cfg::NT, BK = Cfg::BK, BN = Cfg::BN;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T *slab = reinterpret_cast<T *>(lds_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane % MF::MB, ls = lane / MF::MB;

    const int tn = blockIdx.x % args.tiles_n;
    const int64_t ic = blockIdx.x / args.tiles_n;          // i * nchunks + chunk
    const int64_t i = ic / args.nchunks, chunk = ic % args.nchunks;
    const int64_t j_begin = chunk * args.jc;
    const int64_t j_end = (j_begin + args.jc < args.J) ? j_begin + args.jc : args.J;
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t J = args.J, K = args.K, L = args.L;
    const T *Bi = args.B + i * J * K;
    const T *Dt = args.Dt + n0 * args.Kpad;

    const int nks = (int)((K + BK - 1) / BK);
    const int ntiles = (int)((j_end - j_begin + BM - 1) / BM);

    vec_t rs[Cfg::PER_T];

    // slab (jt, ks): rows [0, BM) from B(i, j0.., k0..), rows [BM, BM+32) from Dt(.., k0..)
    auto load_global = [&](int jt, int ks) {
        const int64_t j0 = j_begin + (int64_t)jt * BM, k0 = (int64_t)ks * BK;
#pragma unroll
        for (int p = 0; p < Cfg::PER_T; ++p) {
            const int v = tid + p * NT;
            const int r = v / (BK / VEC), kv = v % (BK / VEC);
            if (p < Cfg::B_PER_T) {
                if constexpr (!GUARD) {
                    rs[p] = __builtin_nontemporal_load(
                        reinterpret_cast<const vec_t *>(Bi + (j0 + r) * K + k0 + kv * VEC));
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const int64_t j = j0 + r, k = k0 + kv * VEC + e;
                        rs[p][e] = (j < J && k < K) ? Bi[j * K + k] : T(0);
                    }
                }
            } else {
                rs[p] = *reinterpret_cast<const vec_t *>(Dt + (int64_t)(r - BM) * args.Kpad + k0 + kv * VEC);
            }
        }
    };

    auto store_lds = [&]() {
#pragma unroll
        for (int p = 0; p < Cfg::PER_T; ++p) {
            const int v = tid + p * NT;
            const int r = v / (BK / VEC), kv = v % (BK / VEC);
            *reinterpret_cast<vec_t *>(slab + r * Cfg::LD_S + kv * VEC) = rs[p];
        }
    };

    typename MF::acc_t acc[LB][MI];
    auto zero_acc = [&]() {
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) acc[lb][mi][v] = T(0);
    };
    zero_acc();
    T lsum[LB][MF::NACC];                 // running sum for l = mttkrp_l_of(v, lb, lane)
#pragma unroll
    for (int lb = 0; lb < LB; ++lb)
#pragma unroll
        for (int v = 0; v < MF::NACC; ++v) lsum[lb][v] = T(0);

    // this wavefront's quarter of the slab's k range; lane (li, ls) reads k-slot ls
    const int koff = wave * Cfg::KG_PER_WAVE * KG + ls * KV;
    const T *b_rd = slab + li * Cfg::LD_S + koff;                               // B rows (j)
    const T *d_rd = slab + (BM + (LB == 1 ? li : 2 * li)) * Cfg::LD_S + koff;   // Dt rows (l)

    auto compute = [&]() {
#pragma unroll
        for (int g = 0; g < Cfg::KG_PER_WAVE; ++g) {
            vec_t b[MI], d[LB];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                b[mi] = *reinterpret_cast<const vec_t *>(b_rd + mi * MF::NB * Cfg::LD_S + g * KG);
#pragma unroll
            for (int lb = 0; lb < LB; ++lb)
                d[lb] = *reinterpret_cast<const vec_t *>(d_rd + lb * Cfg::LD_S + g * KG);
#pragma unroll
            for (int t = 0; t < KV; ++t)
#pragma unroll
                for (int lb = 0; lb < LB; ++lb)
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        acc[lb][mi] = MF::run(d[lb][t], b[mi][t], acc[lb][mi]);
        }
    };

    // Scale this tile's Tt(l, j) by C(j, l) and add into the lane's running sums.
    auto fold_tile = [&](int jt) {
        const int64_t j0 = j_begin + (int64_t)jt * BM;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int64_t j = j0 + mi * MF::NB + li;
            if constexpr (!GUARD) {
                const T *crow = args.C + j * L + n0;
                vec_t c[4];
                if constexpr (sizeof(T) == 4) {
                    // lane owns l = 8q + 4*ls + r: four neighbours per q
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        c[q] = *reinterpret_cast<const vec_t *>(crow + 8 * q + 4 * ls);
#pragma unroll
                    for (int v = 0; v < MF::NACC; ++v)
                        lsum[0][v] = fma_t(acc[0][mi][v], c[v >> 2][v & 3], lsum[0][v]);
                } else {
                    // lane owns l = 2*(4v + ls) + lb: two neighbours per v
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        c[v] = *reinterpret_cast<const vec_t *>(crow + 2 * (4 * v + ls));
#pragma unroll
                    for (int v = 0; v < MF::NACC; ++v)
#pragma unroll
                        for (int lb = 0; lb < LB; ++lb)
                            lsum[lb][v] = fma_t(acc[lb][mi][v], c[v][lb], lsum[lb][v]);
                }
            } else {
#pragma unroll
                for (int lb = 0; lb < LB; ++lb)
#pragma unroll
                    for (int v = 0; v < MF::NACC; ++v) {
                        const int64_t l = n0 + mttkrp_l_of<T>(v, lb, lane);
                        const T f = (j < J && l < L) ? args.C[j * L + l] : T(0);
                        lsum[lb][v] = fma_t(acc[lb][mi][v], f, lsum[lb][v]);
                    }
            }
        }
        zero_acc();
    };

    int jt = 0, ks = 0;
    if (ntiles > 0 && nks > 0) load_global(0, 0);
    while (jt < ntiles && nks > 0) {
        int njt = jt, nks_next = ks + 1;
        if (nks_next == nks) { nks_next = 0; njt = jt + 1; }
        const bool more = njt < ntiles;
        __syncthreads();                 // everyone is done reading the previous slab
        store_lds();
        // past the end: a redundant reload of the last slab, never out of bounds
        load_global(more ? njt : jt, more ? nks_next : ks);
        __syncthreads();                 // slab visible
        compute();
        if (nks_next == 0) fold_tile(jt);
        jt = njt;
        ks = nks_next;
    }

    // lane sums -> LDS -> one sum per l, in a fixed order (two stages)
    __syncthreads();
    T *red = slab;                        // [NSUM][256]
#pragma unroll
    for (int lb = 0; lb < LB; ++lb)
#pragma unroll
        for (int v = 0; v < MF::NACC; ++v) red[(lb * MF::NACC + v) * NT + tid] = lsum[lb][v];
    __syncthreads();
    // thread (part, l): l = tid % 32 is owned by the lanes of one k-slot, in one element (lb, v)
    const int l = tid & 31, part = tid >> 5;                  // 8 parts
    int ls_l, v_l, lb_l;
    if (sizeof(T) == 4) { ls_l = (l >> 2) & 1; v_l = 4 * (l >> 3) + (l & 3); lb_l = 0; }
    else { lb_l = l & 1; ls_l = (l >> 1) & 3; v_l = l >> 3; }
    const T *src = red + (lb_l * MF::NACC + v_l) * NT;
    // owners: wave w, lane ls_l*MB + x; each part adds a fixed eighth of them, in order
    constexpr int OWNERS = 4 * MF::MB, PER_PART = OWNERS / 8;
    T s = T(0);
#pragma unroll
    for (int o = 0; o < PER_PART; ++o) {
        const int idx = part * PER_PART + o;
        s += src[(idx / MF::MB) * 64 + ls_l * MF::MB + (idx % MF::MB)];
    }
    __syncthreads();
    red[tid] = s;                                              // [8 parts][32]
    __syncthreads();
    if (tid < BN && n0 + tid < L) {
        T tot = T(0);
#pragma unroll
        for (int p = 0; p < 8; ++p) tot += red[p * 32 + tid];
        args.partial[ic * L + n0 + tid] = tot;
    }
}

}  // namespace distal
