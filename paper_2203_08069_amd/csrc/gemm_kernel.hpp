// MFMA contraction kernel for gfx950: one template serves the matrix-multiply
// tile step and TTM (the same contraction on the (I*J) x K view of the tensor).
//
// Work decomposition
//   grid   : one workgroup per BM x BN output tile, block ids remapped so that
//            each of the 8 XCDs (one L2 each) works a compact group of tiles
//   block  : WAVES_M x WAVES_N wavefronts of 64 lanes, each owning a
//            (BM/WAVES_M) x (BN/WAVES_N) sub-tile held in MFMA accumulators
//   k-loop : BK-deep slabs of both operands, global -> registers -> LDS, two LDS
//            buffers, one barrier per slab; the next slab's global loads are in
//            flight while the current one is multiplied (buffer loads: the slab's
//            base in scalar registers, a fixed 32-bit offset per lane)
//   MFMA   : binary64 16x16x4; binary32 32x32x2 on the large tiles and 16x16x4 (FINE)
//            on tiles up to 128 x 128, which are cut into eight wavefronts
//   two kernels: contract_kernel checks bounds and alignment per tile and serves any
//            shape; contract_fast_kernel assumes whole aligned tiles and has a
//            straight-line k-loop
//
// Operand-to-lane assignment.  An MFMA contracts KS "k-slots" held by different
// lane groups.  Which k a slot carries is free as long as both operands agree,
// so slot s of the t-th MFMA of a group of KG = KS*KV k-values carries
// k = s*KV + t: a lane then reads its KV values for KV consecutive MFMAs as ONE
// 16-byte LDS read of the row-major A slab.  In the same way the CV column
// blocks that share an LDS read take interleaved columns (lane jj of block q
// owns column jj*CV + q), so a lane reads CV neighbouring B values at once and
// finally owns CV neighbouring outputs, which it stores as one vector.
//
// TA = true contracts over the ROWS of the left operand (C = At^T * B with At stored
// K x M, row-major): the contractions over a non-last mode of a tensor have this
// form.  The left slab is then staged like the right one (k rows, m contiguous) and
// read the same way: RV row blocks that share an LDS read own interleaved rows.
// blockIdx.y selects one problem of a batch (operands advance by fixed strides).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tile_map.hpp"

namespace distal {

typedef double v2d __attribute__((ext_vector_type(2)));
typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <typename T, int N> struct VecOf;
template <> struct VecOf<double, 1> { typedef double type; };
template <> struct VecOf<double, 2> { typedef v2d type; };
template <> struct VecOf<float, 1> { typedef float type; };
template <> struct VecOf<float, 2> { typedef v2f type; };
template <> struct VecOf<float, 4> { typedef v4f type; };

// The same vectors as they sit in global memory: only element-aligned.  Operands may be views
// whose base or leading dimension is not a multiple of 16 bytes; the hardware serves such
// accesses with the same wide instruction, so the kernels make no alignment promise for them.
template <typename T, int N> struct GlobalVecOf {
    typedef typename VecOf<T, N>::type type __attribute__((aligned(sizeof(T))));
};

// Fused multiply-add in the element type (the unsuffixed builtin is binary64 only).
__device__ __forceinline__ float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }

// Per-dtype MFMA shape and register layout.
//   lane -> (row-or-column index within the block, k-slot) for the operands;
//   accumulator register v of a lane -> output row within the block.
template <typename T> struct Mfma;

template <> struct Mfma<double> {          // v_mfma_f64_16x16x4_f64
    static constexpr int MB = 16, NB = 16, KS = 4, NACC = 4;
    typedef v4d acc_t;
    static __device__ __forceinline__ acc_t run(double a, double b, acc_t c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int out_row(int v, int lane) { return 4 * v + (lane >> 4); }
};

template <> struct Mfma<float> {           // v_mfma_f32_32x32x2_f32
    static constexpr int MB = 32, NB = 32, KS = 2, NACC = 16;
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int out_row(int v, int lane) {
        return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    }
};

template <typename T>
struct ContractArgs {
    const T *A;          // left operand: M x K (TA = false) or K x M (TA = true), row stride lda
    const T *B;          // right operand (K x N), row stride ldb
    T *C;                // output (M x N), row stride ldc
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    int accumulate;
    int tiles_m, tiles_n;
    int a_vec_ok, b_vec_ok, c_vec_ok;   // 16-byte vector access is legal on that operand
    int64_t batch_a, batch_b, batch_c;  // element strides between the problems of a batch (blockIdx.y)
    int64_t n_before;    // columns of the same rows of B that lie before B (a product that is the right
                         // part of a wider one): the straight-line kernel may read back into them
};

// binary32 also has the 16 x 16 x 4 instruction, at the same rate: four times as many blocks per
// tile, so a small tile can be cut into eight wavefronts that still own 2 x 2 blocks each (FINE).
struct MfmaFineF32 {                       // v_mfma_f32_16x16x4_f32
    static constexpr int MB = 16, NB = 16, KS = 4, NACC = 4;
    typedef v4f acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int out_row(int v, int lane) { return 4 * (lane >> 4) + v; }
};
template <typename T, bool FINE> struct MfmaPick { typedef Mfma<T> type; };
template <> struct MfmaPick<float, true> { typedef MfmaFineF32 type; };

template <typename T, int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TA = false, bool FINE = false>
struct ContractCfg {
    typedef typename MfmaPick<T, FINE>::type MF;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int VEC = 16 / (int)sizeof(T);      // elements per 16-byte access
    static constexpr int KV = VEC;                        // consecutive k per lane per A read
    static constexpr int KG = MF::KS * KV;                // k-values per MFMA group
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int MI = WTM / MF::MB, NI = WTN / MF::NB;
    static constexpr int CV = (NI % 2 == 0) ? 2 : 1;      // column blocks sharing one B read
    static constexpr int NG = NI / CV;
    static constexpr int RV = (TA && MI % 2 == 0) ? 2 : 1; // row blocks sharing one A read (TA only)
    static constexpr int MG = MI / RV;
    // LDS row strides (elements), chosen with the bank-conflict counter.  binary32: every row padded
    // by 16 bytes, no conflicts.  binary64, whose operand reads are 16 bytes per lane: that pad on the
    // wide rows (BN elements of the right slab, BM of a transposed left one) put 40 % of the LDS
    // cycles into conflicts and is left out; the BK-long rows of a left slab take 32 bytes (with 16,
    // 18 % conflicts remained; with 32, none).  8192^3: 91.2 -> 92.3 % of peak, k-steps of 256: +1.2.
    static constexpr int WIDE_PAD = sizeof(T) == 8 ? 0 : VEC;
    static constexpr int LDA_S = TA ? BM + WIDE_PAD : BK + (sizeof(T) == 8 ? 2 * VEC : VEC);
    static constexpr int LDB_S = BN + WIDE_PAD;
    static constexpr int A_ROWLEN = TA ? BM : BK;         // contiguous elements per staged A row
    static constexpr int A_ELEMS = (TA ? BK : BM) * LDA_S, B_ELEMS = BK * LDB_S;
    static constexpr int STAGE_ELEMS = A_ELEMS + B_ELEMS;
    static constexpr int LDS_BYTES = 2 * STAGE_ELEMS * (int)sizeof(T);
    static constexpr int A_VECS = BM * (BK / VEC), B_VECS = BK * (BN / VEC);
    static constexpr int A_PER_T = (A_VECS + NT - 1) / NT, B_PER_T = (B_VECS + NT - 1) / NT;
    static constexpr int GROUP_M = (BM > BN) ? 4 : 8;     // tile rows per band (see tile_of_block)
    static constexpr bool TRANS_A = TA;
    static_assert(BM % (WAVES_M * MF::MB) == 0 && BN % (WAVES_N * MF::NB) == 0, "tile shape");
    static_assert(BK % KG == 0, "BK must hold whole MFMA k-groups");
};


// Lane offsets (elements) of the operand reads inside a staged slab pair.
template <typename Cfg>
__device__ __forceinline__ int a_read_offset(int wm, int li, int ls) {
    if constexpr (Cfg::TRANS_A) return (ls * Cfg::KV) * Cfg::LDA_S + wm * Cfg::WTM + li * Cfg::RV;
    else return (wm * Cfg::WTM + li) * Cfg::LDA_S + ls * Cfg::KV;
}
template <typename Cfg>
__device__ __forceinline__ int b_read_offset(int wn, int li, int ls) {
    return Cfg::A_ELEMS + (ls * Cfg::KV) * Cfg::LDB_S + wn * Cfg::WTN + li * Cfg::CV;
}

// Output row (within the wavefront's sub-tile) of accumulator register v of row block mi.
template <typename Cfg>
__device__ __forceinline__ int sub_tile_row(int mi, int v, int lane) {
    typedef typename Cfg::MF MF;
    if constexpr (Cfg::TRANS_A)
        return (mi / Cfg::RV) * (MF::MB * Cfg::RV) + MF::out_row(v, lane) * Cfg::RV + mi % Cfg::RV;
    else
        return mi * MF::MB + MF::out_row(v, lane);
}

// MFMA k-groups [KG_LO, KG_HI) of one staged slab pair; `as` and `bs` point at the lane's
// read positions (a_read_offset / b_read_offset) of that stage.
template <typename T, typename Cfg, int KG_LO, int KG_HI>
__device__ __forceinline__ void mfma_groups(const T *as, const T *bs,
                                            typename Cfg::MF::acc_t (&acc)[Cfg::MI][Cfg::NI]) {
    typedef typename Cfg::MF MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    typedef typename VecOf<T, Cfg::CV>::type cvec_t;
    typedef typename VecOf<T, Cfg::RV>::type rvec_t;
    constexpr int KV = Cfg::KV, KG = Cfg::KG, MI = Cfg::MI, NI = Cfg::NI, CV = Cfg::CV, NG = Cfg::NG;
    constexpr int RV = Cfg::RV, MG = Cfg::MG;
#pragma unroll
    for (int kg = KG_LO; kg < KG_HI; ++kg) {
        T av[KV][MI];
        if constexpr (!Cfg::TRANS_A) {
            vec_t a[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                a[mi] = *reinterpret_cast<const vec_t *>(as + mi * MF::MB * Cfg::LDA_S + kg * KG);
#pragma unroll
            for (int t = 0; t < KV; ++t)
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) av[t][mi] = a[mi][t];
        } else {
            rvec_t a[KV][MG];
#pragma unroll
            for (int t = 0; t < KV; ++t)
#pragma unroll
                for (int h = 0; h < MG; ++h)
                    a[t][h] = *reinterpret_cast<const rvec_t *>(as + (kg * KG + t) * Cfg::LDA_S
                                                                + h * MF::MB * RV);
#pragma unroll
            for (int t = 0; t < KV; ++t)
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    if constexpr (RV == 1) av[t][mi] = a[t][mi];
                    else av[t][mi] = a[t][mi / RV][mi % RV];
                }
        }
        cvec_t b[KV][NG];
#pragma unroll
        for (int t = 0; t < KV; ++t)
#pragma unroll
            for (int g = 0; g < NG; ++g)
                b[t][g] = *reinterpret_cast<const cvec_t *>(bs + (kg * KG + t) * Cfg::LDB_S
                                                            + g * MF::NB * CV);
#pragma unroll
        for (int t = 0; t < KV; ++t)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    T bv;
                    if constexpr (CV == 1) bv = b[t][ni];
                    else bv = b[t][ni / CV][ni % CV];
                    acc[mi][ni] = MF::run(av[t][mi], bv, acc[mi][ni]);
                }
    }
}

template <typename T, int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TA = false>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N, 2)
contract_kernel(ContractArgs<T> args) {
    typedef ContractCfg<T, BM, BN, BK, WAVES_M, WAVES_N, TA> Cfg;
    typedef Mfma<T> MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    typedef typename VecOf<T, Cfg::CV>::type cvec_t;
    constexpr int VEC = Cfg::VEC, KG = Cfg::KG, MI = Cfg::MI, NI = Cfg::NI;
    constexpr int CV = Cfg::CV, NG = Cfg::NG, NT = Cfg::NT;
    constexpr int ARL = Cfg::A_ROWLEN / VEC;          // 16-byte pieces per staged A row

    args.A += (int64_t)blockIdx.y * args.batch_a;
    args.B += (int64_t)blockIdx.y * args.batch_b;
    args.C += (int64_t)blockIdx.y * args.batch_c;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int li = lane % MF::MB;          // row (A) / column (B) index inside an MFMA block
    const int ls = lane / MF::MB;          // k-slot

    int tm, tn;
    tile_of_block<Cfg::GROUP_M>(blockIdx.x, gridDim.x, args.tiles_m, args.tiles_n, tm, tn);

    const int64_t m0 = (int64_t)tm * BM, mlimit = args.M;
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t K = args.K;

    const bool a_fast = args.a_vec_ok && (m0 + BM <= mlimit);
    const bool b_fast = args.b_vec_ok && (n0 + BN <= args.N);

    // the next slab waits in these registers while it is in flight from HBM/L2
    vec_t ra_next[Cfg::A_PER_T], rb_next[Cfg::B_PER_T];

    auto load_global = [&](vec_t (&ra)[Cfg::A_PER_T], vec_t (&rb)[Cfg::B_PER_T], int64_t k0) {
        const bool kfull = (k0 + BK <= K);
        if (a_fast && kfull) {
#pragma unroll
            for (int p = 0; p < Cfg::A_PER_T; ++p) {
                const int v = tid + p * NT;
                if (Cfg::A_VECS % NT != 0 && v >= Cfg::A_VECS) break;
                const int r = v / ARL, kv = v % ARL;
                if constexpr (TA)
                    ra[p] = *reinterpret_cast<const vec_t *>(args.A + (k0 + r) * args.lda + m0 + kv * VEC);
                else
                    ra[p] = *reinterpret_cast<const vec_t *>(args.A + (m0 + r) * args.lda + k0 + kv * VEC);
            }
        } else {
#pragma unroll
            for (int p = 0; p < Cfg::A_PER_T; ++p) {
                const int v = tid + p * NT;
                if (Cfg::A_VECS % NT != 0 && v >= Cfg::A_VECS) break;
                const int r = v / ARL, kv = v % ARL;
                T tmp[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    if constexpr (TA) {
                        const int64_t k = k0 + r, row = m0 + kv * VEC + e;
                        tmp[e] = (row < mlimit && k < K) ? args.A[k * args.lda + row] : T(0);
                    } else {
                        const int64_t row = m0 + r, k = k0 + kv * VEC + e;
                        tmp[e] = (row < mlimit && k < K) ? args.A[row * args.lda + k] : T(0);
                    }
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) ra[p][e] = tmp[e];
            }
        }
        if (b_fast && kfull) {
#pragma unroll
            for (int p = 0; p < Cfg::B_PER_T; ++p) {
                const int v = tid + p * NT;
                if (Cfg::B_VECS % NT != 0 && v >= Cfg::B_VECS) break;
                const int r = v / (BN / VEC), cv = v % (BN / VEC);
                rb[p] = *reinterpret_cast<const vec_t *>(args.B + (k0 + r) * args.ldb + n0 + cv * VEC);
            }
        } else {
#pragma unroll
            for (int p = 0; p < Cfg::B_PER_T; ++p) {
                const int v = tid + p * NT;
                if (Cfg::B_VECS % NT != 0 && v >= Cfg::B_VECS) break;
                const int r = v / (BN / VEC), cv = v % (BN / VEC);
                T tmp[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int64_t k = k0 + r, col = n0 + cv * VEC + e;
                    tmp[e] = (k < K && col < args.N) ? args.B[k * args.ldb + col] : T(0);
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) rb[p][e] = tmp[e];
            }
        }
    };

    auto store_lds = [&](const vec_t (&ra)[Cfg::A_PER_T], const vec_t (&rb)[Cfg::B_PER_T], int stage) {
        T *as = lds + stage * Cfg::STAGE_ELEMS;
        T *bs = as + Cfg::A_ELEMS;
#pragma unroll
        for (int p = 0; p < Cfg::A_PER_T; ++p) {
            const int v = tid + p * NT;
            if (Cfg::A_VECS % NT != 0 && v >= Cfg::A_VECS) break;
            const int r = v / ARL, kv = v % ARL;
            *reinterpret_cast<vec_t *>(as + r * Cfg::LDA_S + kv * VEC) = ra[p];
        }
#pragma unroll
        for (int p = 0; p < Cfg::B_PER_T; ++p) {
            const int v = tid + p * NT;
            if (Cfg::B_VECS % NT != 0 && v >= Cfg::B_VECS) break;
            const int r = v / (BN / VEC), cv = v % (BN / VEC);
            *reinterpret_cast<vec_t *>(bs + r * Cfg::LDB_S + cv * VEC) = rb[p];
        }
    };

    typename MF::acc_t acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) acc[mi][ni][v] = T(0);

    const int a_rd = a_read_offset<Cfg>(wm, li, ls), b_rd = b_read_offset<Cfg>(wn, li, ls);
    auto compute = [&](int stage) {
        const T *st = lds + stage * Cfg::STAGE_ELEMS;
        mfma_groups<T, Cfg, 0, BK / KG>(st + a_rd, st + b_rd, acc);
    };

    // Slab t+1 sits in registers while slab t is multiplied; once it has been written to
    // the idle LDS buffer the registers are refilled with slab t+2.  Slab indices past the
    // end are clamped to the last slab: those loads are redundant cache hits, never out of
    // bounds, and keep the loop free of divergence.
    const int64_t nk = (K + BK - 1) / BK;
    auto k_of = [&](int64_t t) { return (t < nk ? t : nk - 1) * BK; };
    if (nk > 0) {
        load_global(ra_next, rb_next, k_of(0));
        store_lds(ra_next, rb_next, 0);
        load_global(ra_next, rb_next, k_of(1));
    }
    __syncthreads();
    for (int64_t t = 0; t < nk; ++t) {
        const int stage = (int)(t & 1);
        compute(stage);
        if (t + 1 < nk) store_lds(ra_next, rb_next, stage ^ 1);
        load_global(ra_next, rb_next, k_of(t + 2));
        __syncthreads();
    }

    // epilogue: accumulators -> C, CV neighbouring columns per store
    const bool c_fast = args.c_vec_ok && (m0 + BM <= args.M) && (n0 + BN <= args.N);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) {
                const int64_t row = m0 + wm * Cfg::WTM + sub_tile_row<Cfg>(mi, v, lane);
                const int64_t col = n0 + wn * Cfg::WTN + g * (MF::NB * CV) + li * CV;
                T *cp = args.C + row * args.ldc + col;
                if (c_fast) {
                    cvec_t o;
                    if constexpr (CV == 1) {
                        o = acc[mi][g][v];
                        if (args.accumulate) o += *cp;
                        *cp = o;
                    } else {
#pragma unroll
                        for (int q = 0; q < CV; ++q) o[q] = acc[mi][g * CV + q][v];
                        if (args.accumulate) o += *reinterpret_cast<const cvec_t *>(cp);
                        *reinterpret_cast<cvec_t *>(cp) = o;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < CV; ++q) {
                        if (row < args.M && col + q < args.N) {
                            T o = acc[mi][g * CV + q][v];
                            if (args.accumulate) o += cp[q];
                            cp[q] = o;
                        }
                    }
                }
            }
}

// ---------------------------------------------------------------------------
// The same contraction for the case every tile and slab is full and every operand
// 16-byte aligned (M % BM == 0, N % BN == 0, K % BK == 0, aligned bases and leading
// dimensions).  No bounds checks and no branches inside the k-loop: its body is one
// straight-line block, so the LDS writes of the next slab and the global loads of the
// slab after it are issued between the MFMAs of the current slab, in the issue slots
// the 64-cycle MFMAs leave free, instead of in a burst of their own.
//
// EDGE = true serves M and N that are not whole tiles at no cost in the k-loop: a 16-byte
// piece that lies past the edge is fetched from the last valid row (or last valid piece of a
// row) instead, so every load stays in bounds and the rows and columns it feeds hold values
// that no valid output depends on; the epilogue stores only what lies inside M x N.
// Pieces must not straddle an edge: N (and M, when TA) a multiple of the 16-byte vector - except
// in the SHIFT forms of the edge kernels, which take an N that is not (N % VEC != 0, and N - VEC
// columns or more exist in B's rows counting those before the pointer): the piece that straddles
// the end of a row of B is fetched VEC columns before the end and shifted in registers, and the
// last column of C is accessed on its own.  The shift costs the k-loop about 3 %, which is why
// it is a form of its own.
// EDGE = 2 also takes K >= BK that is not a multiple of BK (without TA: a multiple of the
// vector, pieces of A run along k): the trailing terms are one zero-filled slab after the loop.
// In the other forms K is a multiple of BK.
//
// ACC_INIT = true is the accumulating product (args.accumulate is taken as set) with the old
// values of C loaded into the accumulators before the first slab instead of added in the
// epilogue, which then only stores: nothing is waited for at the end of a tile.  That pays
// where the k-loop is short and the tile small - binary32, tiles up to 128 x 128, at most 256
// terms (64 x 128 tiles at K = 128: +7 %) - and costs 1..4 % everywhere else (the loads then
// sit in front of the first multiply with nothing to hide behind), so the host launches this
// form there only; binary64 shows no gain at any shape and always adds in the epilogue.
// ---------------------------------------------------------------------------
template <typename T, int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TA = false, int EDGE = 0, bool ACC_INIT = false,
          bool FINE = false, bool SHIFT = false>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N, (WAVES_M * WAVES_N >= 8) ? 4 : 2)
contract_fast_kernel(ContractArgs<T> args) {
    typedef ContractCfg<T, BM, BN, BK, WAVES_M, WAVES_N, TA, FINE> Cfg;
    typedef typename Cfg::MF MF;
    typedef typename VecOf<T, Cfg::VEC>::type vec_t;
    typedef typename VecOf<T, Cfg::CV>::type cvec_t;
    typedef typename GlobalVecOf<T, Cfg::CV>::type gcvec_t;
    constexpr int VEC = Cfg::VEC, KG = Cfg::KG, MI = Cfg::MI, NI = Cfg::NI;
    constexpr int CV = Cfg::CV, NG = Cfg::NG, NT = Cfg::NT, NKG = BK / KG;
    constexpr int ARL = Cfg::A_ROWLEN / VEC;          // 16-byte pieces per staged A row
    // rank-sized tiles, and the binary64 64 x 64 tile in its eight-wavefront cut (grids of at most two
    // tiles per compute unit): two slabs of loads in flight
    constexpr bool DEEP = BM == 32 || BN == 32 || (sizeof(T) == 8 && BM * BN == 64 * 64 && WAVES_M * WAVES_N == 8);
    static_assert(Cfg::A_VECS % NT == 0 && Cfg::B_VECS % NT == 0, "slab vectors must divide over threads");

    args.A += (int64_t)blockIdx.y * args.batch_a;
    args.B += (int64_t)blockIdx.y * args.batch_b;
    args.C += (int64_t)blockIdx.y * args.batch_c;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int li = lane % MF::MB, ls = lane / MF::MB;

    int tm, tn;
    tile_of_block<Cfg::GROUP_M>(blockIdx.x, gridDim.x, args.tiles_m, args.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    const int64_t nk = args.K / BK;

    // Per-thread byte offsets of its 16-byte pieces from the tile's first row and column, and where
    // they go in LDS.  The loads are buffer loads: the slab's base travels in a descriptor in scalar
    // registers and a lane supplies its 32-bit offset, which never changes, so no vector arithmetic
    // is spent on addresses inside the k-loop (with 64-bit pointers per lane the loop held three
    // 64-bit vector adds per load; together with the constant LDS buffers of the two-slab trip
    // below their removal was worth 2.4 points at 8192^3 and 5 to 9 at 2000^3...3000^3).  The offsets
    // are unsigned 32-bit: the host launches this kernel only where (rows of a slab - 1) x leading
    // dimension fits (slab_offsets_fit of the host-side planning), and bounds checking by the descriptor is off (its range is
    // the whole 4 GiB): every address is in bounds by construction, exactly as with pointers.
    int a_off[Cfg::A_PER_T], b_off[Cfg::B_PER_T];
    int a_lds[Cfg::A_PER_T], b_lds[Cfg::B_PER_T];
    const char *a_tile = reinterpret_cast<const char *>(args.A + (TA ? m0 : m0 * args.lda));
    // the B offsets count from column nb: n0, or N - VEC where the last tile is narrower than a piece
    const int64_t nb = (SHIFT && n0 > args.N - VEC) ? args.N - VEC : n0;
    const char *b_tile = reinterpret_cast<const char *>(args.B + nb);
#pragma unroll
    for (int p = 0; p < Cfg::A_PER_T; ++p) {
        const int v = tid + p * NT, r = v / ARL, kv = v % ARL;
        if constexpr (TA) {
            int64_t m = m0 + kv * VEC;
            if (EDGE && m > args.M - VEC) m = args.M - VEC;
            a_off[p] = (int)(unsigned)(((int64_t)r * args.lda + (m - m0)) * (int64_t)sizeof(T));
        } else {
            int64_t m = m0 + r;
            if (EDGE && m > args.M - 1) m = args.M - 1;
            a_off[p] = (int)(unsigned)(((m - m0) * args.lda + kv * VEC) * (int64_t)sizeof(T));
        }
        a_lds[p] = r * Cfg::LDA_S + kv * VEC;
    }
    // N that is not a multiple of the vector (the SHIFT forms, which are EDGE forms): the piece that
    // holds the last N % VEC columns is fetched from column N - VEC like the pieces past the edge,
    // and on its way to LDS its values move down by n_shift places, so the valid columns sit where
    // the multiply expects them (what follows them in the piece feeds columns that are never stored).
    static_assert(!SHIFT || EDGE != 0, "only the edge forms shift");
    const int n_shift = SHIFT ? (VEC == 2 ? 1 : (int)(VEC - args.N % VEC)) : 0;     // block-uniform, 1 ... VEC - 1
    bool b_fix[Cfg::B_PER_T];
#pragma unroll
    for (int p = 0; p < Cfg::B_PER_T; ++p) {
        const int v = tid + p * NT, r = v / (BN / VEC), cv = v % (BN / VEC);
        int64_t n = n0 + cv * VEC;
        b_fix[p] = SHIFT && n == args.N - args.N % VEC;
        if (EDGE && n > args.N - VEC) n = args.N - VEC;
        b_off[p] = (int)(unsigned)(((int64_t)r * args.ldb + (n - nb)) * (int64_t)sizeof(T));
        b_lds[p] = Cfg::A_ELEMS + r * Cfg::LDB_S + cv * VEC;
    }
    auto b_piece = [&](const vec_t &x, int p) -> vec_t {       // the piece as it goes to LDS
        if constexpr (!SHIFT) return x;
        vec_t y = x;                                            // y[e] = x[e + n_shift] where that exists
        if constexpr (VEC == 2) {
            y[0] = x[1];
        } else {
            y[0] = n_shift == 1 ? x[1] : (n_shift == 2 ? x[2] : x[3]);
            y[1] = n_shift == 1 ? x[2] : x[3];
            y[2] = x[3];
        }
        return b_fix[p] ? y : x;
    };
    // raw buffer, no stride, the full 32-bit range; word 3 is the 32-bit data format of this family
    auto slab_rsrc = [&](const char *base) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, -1, 0x00020000);
    };

    vec_t ra[Cfg::A_PER_T], rb[Cfg::B_PER_T];
    // slab index past the end is clamped to the last slab: a redundant, in-bounds reload
    auto load_into = [&](vec_t (&xa)[Cfg::A_PER_T], vec_t (&xb)[Cfg::B_PER_T], int64_t t) {
        const int64_t k0 = (t < nk ? t : nk - 1) * BK;
        const auto ar = slab_rsrc(a_tile + (TA ? k0 * args.lda : k0) * (int64_t)sizeof(T));
        const auto br = slab_rsrc(b_tile + k0 * args.ldb * (int64_t)sizeof(T));
#pragma unroll
        for (int p = 0; p < Cfg::A_PER_T; ++p)
            xa[p] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(ar, a_off[p], 0, 0));
#pragma unroll
        for (int p = 0; p < Cfg::B_PER_T; ++p)
            xb[p] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(br, b_off[p], 0, 0));
    };
    auto load_global = [&](int64_t t) { load_into(ra, rb, t); };
    auto store_lds = [&](int stage) {
        T *st = lds + stage * Cfg::STAGE_ELEMS;
#pragma unroll
        for (int p = 0; p < Cfg::A_PER_T; ++p) *reinterpret_cast<vec_t *>(st + a_lds[p]) = ra[p];
#pragma unroll
        for (int p = 0; p < Cfg::B_PER_T; ++p) *reinterpret_cast<vec_t *>(st + b_lds[p]) = b_piece(rb[p], p);
    };

    typename MF::acc_t acc[MI][NI];
    if constexpr (ACC_INIT) {
        // the accumulators start from the old values of C, requested ahead of the first slabs
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) {
                    const int64_t row = m0 + wm * Cfg::WTM + sub_tile_row<Cfg>(mi, v, lane);
                    const int64_t col = n0 + wn * Cfg::WTN + g * (MF::NB * CV) + li * CV;
                    const bool inside = !EDGE || (row < args.M && col < args.N);
                    const T *cp = args.C + row * args.ldc + col;
                    if constexpr (CV == 1) {
                        acc[mi][g][v] = inside ? *cp : T(0);
                    } else {
                        cvec_t o = cvec_t(T(0));
                        if (inside && (!SHIFT || col + CV <= args.N)) o = *reinterpret_cast<const gcvec_t *>(cp);
                        else if (inside) o[0] = *cp;            // the row's last column: CV is 2
#pragma unroll
                        for (int q = 0; q < CV; ++q) acc[mi][g * CV + q][v] = o[q];
                    }
                }
    } else {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < MF::NACC; ++v) acc[mi][ni][v] = T(0);
    }

    const int a_rd = a_read_offset<Cfg>(wm, li, ls), b_rd = b_read_offset<Cfg>(wn, li, ls);

    if constexpr (DEEP) {
        // Narrow tiles do 16 flop per byte of the large operand: the product is bound by HBM, and one
        // slab in flight per workgroup is too little to cover its latency.  (The same holds for a small
        // tile that is alone on its compute unit: a slab of a 64 x 64 tile is multiplied in less time
        // than a load takes.  Measured in one process: binary64 1000^3 59 -> 65 % of peak, 1024 x 1024 x
        // 8192 82.8 -> 86.5; the four-wavefront cut for larger grids loses two points with it - 3000^3
        // 86.4 -> 84.4 - and the binary32 tiles neither gain nor lose, so they stay as they were.)
        // Two register sets: slab
        // t is in LDS buffer t & 1, slab t+1 in one set, slab t+2 in flight into the other, and
        // slab t+3 is requested into the first as soon as it has been copied to LDS.
        vec_t ra2[Cfg::A_PER_T], rb2[Cfg::B_PER_T];
        auto store_from = [&](const vec_t (&xa)[Cfg::A_PER_T], const vec_t (&xb)[Cfg::B_PER_T], int stage) {
            T *st = lds + stage * Cfg::STAGE_ELEMS;
#pragma unroll
            for (int p = 0; p < Cfg::A_PER_T; ++p) *reinterpret_cast<vec_t *>(st + a_lds[p]) = xa[p];
#pragma unroll
            for (int p = 0; p < Cfg::B_PER_T; ++p) *reinterpret_cast<vec_t *>(st + b_lds[p]) = b_piece(xb[p], p);
        };
        const T *st0 = lds, *st1 = lds + Cfg::STAGE_ELEMS;
        load_into(ra, rb, 0);
        store_from(ra, rb, 0);
        load_into(ra, rb, 1);
        load_into(ra2, rb2, 2);
        __syncthreads();
        int64_t t = 0;
        for (; t + 2 <= nk; t += 2) {
            mfma_groups<T, Cfg, 0, (NKG + 1) / 2>(st0 + a_rd, st0 + b_rd, acc);
            store_from(ra, rb, 1);           // slab t+1
            load_into(ra, rb, t + 3);
            mfma_groups<T, Cfg, (NKG + 1) / 2, NKG>(st0 + a_rd, st0 + b_rd, acc);
            __syncthreads();
            mfma_groups<T, Cfg, 0, (NKG + 1) / 2>(st1 + a_rd, st1 + b_rd, acc);
            store_from(ra2, rb2, 0);         // slab t+2 (on the last pass: a copy nobody reads)
            load_into(ra2, rb2, t + 4);
            mfma_groups<T, Cfg, (NKG + 1) / 2, NKG>(st1 + a_rd, st1 + b_rd, acc);
            __syncthreads();
        }
        if (t < nk) {                        // an odd number of slabs: the last one sits in buffer 0
            mfma_groups<T, Cfg, 0, NKG>(st0 + a_rd, st0 + b_rd, acc);
            __syncthreads();                 // both buffers are free again (the trailing-terms slab reuses one)
        }
    } else {
        // slab t is in LDS buffer t & 1; slab t+1 is in registers; slab t+2 is requested during the
        // multiply of slab t.  Two slabs per trip, so that the buffer of each half is a constant and
        // the LDS addresses need no arithmetic inside the loop.
        const T *st0 = lds, *st1 = lds + Cfg::STAGE_ELEMS;
        load_global(0);
        store_lds(0);
        load_global(1);
        __syncthreads();
        int64_t t = 0;
        for (; t + 2 <= nk; t += 2) {
            mfma_groups<T, Cfg, 0, (NKG + 1) / 2>(st0 + a_rd, st0 + b_rd, acc);
            store_lds(1);                // slab t+1
            load_global(t + 2);
            mfma_groups<T, Cfg, (NKG + 1) / 2, NKG>(st0 + a_rd, st0 + b_rd, acc);
            __syncthreads();
            mfma_groups<T, Cfg, 0, (NKG + 1) / 2>(st1 + a_rd, st1 + b_rd, acc);
            store_lds(0);                // slab t+2 (on the last pass: a copy nobody reads)
            load_global(t + 3);
            mfma_groups<T, Cfg, (NKG + 1) / 2, NKG>(st1 + a_rd, st1 + b_rd, acc);
            __syncthreads();
        }
        if (t < nk) {                    // an odd number of slabs: the last one sits in buffer 0
            mfma_groups<T, Cfg, 0, NKG>(st0 + a_rd, st0 + b_rd, acc);
            __syncthreads();             // both buffers are free again (the trailing-terms slab reuses one)
        }
    }

    if constexpr (EDGE == 2) {
        // the K % BK trailing terms: one more slab whose pieces past K are zero, staged after
        // the loop's last barrier (both buffers are free then) and multiplied in full
        const int tail = (int)(args.K - nk * BK);            // block-uniform
        if (tail > 0) {
            const auto ar = slab_rsrc(a_tile + (TA ? nk * BK * args.lda : nk * BK) * (int64_t)sizeof(T));
            const auto br = slab_rsrc(b_tile + nk * BK * args.ldb * (int64_t)sizeof(T));
#pragma unroll
            for (int p = 0; p < Cfg::A_PER_T; ++p) {
                const int v = tid + p * NT, r = v / ARL, kv = v % ARL;
                const bool valid = TA ? r < tail : kv * VEC < tail;
                ra[p] = valid ? __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(ar, a_off[p], 0, 0)) : vec_t(T(0));
            }
#pragma unroll
            for (int p = 0; p < Cfg::B_PER_T; ++p) {
                const int r = (tid + p * NT) / (BN / VEC);
                rb[p] = r < tail ? __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(br, b_off[p], 0, 0)) : vec_t(T(0));
            }
            store_lds(0);
            __syncthreads();
            mfma_groups<T, Cfg, 0, NKG>(lds + a_rd, lds + b_rd, acc);
        }
    }

    // epilogue: accumulators -> C, CV neighbouring columns per store.  C is streamed - read at most
    // once and written once per launch - so its accesses carry the non-temporal hint and leave the
    // caches to the operand panels, which are what is re-read (shallow k-steps under `accumulate`:
    // +2...5 %; deep products: no difference; the same hint on the up-front loads of the ACC_INIT
    // form cost 4 % at K = 128 and is not used).  (Under `accumulate` each
    // old vector is fetched right before its add; requesting them in batches ahead of the adds
    // measured 2-3 % slower on the shallow k-steps it was meant for: the other workgroup on the
    // compute unit hides the waits, and the burst only adds contention.)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < MF::NACC; ++v) {
                const int64_t row = m0 + wm * Cfg::WTM + sub_tile_row<Cfg>(mi, v, lane);
                const int64_t col = n0 + wn * Cfg::WTN + g * (MF::NB * CV) + li * CV;
                if (EDGE && (row >= args.M || col >= args.N)) continue;
                T *cp = args.C + row * args.ldc + col;
                cvec_t o;
                if constexpr (CV == 1) {
                    o = acc[mi][g][v];
                    if (!ACC_INIT && args.accumulate) o += __builtin_nontemporal_load(cp);
                    __builtin_nontemporal_store(o, cp);
                } else {
#pragma unroll
                    for (int q = 0; q < CV; ++q) o[q] = acc[mi][g * CV + q][v];
                    if (SHIFT && col + CV > args.N) {           // the row's last column on its own: CV is 2
                        T o0 = o[0];
                        if (!ACC_INIT && args.accumulate) o0 += __builtin_nontemporal_load(cp);
                        __builtin_nontemporal_store(o0, cp);
                        continue;
                    }
                    if (!ACC_INIT && args.accumulate) o += __builtin_nontemporal_load(reinterpret_cast<const gcvec_t *>(cp));
                    __builtin_nontemporal_store(o, reinterpret_cast<gcvec_t *>(cp));
                }
            }
}

}  // namespace distal
