// Bandwidth-bound kernels for gfx950: TTV and the tensor inner product.
// Both stream their tensor operands from HBM exactly once with 16-byte loads
// per lane; arithmetic and reductions are arranged so that nothing but the
// loads sits on the critical path.
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"   // vector typedefs only

namespace distal {

// Rotate within rows of 16 lanes (DPP row_ror:n) - the cross-lane step of the
// 16-lane reductions below; costs one VALU slot and no LDS traffic.
template <int N>
__device__ __forceinline__ float row_ror(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x),
                                                                  0x120 + N, 0xf, 0xf, false));
}
template <int N>
__device__ __forceinline__ double row_ror(double x) {
    const unsigned long long u = __builtin_bit_cast(unsigned long long, x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)u, 0x120 + N, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), 0x120 + N, 0xf, 0xf, false);
    return __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
}

// Sum over each aligned group of 16 lanes; every lane of the group gets the sum.
// The order of additions is fixed by the lane numbers.
template <typename T>
__device__ __forceinline__ T sum16(T x) {
    x += row_ror<8>(x);
    x += row_ror<4>(x);
    x += row_ror<2>(x);
    x += row_ror<1>(x);
    return x;
}

// Sum over the 64 lanes of a wavefront; valid in every lane.
__device__ __forceinline__ double sum64(double x) {
    x = sum16(x);
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

// ---------------------------------------------------------------------------
// TTV   A(r) = sum_k B(r, k) * c(k),  r = i*J + j  (rows of K contiguous values)
//
// 16 lanes share a row: lane q of the group reads 16-byte pieces q, q+16, ...
// of the row, so the four groups of a wavefront stream four rows at once and a
// wavefront load touches four 256-byte runs.  c is staged in LDS once per block.
// UNROLL row pieces are in flight per lane before the first multiply.
// UNALIGNED: rows and c may start at any element (K odd, views): the same 16-byte loads, typed as
// element-aligned (the hardware serves them at any element alignment), pieces counted from the
// start of each row, and the K % VEC trailing elements of a row taken by the group's first lanes.
// ---------------------------------------------------------------------------
template <typename T, int UNROLL, bool C_IN_LDS, bool UNALIGNED = false>
__global__ void __launch_bounds__(256)
ttv_vec_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
               int64_t rows, int64_t K) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    typedef typename std::conditional<UNALIGNED, typename GlobalVecOf<T, VEC>::type, vec_t>::type gvec_t;
    static_assert(!(C_IN_LDS && UNALIGNED), "the staged copy of c assumes aligned pieces");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const gvec_t *cv;
    const int64_t kvecs = K / VEC;
    if constexpr (C_IN_LDS) {
        vec_t *cl = reinterpret_cast<vec_t *>(lds_raw);
        for (int64_t v = threadIdx.x; v < kvecs; v += 256)
            cl[v] = reinterpret_cast<const vec_t *>(c)[v];
        __syncthreads();
        cv = cl;
    } else {
        cv = reinterpret_cast<const gvec_t *>(c);
    }
    const int q = threadIdx.x & 15;
    const int64_t group = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int64_t stride = (int64_t)gridDim.x * 16;
    for (int64_t r = group; r < rows; r += stride) {
        const gvec_t *row = reinterpret_cast<const gvec_t *>(B + r * K);
        T acc = T(0);
        int64_t v = q;
        // whole trips of UNROLL pieces per lane (the same count for every lane of the group) ...
        for (; v - q + 16 * UNROLL <= kvecs; v += 16 * UNROLL) {
            vec_t b[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) b[u] = __builtin_nontemporal_load(row + v + 16 * u);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const vec_t cc = cv[v + 16 * u];
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc = fma_t(b[u][e], cc[e], acc);
            }
        }
        // ... then the rest of the row in predicated trips of four
        for (; v - q < kvecs; v += 16 * 4) {
            vec_t b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                b[u] = v + 16 * u < kvecs ? __builtin_nontemporal_load(row + v + 16 * u) : vec_t(T(0));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const vec_t cc = v + 16 * u < kvecs ? cv[v + 16 * u] : vec_t(T(0));
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc = fma_t(b[u][e], cc[e], acc);
            }
        }
        if constexpr (UNALIGNED) {
            const int64_t kt = kvecs * VEC + q;
            if (kt < K) acc = fma_t(B[r * K + kt], c[kt], acc);
        }
        acc = sum16(acc);
        if (q == 0) A[r] = acc;
    }
}

// Any K, any alignment: same 16-lanes-per-row shape with element loads.
// Short rows (at most 16 pieces of 16 bytes: one piece per lane of a group).  A row then gives a
// lane a single load, so RU rows are taken at once to keep RU loads per lane in flight; the
// lane's piece of c stays in a register.
template <typename T, int RU>
__global__ void __launch_bounds__(256)
ttv_short_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                 int64_t rows, int64_t K) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    const int kvecs = (int)(K / VEC);                 // <= 16
    const int q = threadIdx.x & 15;
    const bool mine = q < kvecs;
    const vec_t cc = mine ? reinterpret_cast<const vec_t *>(c)[q] : vec_t(T(0));
    const int64_t group = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int64_t stride = (int64_t)gridDim.x * 16;
    for (int64_t r0 = group; r0 < rows; r0 += stride * RU) {
        vec_t b[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int64_t r = r0 + u * stride;
            b[u] = (mine && r < rows) ? __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(B + r * K) + q)
                                      : vec_t(T(0));
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            T acc = T(0);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc = fma_t(b[u][e], cc[e], acc);
            acc = sum16(acc);
            const int64_t r = r0 + u * stride;
            if (q == 0 && r < rows) A[r] = acc;
        }
    }
}

// One step of ttv_row_kernel: PU pieces (v, v+64, ...) of each of the RW rows r .. r+RW-1, rows
// at or past `hi` replaced by row hi-1.
template <typename T, int RW, int PU>
__device__ __forceinline__ void ttv_row_load(typename VecOf<T, 16 / (int)sizeof(T)>::type (&b)[RW][PU],
                                             const T *__restrict__ B, int64_t K, int64_t r, int64_t hi, int64_t v) {
    typedef typename VecOf<T, 16 / (int)sizeof(T)>::type vec_t;
#pragma unroll
    for (int t = 0; t < RW; ++t) {
        const vec_t *row = reinterpret_cast<const vec_t *>(B + (r + t < hi ? r + t : hi - 1) * K) + v;
#pragma unroll
        for (int u = 0; u < PU; ++u) b[t][u] = __builtin_nontemporal_load(row + 64 * u);
    }
}

// One step of ttv_row_kernel on the pieces in `cur` (rows r .., pieces v0 + lane + 64u): issues
// the next step's loads into `nxt` first, then multiplies, and when the rows are complete adds
// across the wavefront and stores.  Advances (r, v0); false when there is no next step.
template <typename T, int RW, int PU>
__device__ __forceinline__ bool ttv_row_step(typename VecOf<T, 16 / (int)sizeof(T)>::type (&cur)[RW][PU],
                                             typename VecOf<T, 16 / (int)sizeof(T)>::type (&nxt)[RW][PU],
                                             T (&acc)[RW], const T *__restrict__ B,
                                             const typename VecOf<T, 16 / (int)sizeof(T)>::type *__restrict__ cv,
                                             T *__restrict__ A, int64_t K, int64_t kvecs, int64_t hi, int lane,
                                             int64_t &r, int64_t &v0) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    int64_t v1 = v0 + 64 * PU, r1 = r;
    if (v1 >= kvecs) { v1 = 0; r1 = r + 4 * RW; }
    const bool more = r1 < hi;
    if (more) ttv_row_load<T, RW, PU>(nxt, B, K, r1, hi, v1 + lane);
#pragma unroll
    for (int u = 0; u < PU; ++u) {
        const vec_t cc = cv[v0 + lane + 64 * u];
#pragma unroll
        for (int t = 0; t < RW; ++t)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[t] = fma_t(cur[t][u][e], cc[e], acc[t]);
    }
    if (v1 == 0) {                              // the rows are complete
        T out = T(0);
#pragma unroll
        for (int t = 0; t < RW; ++t) {
            T s = sum16(acc[t]);
            s += __shfl_xor(s, 16);
            s += __shfl_xor(s, 32);
            if (lane == t) out = s;
            acc[t] = T(0);
        }
        if (lane < RW && r + lane < hi) A[r + lane] = out;
    }
    r = r1;
    v0 = v1;
    return more;
}

// Rows of at least 64 pieces, many of them: a wavefront takes RW whole rows per trip (lane l
// reads pieces l, l+64, ... of each, PU of them per row in flight, RW * PU = 8), and a workgroup
// owns a contiguous range of `per` rows (a multiple of 4 * RW), so with one workgroup per compute
// unit the chip reads 256 sequential streams - the pattern HBM serves fastest here.  c comes
// through the caches (staging it in LDS gains nothing).  K / VEC must be a multiple of 64 * PU.
// Rows past the range's end are clamped to its last row and not stored.  The loads of the next
// step are issued before the arithmetic and the reduction of the current one, so the stream
// never pauses for a row's sum.  Each row's sum is formed in an order fixed by K alone.
template <typename T, int RW, int PU>
__global__ void __launch_bounds__(256)
ttv_row_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
               int64_t rows, int64_t K, int64_t per) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    const int64_t kvecs = K / VEC;
    const vec_t *cv = reinterpret_cast<const vec_t *>(c);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t lo = (int64_t)blockIdx.x * per;
    const int64_t hi = lo + per < rows ? lo + per : rows;
    int64_t r = lo + w * RW;
    if (r >= hi) return;

    vec_t even[RW][PU], odd[RW][PU];           // steps alternate between the two register sets
    T acc[RW];
#pragma unroll
    for (int t = 0; t < RW; ++t) acc[t] = T(0);
    int64_t v0 = 0;
    ttv_row_load<T, RW, PU>(even, B, K, r, hi, v0 + lane);
    for (;;) {
        if (!ttv_row_step<T, RW, PU>(even, odd, acc, B, cv, A, K, kvecs, hi, lane, r, v0)) break;
        if (!ttv_row_step<T, RW, PU>(odd, even, acc, B, cv, A, K, kvecs, hi, lane, r, v0)) break;
    }
}

// Few, long rows: one workgroup per row (256 lanes stride the row), so that a tensor with too few
// rows for the 16-lane kernel still fills the chip.  Lanes, then wavefronts, are added in a fixed
// order.  c is read from global memory (it is as long as a row and stays in L2).
template <typename T, int UNROLL>
__global__ void __launch_bounds__(256)
ttv_wide_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                int64_t rows, int64_t K) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    __shared__ T wsum[4];
    const int64_t kvecs = K / VEC;
    const vec_t *cv = reinterpret_cast<const vec_t *>(c);
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const vec_t *row = reinterpret_cast<const vec_t *>(B + r * K);
        T acc = T(0);
        int64_t v = threadIdx.x;
        for (; v + 256 * (UNROLL - 1) < kvecs; v += 256 * UNROLL) {
            vec_t b[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) b[u] = __builtin_nontemporal_load(row + v + 256 * u);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const vec_t cc = cv[v + 256 * u];
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc = fma_t(b[u][e], cc[e], acc);
            }
        }
        for (; v < kvecs; v += 256) {
            const vec_t b = __builtin_nontemporal_load(row + v);
            const vec_t cc = cv[v];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc = fma_t(b[e], cc[e], acc);
        }
        acc = sum16(acc);
        acc += __shfl_xor(acc, 16);
        acc += __shfl_xor(acc, 32);
        __syncthreads();                       // the previous row's sums have been read
        if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
        __syncthreads();
        if (threadIdx.x == 0) A[r] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
    }
}

// TTV along a mode that is not the contiguous one, as a weighted sum of rows:
//   out(b, n) = sum_r c(r) * B(b, r, n),  n contiguous  (mode 0: b = 1, r = i, n = (j,k);
//   mode 1: b = i, r = j, n = k).
// A lane owns VEC neighbouring n of one b and walks r, UNROLL 16-byte loads in flight; what the
// lanes of a wavefront read for one r is contiguous, so the stream is fully coalesced.  Each output
// is summed by one lane in increasing r: no reduction across lanes, nothing to make deterministic.
// UNALIGNED: N >= VEC of any parity and operands at any element alignment: the same 16-byte accesses
// typed as element-aligned, and a last piece that starts at N - VEC, overlapping its neighbour (the
// outputs they share are summed twice in the same order and stored twice with the same value).
template <typename T, int UNROLL, bool UNALIGNED = false>
__global__ void __launch_bounds__(256)
ttv_left_vec_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                    int64_t batch, int64_t R, int64_t N) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename std::conditional<UNALIGNED, typename GlobalVecOf<T, VEC>::type, typename VecOf<T, VEC>::type>::type vec_t;
    const int64_t nv = UNALIGNED ? (N + VEC - 1) / VEC : N / VEC, total = batch * nv;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        const int64_t b = v / nv;
        int64_t n = (v % nv) * VEC;
        if (UNALIGNED && n > N - VEC) n = N - VEC;
        const T *col = B + b * R * N + n;
        vec_t acc = vec_t(T(0));
        int64_t r = 0;
        for (; r + UNROLL <= R; r += UNROLL) {
            vec_t x[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                x[u] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(col + (r + u) * N));
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const T w = c[r + u];
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = fma_t(x[u][e], w, acc[e]);
            }
        }
        for (; r < R; ++r) {
            const vec_t x = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(col + r * N));
            const T w = c[r];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = fma_t(x[e], w, acc[e]);
        }
        *reinterpret_cast<vec_t *>(A + b * N + n) = acc;
    }
}

// The same sum with NV pieces per lane, 4 KiB apart: a workgroup then reads NV * 4 KiB contiguous
// bytes of every row, which suits rows that are far apart (mode 0: consecutive r are a whole
// J x K slice apart).  Needs N to be a multiple of NV * 256 pieces.
template <typename T, int NV, int UNROLL>
__global__ void __launch_bounds__(256)
ttv_left_wide_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                     int64_t batch, int64_t R, int64_t N) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    const int64_t span = (int64_t)NV * 256 * VEC;             // elements of n per workgroup
    const int64_t per_b = N / span, total = batch * per_b;
    for (int64_t g = blockIdx.x; g < total; g += gridDim.x) {
        const int64_t b = g / per_b, n = (g % per_b) * span + (int64_t)threadIdx.x * VEC;
        const T *col = B + b * R * N + n;
        vec_t acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = vec_t(T(0));
        int64_t r = 0;
        for (; r + UNROLL <= R; r += UNROLL) {
            vec_t x[UNROLL][NV];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int q = 0; q < NV; ++q)
                    x[u][q] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(col + (r + u) * N + q * 256 * VEC));
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const T w = c[r + u];
#pragma unroll
                for (int q = 0; q < NV; ++q)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[q][e] = fma_t(x[u][q][e], w, acc[q][e]);
            }
        }
        for (; r < R; ++r) {
            const T w = c[r];
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const vec_t x = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(col + r * N + q * 256 * VEC));
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[q][e] = fma_t(x[e], w, acc[q][e]);
            }
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) *reinterpret_cast<vec_t *>(A + b * N + n + q * 256 * VEC) = acc[q];
    }
}

// The same sum for outputs too few to give every compute unit a workgroup of the kernels above
// (a tall tensor contracted over its long leading mode): W lanes share a run of W pieces of the
// output row and the 256 / W lane groups of the workgroup split the rows r between them (group
// s takes r = s, s + S, s + 2 S, ...: what the groups read together is S consecutive rows),
// UNROLL loads per lane in flight.  The groups' sums meet in LDS and are added in the order of s.
// PV = elements per piece: the 16-byte vector, or 1 for rows shorter than one.  UNALIGNED as in
// ttv_left_vec_kernel: element-aligned accesses and an overlapping last piece (N >= PV).
template <typename T, int PV, int W, int UNROLL, bool UNALIGNED = false>
__global__ void __launch_bounds__(256)
ttv_left_split_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                      int64_t batch, int64_t R, int64_t N) {
    typedef typename VecOf<T, PV>::type lvec_t;
    typedef typename std::conditional<UNALIGNED, typename GlobalVecOf<T, PV>::type, lvec_t>::type vec_t;
    constexpr int S = 256 / W;
    __shared__ lvec_t part[S][W];
    const int64_t np = (N + PV - 1) / PV;                   // pieces per output row (N % PV == 0 unless UNALIGNED)
    const int64_t strips = (np + W - 1) / W, total = batch * strips;
    const int lw = threadIdx.x % W, s = threadIdx.x / W;
    for (int64_t g = blockIdx.x; g < total; g += gridDim.x) {
        const int64_t b = g / strips, piece = (g % strips) * W + lw;
        const bool valid = piece < np;
        int64_t n = (valid ? piece : np - 1) * PV;          // a lane past the end re-reads the last piece
        if (UNALIGNED && n > N - PV) n = N - PV;
        const T *col = B + b * R * N + n;
        vec_t acc = vec_t(T(0));
        int64_t r = s;
        for (; r + (int64_t)(UNROLL - 1) * S < R; r += (int64_t)UNROLL * S) {
            vec_t x[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                x[u] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(col + (r + (int64_t)u * S) * N));
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const T w = c[r + (int64_t)u * S];
                if constexpr (PV == 1) {
                    acc = fma_t(x[u], w, acc);
                } else {
#pragma unroll
                    for (int e = 0; e < PV; ++e) acc[e] = fma_t(x[u][e], w, acc[e]);
                }
            }
        }
        for (; r < R; r += S) {
            const vec_t x = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(col + r * N));
            const T w = c[r];
            if constexpr (PV == 1) {
                acc = fma_t(x, w, acc);
            } else {
#pragma unroll
                for (int e = 0; e < PV; ++e) acc[e] = fma_t(x[e], w, acc[e]);
            }
        }
        part[s][lw] = acc;
        __syncthreads();
        if (s == 0 && valid) {
            vec_t sum = part[0][lw];
#pragma unroll
            for (int q = 1; q < S; ++q) sum += part[q][lw];
            *reinterpret_cast<vec_t *>(A + b * N + n) = sum;
        }
        __syncthreads();                       // the sums have been read before the next strip overwrites them
    }
}

// Same sum, one element per lane: any alignment and any N.
template <typename T>
__global__ void __launch_bounds__(256)
ttv_left_generic_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                        int64_t batch, int64_t R, int64_t N) {
    const int64_t total = batch * N;
    for (int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x; m < total; m += (int64_t)gridDim.x * 256) {
        const int64_t b = m / N, n = m % N;
        const T *col = B + b * R * N + n;
        T acc = T(0);
        for (int64_t r = 0; r < R; ++r) acc = fma_t(col[r * N], c[r], acc);
        A[m] = acc;
    }
}

template <typename T>
__global__ void __launch_bounds__(256)
ttv_generic_kernel(const T *__restrict__ B, const T *__restrict__ c, T *__restrict__ A,
                   int64_t rows, int64_t K) {
    const int q = threadIdx.x & 15;
    const int64_t group = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int64_t stride = (int64_t)gridDim.x * 16;
    for (int64_t r = group; r < rows; r += stride) {
        const T *row = B + r * K;
        T acc = T(0);
        for (int64_t k = q; k < K; k += 16) acc = fma_t(row[k], c[k], acc);
        acc = sum16(acc);
        if (q == 0) A[r] = acc;
    }
}

// ---------------------------------------------------------------------------
// innerprod   a = sum_n B(n) * C(n)   over the n = I*J*K elements, two passes.
//
// Pass 1: block b owns the contiguous run of 16-byte pieces [b*per, (b+1)*per);
// each lane widens its operands to binary64 (a binary32 product is then exact)
// and keeps a binary64 running sum; the extra VALU work hides under the loads.  Lanes -> wavefront -> block are combined in a fixed order and the
// block's binary64 partial goes to the workspace.  Pass 2: one block adds the
// partials and the (< VEC) trailing elements in a fixed order and rounds once.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double piece_dot(const v4f b, const v4f c) {
    // binary32 x binary32 is exact in binary64
    double p = (double)b[0] * (double)c[0];
    p = __builtin_fma((double)b[1], (double)c[1], p);
    p = __builtin_fma((double)b[2], (double)c[2], p);
    p = __builtin_fma((double)b[3], (double)c[3], p);
    return p;
}
__device__ __forceinline__ double piece_dot(const v2d b, const v2d c) {
    return __builtin_fma(b[1], c[1], b[0] * c[0]);
}

// UNALIGNED: the operands may start at any element (views): the same 16-byte loads, typed as
// element-aligned, pieces counted from each operand's own start.
template <typename T, int UNROLL, bool UNALIGNED = false>
__global__ void __launch_bounds__(256)
innerprod_pass1_kernel(const T *__restrict__ B, const T *__restrict__ C, double *__restrict__ partial,
                       int64_t nvec, int64_t per_block) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef typename VecOf<T, VEC>::type vec_t;
    typedef typename std::conditional<UNALIGNED, typename GlobalVecOf<T, VEC>::type, vec_t>::type gvec_t;
    const gvec_t *bv = reinterpret_cast<const gvec_t *>(B);
    const gvec_t *cv = reinterpret_cast<const gvec_t *>(C);
    const int64_t lo = (int64_t)blockIdx.x * per_block;
    const int64_t hi = lo + per_block < nvec ? lo + per_block : nvec;
    double acc = 0.0;
    int64_t v = lo + threadIdx.x;
    for (; v + 256 * (UNROLL - 1) < hi; v += 256 * UNROLL) {
        vec_t b[UNROLL], c[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            b[u] = __builtin_nontemporal_load(bv + v + 256 * u);
            c[u] = __builtin_nontemporal_load(cv + v + 256 * u);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc += piece_dot(b[u], c[u]);
    }
    for (; v < hi; v += 256) acc += piece_dot(bv[v], cv[v]);

    __shared__ double wsum[4];
    acc = sum64(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
}

template <typename T>
__global__ void __launch_bounds__(256)
innerprod_pass2_kernel(const double *__restrict__ partial, int nparts,
                       const T *__restrict__ B, const T *__restrict__ C,
                       int64_t tail_lo, int64_t n, T *__restrict__ out) {
    double acc = 0.0;
    for (int p = threadIdx.x; p < nparts; p += 256) acc += partial[p];
    __shared__ double wsum[4];
    acc = sum64(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
        for (int64_t m = tail_lo; m < n; ++m) s += (double)B[m] * (double)C[m];
        *out = (T)s;
    }
}

// ---------------------------------------------------------------------------
// The last one to three columns of a matrix product, C(i, j) = [C(i, j) +] sum_k A(i,k) B(k,j)
// for j < ncols: the columns whose 16-byte piece would straddle the right edge of B and C when N
// is not a multiple of the vector.  The contraction kernels run the columns before them; these
// few are a matrix-vector product per column, i.e. one stream over the left operand.
// B and C point at the first of the ncols columns; blockIdx.y selects one problem of a batch
// (operands advance by fixed strides).
//
// gemm_fringe_cols_kernel (A is M x K): a workgroup owns 32 rows, 16 lanes share a row (two rows
// per lane group, four 16-byte loads of each in flight) and the columns of B are staged in LDS
// 2048 values of k at a time, so the only HBM stream is A itself.
// gemm_fringe_cols_ta_kernel (the left operand is stored K x M): a lane owns a row i and walks k;
// neighbouring lanes read neighbouring elements.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
gemm_fringe_cols_kernel(const T *__restrict__ A, int64_t lda, const T *__restrict__ B, int64_t ldb,
                        T *__restrict__ C, int64_t ldc, int64_t M, int64_t K, int ncols, int accumulate,
                        int64_t batch_a, int64_t batch_b, int64_t batch_c) {
    constexpr int VEC = 16 / (int)sizeof(T), NC = VEC - 1, KC = 2048, RG = 2, ROWS = 16 * RG, U = 4;
    A += (int64_t)blockIdx.y * batch_a;                    // blockIdx.y: one problem of a batch
    B += (int64_t)blockIdx.y * batch_b;
    C += (int64_t)blockIdx.y * batch_c;
    typedef typename VecOf<T, VEC>::type vec_t;
    typedef typename GlobalVecOf<T, VEC>::type gvec_t;
    __shared__ __attribute__((aligned(16))) T bs[NC][KC];
    const int q = threadIdx.x & 15, grp = threadIdx.x >> 4;
    for (int64_t row0 = (int64_t)blockIdx.x * ROWS; row0 < M; row0 += (int64_t)gridDim.x * ROWS) {
        T acc[RG][NC];
#pragma unroll
        for (int g = 0; g < RG; ++g)
#pragma unroll
            for (int c = 0; c < NC; ++c) acc[g][c] = T(0);
        // rows past M re-read row M-1 and are not stored
        const T *ar[RG];
#pragma unroll
        for (int g = 0; g < RG; ++g) {
            const int64_t r = row0 + grp * RG + g;
            ar[g] = A + (r < M ? r : M - 1) * lda;
        }
        for (int64_t k0 = 0; k0 < K; k0 += KC) {
            const int kc = (int)(K - k0 < KC ? K - k0 : KC);
            __syncthreads();                               // the previous chunk has been consumed
            for (int k = threadIdx.x; k < KC; k += 256)
#pragma unroll
                for (int c = 0; c < NC; ++c) bs[c][k] = (k < kc && c < ncols) ? B[(k0 + k) * ldb + c] : T(0);
            __syncthreads();
            const int kv = kc / VEC;                       // whole 16-byte pieces of this chunk
            int v = q;
            for (; v + 16 * (U - 1) < kv; v += 16 * U) {
                vec_t a[RG][U];
#pragma unroll
                for (int g = 0; g < RG; ++g)
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        a[g][u] = __builtin_nontemporal_load(reinterpret_cast<const gvec_t *>(ar[g] + k0 + (int64_t)(v + 16 * u) * VEC));
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const vec_t b = *reinterpret_cast<const vec_t *>(&bs[c][(v + 16 * u) * VEC]);
#pragma unroll
                        for (int g = 0; g < RG; ++g)
#pragma unroll
                            for (int e = 0; e < VEC; ++e) acc[g][c] = fma_t(a[g][u][e], b[e], acc[g][c]);
                    }
            }
            for (; v < kv; v += 16) {
#pragma unroll
                for (int g = 0; g < RG; ++g) {
                    const vec_t a = *reinterpret_cast<const gvec_t *>(ar[g] + k0 + (int64_t)v * VEC);
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[g][c] = fma_t(a[e], bs[c][v * VEC + e], acc[g][c]);
                }
            }
            for (int k = kv * VEC + q; k < kc; k += 16)   // fewer than VEC trailing elements of the last chunk
#pragma unroll
                for (int g = 0; g < RG; ++g)
#pragma unroll
                    for (int c = 0; c < NC; ++c) acc[g][c] = fma_t(ar[g][k0 + k], bs[c][k], acc[g][c]);
        }
#pragma unroll
        for (int g = 0; g < RG; ++g) {
            const int64_t r = row0 + grp * RG + g;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const T s = sum16(acc[g][c]);
                if (q == 0 && r < M && c < ncols) C[r * ldc + c] = accumulate ? C[r * ldc + c] + s : s;
            }
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(256)
gemm_fringe_cols_ta_kernel(const T *__restrict__ A, int64_t lda, const T *__restrict__ B, int64_t ldb,
                           T *__restrict__ C, int64_t ldc, int64_t M, int64_t K, int ncols, int accumulate,
                           int64_t batch_a, int64_t batch_b, int64_t batch_c) {
    A += (int64_t)blockIdx.y * batch_a;
    B += (int64_t)blockIdx.y * batch_b;
    C += (int64_t)blockIdx.y * batch_c;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < M; i += stride) {
        T acc[3] = {T(0), T(0), T(0)};
        for (int64_t k = 0; k < K; ++k) {
            const T a = A[k * lda + i];
#pragma unroll
            for (int c = 0; c < 3; ++c)
                if (c < ncols) acc[c] = fma_t(a, B[k * ldb + c], acc[c]);
        }
#pragma unroll
        for (int c = 0; c < 3; ++c)
            if (c < ncols) C[i * ldc + c] = accumulate ? C[i * ldc + c] + acc[c] : acc[c];
    }
}

// C(m, n) = [C(m, n) +] W(0, m, n) + W(1, m, n) + ... + W(parts - 1, m, n): the partial products of
// a matrix product cut along k, dense M x N slabs, added in the order of k (so the result is a
// function of the extents only) and only then onto the old C.
template <typename T>
__global__ void __launch_bounds__(256)
splitk_sum_kernel(const T *__restrict__ W, int parts, int64_t M, int64_t N, T *__restrict__ C, int64_t ldc,
                  int accumulate) {
    const int64_t n = M * N;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.x * 256) {
        T s = W[e];
        for (int p = 1; p < parts; ++p) s += W[(int64_t)p * n + e];
        T *c = C + (e / N) * ldc + (e % N);
        *c = accumulate ? *c + s : s;
    }
}

// Row-strided fill, used where an empty sum must still define its output.
template <typename T>
__global__ void __launch_bounds__(256)
fill_kernel(T *__restrict__ out, int64_t rows, int64_t cols, int64_t ld, T value) {
    const int64_t n = rows * cols;
    for (int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x; m < n; m += (int64_t)gridDim.x * 256)
        out[(m / cols) * ld + (m % cols)] = value;
}

}  // namespace distal
