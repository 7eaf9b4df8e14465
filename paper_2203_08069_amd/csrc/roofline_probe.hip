// Measurement aid, not part of the leaf-kernel API (declared in include/distal_probe.h).
//
// distal_probe_stream_mfma reads a dense binary32 I x J x K tensor exactly once with the
// access pattern of the MTTKRP walk kernel (a wavefront keeps 32 rows I-stride apart and one
// 256-byte slice of k, and walks j) and issues the same matrix-pipe work per byte - 32
// v_mfma_f32_32x32x2_f32 per 8 KiB block, one operand scaled by a per-step factor - but has no
// factor matrices, no partial rows and no second kernel: nothing of MTTKRP's bookkeeping.  It
// answers one question: what does that load stream cost on this part once the matrix pipe is
// loaded alongside it?  With lds != 0 a block goes through a wavefront-private LDS patch (as in
// the walk kernel); with lds == 0 the MFMAs take the loaded registers directly and each piece is
// re-requested right after the MFMAs that consumed it.  The accumulators are written out so that
// no work is dead; the values are meaningless.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/distal_probe.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int kPatchStride = 68;             // floats per patch row: 256 B + 16 B
constexpr int64_t kTargetBlocks = 768;       // as the library's MTTKRP plan: three workgroups per CU

struct ProbeArgs {
    const float *B;
    const float *F;      // 1024 factors, one per step (index wraps)
    float *out;          // 16 floats per thread
    int64_t J, K;        // walked extent; row length
    int64_t plane;       // J * K: elements between consecutive rows of a block
    int64_t wsplit;      // steps of j per workgroup
    int kgroups, rgroups;
};

__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool LDS>
__global__ void __launch_bounds__(256, 3) probe_stream_mfma_kernel(const ProbeArgs a) {
    __shared__ __attribute__((aligned(16))) float patch_all[LDS ? 4 * 32 * kPatchStride : 4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int bid = blockIdx.x;
    const int kgp = bid % a.kgroups;   bid /= a.kgroups;
    const int rgrp = bid % a.rgroups;  bid /= a.rgroups;
    const int split = bid;
    const int64_t w_lo = (int64_t)split * a.wsplit;
    const int64_t w_hi = w_lo + a.wsplit < a.J ? w_lo + a.wsplit : a.J;          // w_lo < w_hi by the plan
    // lane's piece u of a block: row 4u + lane/16 of the 32, 16-byte piece lane%16 of the 256-byte slice
    const float *base = a.B + ((int64_t)rgrp * 32 + lane / 16) * a.plane + (int64_t)(kgp * 4 + wave) * 64 + (lane % 16) * 4;
    const int64_t ustride = 4 * a.plane;

    float d[32];
#pragma unroll
    for (int m = 0; m < 32; ++m) d[m] = a.F[(lane * 32 + m) & 1023];
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    v4f x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(base + w_lo * a.K + u * ustride));
    float fn = a.F[w_lo & 1023];
    for (int64_t w = w_lo; w < w_hi; ++w) {
        const float f = fn;
        const int64_t wn = w + 1 < w_hi ? w + 1 : w;        // past the end: a redundant, in-bounds reload
        const float *next = base + wn * a.K;
        fn = a.F[wn & 1023];
        if constexpr (LDS) {
            float *patch = patch_all + wave * 32 * kPatchStride;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                *reinterpret_cast<v4f *>(patch + (lane / 16 + 4 * u) * kPatchStride + (lane % 16) * 4) = x[u];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(next + u * ustride));
            wave_fence();
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const v4f t = *reinterpret_cast<const v4f *>(patch + (lane % 32) * kPatchStride + g * 8 + (lane / 32) * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(d[g * 4 + e] * f, t[e], acc, 0, 0, 0);
            }
            wave_fence();
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(d[u * 4 + e] * f, x[u][e], acc, 0, 0, 0);
                x[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(next + u * ustride));
                __builtin_amdgcn_sched_barrier(0);     // keep each refill next to the MFMAs that freed it
            }
        }
    }
    float *o = a.out + ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16;
#pragma unroll
    for (int v = 0; v < 16; ++v) o[v] = acc[v];
}

// Nothing but matrix instructions on registers: eight independent accumulator chains per
// wavefront, four wavefronts per SIMD, operands that never change.  What this reaches is the rate
// of the matrix pipe at the clock the part holds under that load.  (Four wavefronts per SIMD are
// asked for so that the accumulators stay in one register file: with the default bound the compiler
// moved all of them between the two files in every round, and the loop measured those moves.)
constexpr int kPeakBlocks = 2048, kPeakChains = 8;

__global__ void __launch_bounds__(256, 4)
probe_mfma_peak_f64_kernel(double *out, int64_t iters, double x) {
    v4d acc[kPeakChains];
#pragma unroll
    for (int q = 0; q < kPeakChains; ++q) acc[q] = v4d{0.0, 0.0, 0.0, 0.0};
    const double a = x + (double)(threadIdx.x & 63) * 0.0078125, b = x - (double)(threadIdx.x & 15) * 0.015625;
    for (int64_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int q = 0; q < kPeakChains; ++q) acc[q] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[q], 0, 0, 0);
    }
    v4d s = acc[0];
#pragma unroll
    for (int q = 1; q < kPeakChains; ++q) s += acc[q];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = (s[0] + s[1]) + (s[2] + s[3]);
}

__global__ void __launch_bounds__(256, 4)
probe_mfma_peak_f32_kernel(float *out, int64_t iters, float x) {
    v16f acc[kPeakChains / 2];                       // 16 registers each: four chains keep the pipe full
#pragma unroll
    for (int q = 0; q < kPeakChains / 2; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.0f;
    const float a = x + (float)(threadIdx.x & 63) * 0.0078125f, b = x - (float)(threadIdx.x & 31) * 0.015625f;
    // An operand constraint on the accumulation register file makes the compiler keep the
    // accumulators there (the a[...] form of the instruction): with the accumulators in ordinary
    // vector registers this loop - same instruction, same operands - issued 12 % slower (137.7
    // against 155 TFLOP/s, same clock), which is a property of the loop's fixed registers, not of
    // the pipe; the contraction kernels measured no faster in that form and do not use it.
    asm volatile("" : : "a"(x));
    for (int64_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int q = 0; q < kPeakChains / 2; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < kPeakChains / 2; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[q][v];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

struct ProbePlan { int64_t kgroups, rgroups, wsplit, nsplit, blocks; };

bool probe_plan(int64_t I, int64_t J, int64_t K, ProbePlan *p) {
    if (I <= 0 || J <= 0 || K <= 0 || I % 32 != 0 || K % 256 != 0) return false;
    if (I > (1 << 20) || J > (1 << 20) || K > (1 << 20)) return false;          // keeps every product inside int64
    p->kgroups = K / 256;
    p->rgroups = I / 32;
    const int64_t tasks = p->kgroups * p->rgroups;
    int64_t want = (kTargetBlocks + tasks - 1) / tasks;
    if (want > J) want = J;
    p->wsplit = (J + want - 1) / want;
    p->nsplit = (J + p->wsplit - 1) / p->wsplit;
    p->blocks = tasks * p->nsplit;
    return p->blocks <= (1 << 24);
}

}  // namespace

// A read of `nvec` 16-byte pieces and nothing else: each workgroup owns one contiguous range and
// keeps U loads per lane in flight; the sums only keep the loads alive (one store per workgroup
// whose condition never holds for finite data would let the compiler drop nothing either way:
// the store below is unconditional).
typedef float v4f_probe __attribute__((ext_vector_type(4)));
template <int U>
__global__ void __launch_bounds__(256) probe_hbm_read_kernel(const v4f_probe *__restrict__ src, float *out, int64_t nvec, int64_t per) {
    const int64_t lo = (int64_t)blockIdx.x * per, hi = lo + per < nvec ? lo + per : nvec;
    float s = 0.f;
    for (int64_t v = lo + threadIdx.x; v < hi; v += 256 * U) {
        v4f_probe x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = (v + 256 * u < hi) ? __builtin_nontemporal_load(src + v + 256 * u) : v4f_probe(0.f);
#pragma unroll
        for (int u = 0; u < U; ++u) s += (x[u][0] + x[u][1]) + (x[u][2] + x[u][3]);
    }
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

extern "C" {

size_t distal_probe_hbm_read_out_bytes(int blocks) { return blocks > 0 ? (size_t)blocks * 256 * sizeof(float) : 0; }

int distal_probe_hbm_read(const void *src, int64_t bytes, int blocks, int in_flight, void *out, size_t out_bytes, void *stream) {
    if (!src || !out) return 1;
    if (bytes < 16 || bytes % 16 != 0 || blocks < 1 || blocks > 65536 || (in_flight != 4 && in_flight != 8 && in_flight != 16)) return 2;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) != 0) return 4;
    if (out_bytes < distal_probe_hbm_read_out_bytes(blocks)) return 6;
    const int64_t nvec = bytes / 16;
    int64_t per = (nvec + blocks - 1) / blocks;
    per = (per + 255) / 256 * 256;                     // whole 4 KiB runs per workgroup
    const unsigned nb = (unsigned)((nvec + per - 1) / per);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const v4f_probe *p = static_cast<const v4f_probe *>(src);
    float *o = static_cast<float *>(out);
    if (in_flight == 4) hipLaunchKernelGGL(probe_hbm_read_kernel<4>, dim3(nb), dim3(256), 0, s, p, o, nvec, per);
    else if (in_flight == 8) hipLaunchKernelGGL(probe_hbm_read_kernel<8>, dim3(nb), dim3(256), 0, s, p, o, nvec, per);
    else hipLaunchKernelGGL(probe_hbm_read_kernel<16>, dim3(nb), dim3(256), 0, s, p, o, nvec, per);
    return hipGetLastError() == hipSuccess ? 0 : 7;
}

size_t distal_probe_out_bytes(int64_t I, int64_t J, int64_t K) {
    ProbePlan p;
    if (!probe_plan(I, J, K, &p)) return 0;
    return (size_t)p.blocks * 256 * 16 * sizeof(float);
}

int distal_probe_stream_mfma(int64_t I, int64_t J, int64_t K, const void *B, const void *F, int lds,
                             void *out, size_t out_bytes, void *stream) {
    ProbePlan p;
    if (!probe_plan(I, J, K, &p)) return 2;
    if (!B || !F || !out) return 1;
    if ((reinterpret_cast<uintptr_t>(B) & 15u) != 0) return 4;
    if (out_bytes < distal_probe_out_bytes(I, J, K)) return 6;
    ProbeArgs a{};
    a.B = static_cast<const float *>(B);
    a.F = static_cast<const float *>(F);
    a.out = static_cast<float *>(out);
    a.J = J; a.K = K; a.plane = J * K; a.wsplit = p.wsplit;
    a.kgroups = (int)p.kgroups; a.rgroups = (int)p.rgroups;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lds) hipLaunchKernelGGL(probe_stream_mfma_kernel<true>, dim3((unsigned)p.blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(probe_stream_mfma_kernel<false>, dim3((unsigned)p.blocks), dim3(256), 0, s, a);
    return hipGetLastError() == hipSuccess ? 0 : 7;
}

size_t distal_probe_mfma_peak_out_bytes(int f64) { return (size_t)kPeakBlocks * 256 * (f64 ? sizeof(double) : sizeof(float)); }

double distal_probe_mfma_peak_flops(int f64, int64_t iters) {
    // wavefronts x iterations x instructions per iteration x flop per instruction (16x16x4 resp. 32x32x2, two per term)
    return (double)kPeakBlocks * 4.0 * (double)iters * (double)kPeakChains * (f64 ? 2048.0 : 4096.0);
}

int distal_probe_mfma_peak(int f64, int64_t iters, void *out, size_t out_bytes, void *stream) {
    if (iters < 1 || iters > ((int64_t)1 << 24)) return 2;
    if (!out) return 1;
    if (out_bytes < distal_probe_mfma_peak_out_bytes(f64)) return 6;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (f64) hipLaunchKernelGGL(probe_mfma_peak_f64_kernel, dim3(kPeakBlocks), dim3(256), 0, s, static_cast<double *>(out), iters, 0.5);
    else hipLaunchKernelGGL(probe_mfma_peak_f32_kernel, dim3(kPeakBlocks), dim3(256), 0, s, static_cast<float *>(out), iters, 0.5f);
    return hipGetLastError() == hipSuccess ? 0 : 7;
}

}  // extern "C"
