/*
 * distal_probe.h - a measurement aid that ships beside the leaf-kernel library
 * (libdistal_probe.so).  It is NOT part of the leaf-kernel API of distal.h and
 * computes nothing of the paper's method: it exists so that the benchmark can
 * time, next to the MTTKRP kernel, a synthetic kernel with the same HBM load
 * stream and the same matrix-pipe work per byte but none of MTTKRP's
 * bookkeeping, i.e. the duration below which no rearrangement of that kernel can
 * fall on this part.  (The evaluation section of the paper casts MTTKRP to
 * matrix products plus an element-wise reduction; at rank 32 the product reads
 * 16 flop per byte, so the tensor stream and the matrix pipe are loaded
 * together.)
 */
#ifndef DISTAL_PROBE_H
#define DISTAL_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads the dense row-major binary32 tensor B (I x J x K, DEVICE pointer, 16-byte aligned)
 * once, with the access pattern of the MTTKRP kernel for modes 0 and 1 (a wavefront holds 32
 * rows of the first mode and one 256-byte slice of k and walks j), and issues 32
 * v_mfma_f32_32x32x2_f32 per 32 x 256-byte block, one operand scaled per step.
 *   I a multiple of 32, K a multiple of 256, each extent at most 2^20.
 *   F: DEVICE pointer to 1024 binary32 values (operand and scale factors; any finite values).
 *   lds != 0: each block passes through a wavefront-private LDS patch, as in the MTTKRP kernel;
 *   lds == 0: the MFMAs take the loaded registers directly.
 *   out: DEVICE scratch of at least distal_probe_out_bytes(I, J, K) bytes; receives the
 *   accumulators (meaningless values: they only keep the work alive).
 *   stream: hipStream_t as void*, NULL = default stream.  Asynchronous; nothing is allocated.
 * Returns 0, or 1 (NULL pointer), 2 (extents), 4 (B misaligned), 6 (out too small), 7 (launch).
 */
int distal_probe_stream_mfma(int64_t I, int64_t J, int64_t K, const void *B, const void *F, int lds,
                             void *out, size_t out_bytes, void *stream);

/* Bytes of `out` the call above needs (0 for extents it does not accept). */
size_t distal_probe_out_bytes(int64_t I, int64_t J, int64_t K);

/*
 * The rate of the matrix pipe on registers alone: 2048 workgroups of four wavefronts, each
 * wavefront issuing `iters` rounds of eight independent v_mfma_f64_16x16x4_f64 (f64 != 0) or
 * v_mfma_f32_32x32x2_f32 (f64 == 0) on operands that never change; no memory traffic but one
 * store per lane at the end.  distal_probe_mfma_peak_flops(f64, iters) / duration is what the
 * benchmark's peak denominators (78.6 and 157.3 TFLOP/s) are checked against on the device.
 *   out: DEVICE scratch of at least distal_probe_mfma_peak_out_bytes(f64) bytes.
 *   iters in [1, 2^24].  Asynchronous; nothing is allocated.
 * Returns 0, or 1 (NULL pointer), 2 (iters), 6 (out too small), 7 (launch).
 */
int distal_probe_mfma_peak(int f64, int64_t iters, void *out, size_t out_bytes, void *stream);
size_t distal_probe_mfma_peak_out_bytes(int f64);
double distal_probe_mfma_peak_flops(int f64, int64_t iters);

/*
 * What HBM delivers to a kernel that only reads: `bytes` bytes (a multiple of 16, DEVICE pointer,
 * 16-byte aligned) are read once with 16-byte non-temporal loads, `blocks` workgroups of 256
 * lanes each owning one contiguous range (rounded up to whole 4 KiB runs, so fewer workgroups
 * may be launched), `in_flight` (4, 8 or 16) loads per lane requested before the first is used.
 * bytes / duration is the ceiling the streaming rows of the benchmark (TTV, inner product) are
 * read against, next to the published 8 TB/s.
 *   out: DEVICE scratch of at least distal_probe_hbm_read_out_bytes(blocks) bytes (receives one
 *   partial sum per lane; meaningless values).  Asynchronous; nothing is allocated.
 * Returns 0, or 1 (NULL pointer), 2 (bytes, blocks or in_flight), 4 (src misaligned),
 * 6 (out too small), 7 (launch).
 */
int distal_probe_hbm_read(const void *src, int64_t bytes, int blocks, int in_flight, void *out, size_t out_bytes,
                          void *stream);
size_t distal_probe_hbm_read_out_bytes(int blocks);

#ifdef __cplusplus
}
#endif
#endif /* DISTAL_PROBE_H */
