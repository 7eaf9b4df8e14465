#!/usr/bin/env python3
"""Benchmark of the MI355X leaf-kernel library on one GPU.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--rows all|gemm_f64,...] [--no-cpu-baseline]

Headline (``value``): the matrix-multiply tile step in binary64 at
M = N = K = 8192, operands uniform in [-1, 1) from seed 1 - one GPU's tile of a
weak-scaled distributed product.  A step is one launch of that leaf through the
C ABI with all operands already resident in HBM; K steps are timed between
device synchronisations.

The same run then measures every other row of the hot path at its own full-size
configuration (binary32 GEMM, TTM, MTTKRP, TTV, innerprod) the same way and
reports them under ``rows``, each with the roofline that bounds it.  Per-launch
durations come from HIP events recorded on the stream the kernels run on
(torch's current stream, which is the stream handed to the library).

The CPU oracle is timed beside the GPU on bounded samples of the same seeded
inputs (``cpu_baseline``); that leg is the only place the oracle is used here,
and it doubles as a parity spot-check of the timed outputs.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "GFLOP/s + % MFMA peak (GEMM/TTM/MTTKRP); HBM GB/s (TTV/innerprod)"

# MI355X published peaks
PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the
# same counters on a plain copy kernel of known size; see profiles/.  None = not measured.
MEASURED_TRAFFIC_BYTES = {
    "gemm_f64": 9.133e9, "gemm_f32": 3.535e9, "ttm": 5.518e9, "ttm_mode0": 5.504e9, "ttm_mode1": 5.505e9,
    "mttkrp": 4.331e9, "mttkrp_mode2": 4.328e9, "ttv": 4.299e9, "ttv_mode0": 4.299e9, "innerprod": 8.590e9,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


SETTLE_MS = 40.0   # the part's power management needs a few tens of ms of load to settle


def time_launches(fn, steps, warmup, torch):
    """W warm-up launches, then K timed launches between synchronisations, with per-launch
    HIP-event durations.  For launches much shorter than the settling time of the clocks
    the warm-up is extended (never shortened) until it has covered SETTLE_MS of GPU time."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    est = max(e0.elapsed_time(e1), 1e-3)
    for _ in range(max(warmup - 2, 0, int(SETTLE_MS / est) + 1 - 2)):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    per = [a.elapsed_time(b) for a, b in ev]
    return wall_ms, float(np.mean(per)), float(np.min(per)), float(np.median(per))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--rows", default="all",
                    help="comma list of gemm_f64,gemm_f32,ttm,mttkrp,ttv,innerprod, or all for these six "
                         "(gemm_f64 always runs); "
                         "extra rows, not part of 'all': summa (k-chunk leaf shapes), "
                         "ttv_f64,innerprod_f64,ttm_f64,mttkrp_f64, ttm_mode0,ttm_mode1 (TTM along the "
                         "other modes of the configs[3] tensor), mttkrp_mode1,mttkrp_mode2 (MTTKRP along the "
                         "other modes of the configs[4] tensor), mttkrp_rank64, ttv_mode0,ttv_mode1, "
                         "ttm_rank32 (all three modes at rank 32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB read + 1 GiB write elementwise kernel (torch.add), the known-size "
                         "reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; every figure is a single-MI355X figure. "
            f"--gpus {args.gpus} is not supported (no collectives, no sharding in this library).")
        sys.exit(2)
    if args.steps < 1 or args.warmup < 0:
        log("bench.py: need --steps >= 1 and --warmup >= 0")
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(1)
    from paper_2203_08069_amd import binding, inputs
    from paper_2203_08069_amd.device_inputs import device_tensor
    binding.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    want = set(args.rows.split(",")) | {"gemm_f64"}
    if "all" in want:
        want |= {"gemm_f32", "ttm", "mttkrp", "ttv", "innerprod"}
    cpu = not args.no_cpu_baseline
    if cpu:
        import oracle
        oracle.build()
        cores = oracle.max_threads()
    rows = []
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    def tdt(np_dt):
        return torch.float64 if np.dtype(np_dt) == np.float64 else torch.float32

    def finish(name, workload, dt, fn, flops, bytes_, bound, extra=None):
        wall, mean, mn, med = time_launches(fn, args.steps, args.warmup, torch)
        r = {"row": name, "workload": workload, "dtype": dt, "ms_per_step": wall, "ms_kernel_avg": mean,
             "ms_kernel_min": mn, "ms_kernel_median": med,
             "gflops": flops / mean / 1e6, "gbs": bytes_ / mean / 1e6}
        if bound == "mfma":
            ach = flops / mean / 1e9
            r["roofline"] = {"bound": "mfma", "achieved": ach, "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
                             "frac": ach / PEAK_TFLOPS[dt], "traffic": MEASURED_TRAFFIC_BYTES.get(name)}
        else:
            ach = bytes_ / mean / 1e6
            r["roofline"] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": ach / PEAK_HBM_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(name)}
        if extra:
            r.update(extra)
        rows.append(r)
        log(f"[bench] {name}: {mean:.3f} ms/launch, {r['gflops']:.0f} GFLOP/s, {r['gbs']:.0f} GB/s, "
            f"roofline {r['roofline']['frac'] * 100:.1f}% of {r['roofline']['bound']}")
        return r

    def sample_err(got, ref):
        got = np.asarray(got, dtype=np.float64)
        scale = float(np.max(np.abs(ref))) or 1.0
        return float(np.max(np.abs(got - ref))) / scale

    # ---------------------------------------------------------------- GEMM (configs[1])
    for name, npdt in (("gemm_f64", np.float64), ("gemm_f32", np.float32)):
        if name not in want:
            continue
        n = 8192
        dt = "f64" if npdt == np.float64 else "f32"
        log(f"[bench] {name}: generating operands")
        A = device_tensor(1, 0, (n, n), npdt, device=dev)
        B = device_tensor(1, 1, (n, n), npdt, device=dev)
        C = torch.zeros((n, n), dtype=tdt(npdt), device=dev)
        r = finish(name, f"C(i,j)=sum_k A(i,k)B(k,j), M=N=K={n}, {dt}, uniform[-1,1) seed 1", dt,
                   lambda: binding.distal_gemm(A, B, C), 2.0 * n ** 3, 3.0 * n * n * np.dtype(npdt).itemsize,
                   "mfma")
        if cpu:
            m_s = 96 if name == "gemm_f64" else 24
            rows_idx = np.linspace(0, n - 1, m_s).astype(np.int64)
            hA = np.stack([inputs.values(1, 0, int(i) * n, n, npdt) for i in rows_idx])
            hB = inputs.tensor(1, 1, (n, n), npdt, threads=cores)
            t0 = time.perf_counter()
            ref = oracle.gemm(hA, hB)
            sec = time.perf_counter() - t0
            got = C[torch.from_numpy(rows_idx).to(dev)].cpu().numpy()
            r["cpu_baseline"] = {"value": 2.0 * m_s * n * n / sec / 1e9, "unit": "GFLOP/s", "cores": cores,
                                 "kind": "oracle", "seconds": sec,
                                 "sample": f"{m_s} evenly spaced rows of C (all {n} columns, full K={n})"}
            r["sample_normwise_err"] = sample_err(got, ref)
            del hB
        del A, B, C

    # ---------------------------------------------------------------- SUMMA k-chunk leaf shapes (extra)
    if "summa" in want:
        n = 8192
        A = device_tensor(1, 0, (n, n), np.float64, device=dev)
        B = device_tensor(1, 1, (n, n), np.float64, device=dev)
        C = torch.zeros((n, n), dtype=torch.float64, device=dev)
        for chunk in (256, 512, 1024, 2048):
            finish(f"gemm_f64_summa_chunk{chunk}",
                   f"C += A(:, kc:kc+{chunk}) B(kc:kc+{chunk}, :), M=N={n}: the leaf one processor issues per SUMMA k-step",
                   "f64", lambda: binding.distal_gemm(A[:, 0:chunk], B[0:chunk, :], C, accumulate=True),
                   2.0 * n * n * chunk, 8.0 * (2 * n * chunk + 2 * n * n), "mfma")
        del A, B, C

    # ---------------------------------------------------------------- fp64 higher-order kernels (extra)
    if want & {"ttv_f64", "innerprod_f64", "ttm_f64", "mttkrp_f64"}:
        I = J = K = 1024
        B = device_tensor(2, 0, (I, J, K), np.float64, device=dev)
        if "ttv_f64" in want:
            c = device_tensor(2, 1, (K,), np.float64, device=dev)
            A = torch.empty((I, J), dtype=torch.float64, device=dev)
            finish("ttv_f64", f"TTV B {I}x{J}x{K} f64, seed 2", "f64", lambda: binding.distal_ttv(B, c, A),
                   2.0 * I * J * K, 8.0 * (I * J * K + K + I * J), "hbm")
            del A
        if "innerprod_f64" in want:
            C = device_tensor(2, 2, (I, J, K), np.float64, device=dev)
            a = torch.empty(1, dtype=torch.float64, device=dev)
            finish("innerprod_f64", f"innerprod B,C {I}x{J}x{K} f64, seed 2", "f64",
                   lambda: binding.distal_innerprod(B, C, a), 2.0 * I * J * K, 16.0 * I * J * K, "hbm")
            del C, a
        if "ttm_f64" in want:
            L = 256
            C = device_tensor(3, 1, (K, L), np.float64, device=dev)
            A = torch.empty((I, J, L), dtype=torch.float64, device=dev)
            finish("ttm_f64", f"TTM B {I}x{J}x{K}, C {K}x{L} f64", "f64", lambda: binding.distal_ttm(B, C, A),
                   2.0 * I * J * K * L, 8.0 * (I * J * K + K * L + I * J * L), "mfma")
            del C, A
        if "mttkrp_f64" in want:
            L = 32
            C = device_tensor(4, 1, (J, L), np.float64, device=dev)
            D = device_tensor(4, 2, (K, L), np.float64, device=dev)
            A = torch.empty((I, L), dtype=torch.float64, device=dev)
            r = finish("mttkrp_f64", f"MTTKRP B {I}x{J}x{K}, rank {L} f64", "f64",
                       lambda: binding.distal_mttkrp(B, C, D, A), 2.0 * I * J * K * L + 2.0 * I * J * L,
                       8.0 * (I * J * K + J * L + K * L + I * L), "hbm")
            r["mfma_frac"] = (2.0 * I * J * K * L + 2.0 * I * J * L) / r["ms_kernel_avg"] / 1e9 / PEAK_TFLOPS["f64"]
            del C, D, A
        del B

    # ---------------------------------------------------------------- TTV + innerprod (configs[2])
    if "ttv" in want or "innerprod" in want:
        I = J = K = 1024
        log("[bench] ttv/innerprod: generating operands")
        B = device_tensor(2, 0, (I, J, K), np.float32, device=dev)
        if "ttv" in want:
            c = device_tensor(2, 1, (K,), np.float32, device=dev)
            A = torch.empty((I, J), dtype=torch.float32, device=dev)
            r = finish("ttv", f"A(i,j)=sum_k B(i,j,k)c(k), B {I}x{J}x{K} f32, seed 2", "f32",
                       lambda: binding.distal_ttv(B, c, A), 2.0 * I * J * K, 4.0 * (I * J * K + K + I * J), "hbm")
            if cpu:
                i_s = 256
                hB = inputs.tensor(2, 0, (i_s, J, K), np.float32, threads=cores)
                hc = inputs.values(2, 1, 0, K, np.float32)
                t0 = time.perf_counter()
                ref = oracle.ttv(hB, hc)
                sec = time.perf_counter() - t0
                r["cpu_baseline"] = {"value": 4.0 * (i_s * J * K + K + i_s * J) / sec / 1e9, "unit": "GB/s",
                                     "cores": cores, "kind": "oracle", "seconds": sec,
                                     "sample": f"first {i_s} of {I} i-slices of B"}
                r["sample_normwise_err"] = sample_err(A[:i_s].cpu().numpy(), ref)
            del A
        if "innerprod" in want:
            C = device_tensor(2, 2, (I, J, K), np.float32, device=dev)
            a = torch.empty(1, dtype=torch.float32, device=dev)
            r = finish("innerprod", f"a=sum_ijk B(i,j,k)C(i,j,k), B,C {I}x{J}x{K} f32, seed 2", "f32",
                       lambda: binding.distal_innerprod(B, C, a), 2.0 * I * J * K, 8.0 * I * J * K, "hbm")
            if cpu:
                n_s = 1 << 28
                hB = inputs.tensor(2, 0, (1, 1, n_s), np.float32, threads=cores)
                hC = inputs.tensor(2, 2, (1, 1, n_s), np.float32, threads=cores)
                t0 = time.perf_counter()
                ref = oracle.innerprod(hB, hC)
                sec = time.perf_counter() - t0
                a2 = torch.empty(1, dtype=torch.float32, device=dev)
                binding.distal_innerprod(B.view(-1)[:n_s].view(1, 1, n_s), C.view(-1)[:n_s].view(1, 1, n_s), a2)
                r["cpu_baseline"] = {"value": 8.0 * n_s / sec / 1e9, "unit": "GB/s", "cores": cores,
                                     "kind": "oracle", "seconds": sec,
                                     "sample": f"first 2^28 of 2^30 elements of B and C"}
                r["sample_normwise_err"] = abs(float(a2.item()) - ref) / abs(ref)
                del hB, hC
            del C, a
        del B

    # ---------------------------------------------------------------- TTV along modes 0 and 1 (extra)
    if want & {"ttv_mode0", "ttv_mode1"}:
        I = J = K = 1024
        B = device_tensor(2, 0, (I, J, K), np.float32, device=dev)
        c = device_tensor(2, 1, (K,), np.float32, device=dev)             # I = J = K: the vector fits every mode
        A = torch.empty((I, J), dtype=torch.float32, device=dev)
        for mode in (0, 1):
            if f"ttv_mode{mode}" not in want:
                continue
            r = finish(f"ttv_mode{mode}", f"TTV along mode {mode}, B {I}x{J}x{K} f32, seed 2", "f32",
                       lambda: binding.distal_ttv_mode(mode, B, c, A), 2.0 * I * J * K, 4.0 * (I * J * K + K + I * J), "hbm")
            if cpu:
                # a block of outputs depends on the matching block of B only
                hB = np.ascontiguousarray((B[:, :4, :] if mode == 0 else B[:4]).cpu().numpy())
                t0 = time.perf_counter()
                ref = oracle.ttv_mode(mode, hB, c.cpu().numpy())
                sec = time.perf_counter() - t0
                r["cpu_baseline"] = {"value": hB.nbytes / sec / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
                                     "seconds": sec, "sample": "4 of 1024 slices of B along mode %d" % (1 - mode)}
                r["sample_normwise_err"] = sample_err(A[:4].cpu().numpy(), ref)
        del B, c, A

    # ---------------------------------------------------------------- TTM (configs[3])
    if "ttm" in want:
        I = J = K = 1024
        L = 256
        log("[bench] ttm: generating operands")
        B = device_tensor(3, 0, (I, J, K), np.float32, device=dev)
        C = device_tensor(3, 1, (K, L), np.float32, device=dev)
        A = torch.empty((I, J, L), dtype=torch.float32, device=dev)
        r = finish("ttm", f"A(i,j,l)=sum_k B(i,j,k)C(k,l), B {I}x{J}x{K}, C {K}x{L} f32, seed 3", "f32",
                   lambda: binding.distal_ttm(B, C, A), 2.0 * I * J * K * L,
                   4.0 * (I * J * K + K * L + I * J * L), "mfma")
        if cpu:
            i_s = 16
            hB = inputs.tensor(3, 0, (i_s, J, K), np.float32, threads=cores)
            hC = inputs.tensor(3, 1, (K, L), np.float32)
            t0 = time.perf_counter()
            ref = oracle.ttm(hB, hC)
            sec = time.perf_counter() - t0
            r["cpu_baseline"] = {"value": 2.0 * i_s * J * K * L / sec / 1e9, "unit": "GFLOP/s", "cores": cores,
                                 "kind": "oracle", "seconds": sec, "sample": f"first {i_s} of {I} i-slices"}
            r["sample_normwise_err"] = sample_err(A[:i_s].cpu().numpy(), ref)
        del B, C, A

    # ---------------------------------------------------------------- TTM along modes 0 and 1 (extra)
    if want & {"ttm_mode0", "ttm_mode1"}:
        I = J = K = 1024
        R = 256
        B = device_tensor(3, 0, (I, J, K), np.float32, device=dev)
        C = device_tensor(3, 1, (K, R), np.float32, device=dev)      # I = J = K: one factor serves every mode
        for mode in (0, 1):
            if f"ttm_mode{mode}" not in want:
                continue
            shape = [I, J, K]
            shape[mode] = R
            A = torch.empty(shape, dtype=torch.float32, device=dev)
            r = finish(f"ttm_mode{mode}", f"TTM along mode {mode}, B {I}x{J}x{K}, C {K}x{R} f32, seed 3", "f32",
                       lambda: binding.distal_ttm_mode(mode, B, C, A), 2.0 * I * J * K * R,
                       4.0 * (I * J * K + K * R + I * J * R), "mfma")
            if cpu:
                # outputs that depend on one slice of B only: mode 0 -> A(:, j, :), mode 1 -> A(i, :, :)
                n_s = 8
                hC = inputs.tensor(3, 1, (K, R), np.float32)
                if mode == 0:
                    hB = np.ascontiguousarray(B[:, :n_s, :].cpu().numpy())
                    got = A[:, :n_s, :].cpu().numpy()
                else:
                    hB = np.ascontiguousarray(B[:n_s].cpu().numpy())
                    got = A[:n_s].cpu().numpy()
                t0 = time.perf_counter()
                ref = oracle.ttm_mode(mode, hB, hC)
                sec = time.perf_counter() - t0
                r["cpu_baseline"] = {"value": 2.0 * n_s * J * K * R / sec / 1e9, "unit": "GFLOP/s", "cores": cores,
                                     "kind": "oracle", "seconds": sec,
                                     "sample": f"{n_s} of 1024 slices of the output along mode {1 - mode}"}
                r["sample_normwise_err"] = sample_err(got, ref)
            del A
        del B, C

    # ---------------------------------------------------------------- TTM at rank 32 (extra): HBM-bound
    if "ttm_rank32" in want:
        I = J = K = 1024
        R = 32
        B = device_tensor(3, 0, (I, J, K), np.float32, device=dev)
        C = device_tensor(3, 1, (K, R), np.float32, device=dev)
        for mode in (2, 0, 1):
            shape = [I, J, K]
            shape[mode] = R
            A = torch.empty(shape, dtype=torch.float32, device=dev)
            r = finish(f"ttm_rank32_mode{mode}",
                       f"TTM along mode {mode}, B {I}x{J}x{K}, C {K}x{R} f32, seed 3 (16 flop/B: HBM-bound)", "f32",
                       lambda: binding.distal_ttm_mode(mode, B, C, A), 2.0 * I * J * K * R,
                       4.0 * (I * J * K + K * R + I * J * R), "hbm")
            if cpu:
                n_s = 16
                hC = C.cpu().numpy()
                if mode == 0:
                    hB, got = np.ascontiguousarray(B[:, :n_s, :].cpu().numpy()), A[:, :n_s, :].cpu().numpy()
                else:
                    hB, got = np.ascontiguousarray(B[:n_s].cpu().numpy()), A[:n_s].cpu().numpy()
                t0 = time.perf_counter()
                ref = oracle.ttm_mode(mode, hB, hC)
                sec = time.perf_counter() - t0
                r["cpu_baseline"] = {"value": 2.0 * n_s * J * K * R / sec / 1e9, "unit": "GFLOP/s", "cores": cores,
                                     "kind": "oracle", "seconds": sec, "sample": f"{n_s} of 1024 slices of the output"}
                r["sample_normwise_err"] = sample_err(got, ref)
            del A
        del B, C

    # ---------------------------------------------------------------- MTTKRP (configs[4])
    if "mttkrp" in want:
        I = J = K = 1024
        L = 32
        log("[bench] mttkrp: generating operands")
        B = device_tensor(4, 0, (I, J, K), np.float32, device=dev)
        C = device_tensor(4, 1, (J, L), np.float32, device=dev)
        D = device_tensor(4, 2, (K, L), np.float32, device=dev)
        A = torch.empty((I, L), dtype=torch.float32, device=dev)
        flops = 2.0 * I * J * K * L + 2.0 * I * J * L       # factored form: matrix products, then the j-reduction
        bytes_ = 4.0 * (I * J * K + J * L + K * L + I * L)
        r = finish("mttkrp", f"A(i,l)=sum_jk B(i,j,k)C(j,l)D(k,l), B {I}x{J}x{K}, C,D {J}x{L} f32, seed 4",
                   "f32", lambda: binding.distal_mttkrp(B, C, D, A), flops, bytes_, "hbm")
        r["mfma_frac"] = flops / r["ms_kernel_avg"] / 1e9 / PEAK_TFLOPS["f32"]
        if cpu:
            i_s = 32
            hB = inputs.tensor(4, 0, (i_s, J, K), np.float32, threads=cores)
            hC, hD = inputs.tensor(4, 1, (J, L), np.float32), inputs.tensor(4, 2, (K, L), np.float32)
            t0 = time.perf_counter()
            ref = oracle.mttkrp(hB, hC, hD)
            sec = time.perf_counter() - t0
            r["cpu_baseline"] = {"value": (2.0 * i_s * J * K * L + 2.0 * i_s * J * L) / sec / 1e9,
                                 "unit": "GFLOP/s", "cores": cores, "kind": "oracle", "seconds": sec,
                                 "sample": f"first {i_s} of {I} i-slices"}
            r["sample_normwise_err"] = sample_err(A[:i_s].cpu().numpy(), ref)
        del B, C, D, A

    # ---------------------------------------------------------------- MTTKRP at rank 64 (extra): MFMA-bound
    if "mttkrp_rank64" in want:
        I = J = K = 1024
        L = 64
        B = device_tensor(4, 0, (I, J, K), np.float32, device=dev)
        C = device_tensor(4, 1, (J, L), np.float32, device=dev)
        D = device_tensor(4, 2, (K, L), np.float32, device=dev)
        A = torch.empty((I, L), dtype=torch.float32, device=dev)
        flops = 2.0 * I * J * K * L + 2.0 * I * J * L
        r = finish("mttkrp_rank64", f"MTTKRP B {I}x{J}x{K}, rank {L} f32 (arithmetic intensity 32 flop/B: MFMA-bound)",
                   "f32", lambda: binding.distal_mttkrp(B, C, D, A), flops,
                   4.0 * (I * J * K + J * L + K * L + I * L), "mfma")
        if cpu:
            i_s = 16
            hB = np.ascontiguousarray(B[:i_s].cpu().numpy())
            t0 = time.perf_counter()
            ref = oracle.mttkrp(hB, C.cpu().numpy(), D.cpu().numpy())
            sec = time.perf_counter() - t0
            r["cpu_baseline"] = {"value": 3.0 * i_s * J * K * L / sec / 1e9, "unit": "GFLOP/s", "cores": cores,
                                 "kind": "oracle", "seconds": sec, "sample": f"first {i_s} of {I} output rows"}
            r["sample_normwise_err"] = sample_err(A[:i_s].cpu().numpy(), ref)
        del B, C, D, A

    # ---------------------------------------------------------------- MTTKRP along modes 1 and 2 (extra)
    if want & {"mttkrp_mode0", "mttkrp_mode1", "mttkrp_mode2"}:
        I = J = K = 1024
        L = 32
        B = device_tensor(4, 0, (I, J, K), np.float32, device=dev)
        C = device_tensor(4, 1, (J, L), np.float32, device=dev)       # I = J = K: the factors fit every mode
        D = device_tensor(4, 2, (K, L), np.float32, device=dev)
        A = torch.empty((I, L), dtype=torch.float32, device=dev)
        flops = 2.0 * I * J * K * L + 2.0 * I * J * L
        bytes_ = 4.0 * (I * J * K + J * L + K * L + I * L)
        for mode in (0, 1, 2):
            if f"mttkrp_mode{mode}" not in want:
                continue
            r = finish(f"mttkrp_mode{mode}", f"MTTKRP along mode {mode}, B {I}x{J}x{K}, rank {L} f32, seed 4", "f32",
                       lambda: binding.distal_mttkrp_mode(mode, B, C, D, A), flops, bytes_, "hbm")
            r["mfma_frac"] = flops / r["ms_kernel_avg"] / 1e9 / PEAK_TFLOPS["f32"]
            if cpu:
                # output row x depends only on the slice of B with that mode fixed at x
                n_s = 8
                hB = np.ascontiguousarray((B[:n_s], B[:, :n_s, :], B[:, :, :n_s])[mode].cpu().numpy())
                hC, hD = C.cpu().numpy(), D.cpu().numpy()
                t0 = time.perf_counter()
                ref = oracle.mttkrp_mode(mode, hB, hC, hD)
                sec = time.perf_counter() - t0
                r["cpu_baseline"] = {"value": 2.0 * n_s * I * J * L * 1.5 / sec / 1e9, "unit": "GFLOP/s",
                                     "cores": cores, "kind": "oracle", "seconds": sec,
                                     "sample": f"first {n_s} of 1024 output rows (3 flop per term, as the oracle "
                                               "sums the literal triple product)"}
                r["sample_normwise_err"] = sample_err(A[:n_s].cpu().numpy(), ref)
        del B, C, D, A

    head = rows[0]
    out = {
        "metric": METRIC,
        "value": head["gflops"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": head["workload"], "step": "one distal_gemm launch, operands resident in HBM",
                   "baseline_config": "configs[1]"},
        "roofline": head["roofline"],
        "cpu_baseline": head.get("cpu_baseline"),
        "rows": rows,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
