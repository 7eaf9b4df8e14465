#!/usr/bin/env python3
"""Benchmark of the MI355X leaf-kernel library on one GPU.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--rows all|core|name,name,...] [--no-cpu-baseline]

Headline (``value``): the matrix-multiply tile step in binary64 at
M = N = K = 8192, operands uniform in [-1, 1) from seed 1 - one GPU's tile of a
weak-scaled distributed product.  A step is one launch of that leaf through the
C ABI with all operands already resident in HBM; K steps are timed between
device synchronisations.

The same run then measures every other row of the hot path at its own full-size
configuration the same way and reports them under ``rows``, each with the roofline
that bounds it and the CPU oracle timed on a bounded sample of the same inputs:

    core   gemm_f64 gemm_f32 ttm mttkrp ttv innerprod           (the five expressions)
    all    core + the k-step leaf shapes of the schedules (summa), one whole SUMMA
           schedule issued by the schedule driver (summa_schedule), mid-size and
           misaligned products (gemm_shapes), the binary64 forms of the higher-order
           calls (*_f64), every other mode (ttm_mode*, ttv_mode*, mttkrp_mode*),
           rank-sized factors (ttm_rank32, mttkrp_rank64), the synthetic
           stream + MFMA kernel timed next to MTTKRP (mttkrp_floor) and the
           register-only matrix-instruction loop and the read-only stream that check
           the peak denominators on the device (mfma_peak, hbm_peak)

Per-launch durations come from HIP events recorded on the stream the kernels run on
(torch's current stream, which is the stream handed to the library).  ``roofline.traffic``
is read from the rocprofv3 summary under profiles/ that covers the row's kernel
(``traffic_source`` names the file; null where no summary exists): it was measured in the
profiling runs those files describe, not in this run.

The CPU oracle is used only in the ``cpu_baseline`` leg, outside the timed region; that
leg doubles as a parity spot-check of the timed outputs (``sample_normwise_err``).

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import re
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

CORE = ["gemm_f64", "gemm_f32", "ttm", "mttkrp", "ttv", "innerprod"]
EXTRA = ["summa", "summa_schedule", "gemm_shapes", "ttv_f64", "innerprod_f64", "ttm_f64", "mttkrp_f64", "ttv_mode0", "ttv_mode1",
         "ttm_mode0", "ttm_mode1", "ttm_rank32", "mttkrp_floor", "mttkrp_rank64", "mttkrp_mode1", "mttkrp_mode2", "mfma_peak", "hbm_peak"]

# rocprofv3 summary that covers a row's dominant kernel (HBM traffic per launch is read from it)
PROFILE_OF_ROW = {
    "gemm_f64": "contract_fast_kernel_f64_gemm_8192.md",
    "gemm_f32": "contract_fast_kernel_f32_gemm_8192.md",
    "gemm_f64_summa_chunk128": "contract_fast_kernel_f64_summa_kstep_8192x8192x128.md",
    "gemm_f64_summa_chunk256": "contract_fast_kernel_f64_summa_kstep_8192x8192x256.md",
    "gemm_f64_summa_chunk512": "contract_fast_kernel_f64_summa_kstep_8192x8192x512.md",
    "ttm": "contract_fast_kernel_f32_ttm_1024x1024x1024x256.md",
    "ttm_mode0": "contract_fast_kernel_tn_f32_ttm_mode0_1024x1024x1024x256.md",
    "ttm_mode1": "contract_fast_kernel_tn_f32_ttm_mode1_1024x1024x1024x256.md",
    "ttm_rank32_mode2": "ttm_slices_kernel_f32_1024_rank32.md",
    "mttkrp": "mttkrp_walk_kernel_f32_1024_rank32.md",
    "mttkrp_mode1": "mttkrp_walk_kernel_f32_1024_rank32.md",
    "mttkrp_mode2": "mttkrp_mode2_kernel_f32_1024_rank32.md",
    "ttv": "ttv_row_kernel_f32_1024.md",
    "ttv_mode0": "ttv_left_wide_kernel_f32_mode0_1024.md",
    "innerprod": "innerprod_pass1_kernel_f32_1024.md",
    "ttv_f64": "ttv_row_kernel_f64_1024.md",
    "innerprod_f64": "innerprod_pass1_kernel_f64_1024.md",
    "ttm_f64": "contract_fast_kernel_f64_ttm_1024x1024x1024x256.md",
    "mttkrp_f64": "mttkrp_walk_kernel_f64_1024_rank32.md",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(row):
    """(bytes per launch, source file) from the committed rocprofv3 summary of the row's kernel."""
    name = PROFILE_OF_ROW.get(row)
    if not name:
        return None, None
    path = os.path.join(ROOT, "profiles", name)
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m = re.search(r"HBM-side traffic per launch \(scaled\)\s*\|[^|]*total\s+([0-9.eE+-]+)\s*B", text)
    return (float(m.group(1)), "profiles/" + name) if m else (None, None)


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
                    help="'all' (default), 'core' (" + ",".join(CORE) + "), or a comma list of these and of "
                         + ",".join(EXTRA) + "; gemm_f64, the headline, always runs")
    ap.add_argument("--summa-chunks", default="128,256,512,1024,2048",
                    help="k-step depths of the summa rows (a profiler run takes one depth at a time)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--host-inputs", action="store_true",
                    help="generate the operands with numpy on the host and copy them (slow); the default fills "
                         "them in place with the same generator evaluated by torch integer operations")
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
    from paper_2203_08069_amd import binding, inputs, device_inputs
    binding.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    want = set(args.rows.split(",")) | {"gemm_f64"}
    if "all" in want:
        want |= set(CORE) | set(EXTRA)
    if "core" in want:
        want |= set(CORE)
    unknown = want - set(CORE) - set(EXTRA) - {"all", "core"}
    if unknown:
        log(f"bench.py: unknown rows {sorted(unknown)}")
        sys.exit(2)
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

    def dname(np_dt):
        return "f64" if np.dtype(np_dt) == np.float64 else "f32"

    def operand(seed, ordinal, shape, npdt):
        if args.host_inputs:
            return device_inputs.device_tensor(seed, ordinal, shape, npdt, device=dev)
        return device_inputs.generate_on_device(seed, ordinal, shape, npdt, device=dev)

    def finish(name, workload, dt, fn, flops, bytes_, bound):
        wall, mean, mn, med = time_launches(fn, args.steps, args.warmup, torch)
        traffic, source = measured_traffic(name)
        r = {"row": name, "workload": workload, "dtype": dt, "ms_per_step": wall, "ms_kernel_avg": mean,
             "ms_kernel_min": mn, "ms_kernel_median": med,
             "gflops": flops / mean / 1e6, "gbs": bytes_ / mean / 1e6}
        if bound == "mfma":
            ach = flops / mean / 1e9
            r["roofline"] = {"bound": "mfma", "achieved": ach, "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
                             "frac": ach / PEAK_TFLOPS[dt], "traffic": traffic, "traffic_source": source}
        else:
            ach = bytes_ / mean / 1e6
            r["roofline"] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": ach / PEAK_HBM_GBS, "traffic": traffic, "traffic_source": source}
        rows.append(r)
        log(f"[bench] {name}: {mean:.3f} ms/launch, {r['gflops']:.0f} GFLOP/s, {r['gbs']:.0f} GB/s, "
            f"roofline {r['roofline']['frac'] * 100:.1f}% of {r['roofline']['bound']}")
        return r

    def sample_err(got, ref):
        got = np.asarray(got, dtype=np.float64)
        scale = float(np.max(np.abs(ref))) or 1.0
        return float(np.max(np.abs(got - ref))) / scale

    def baseline(r, oracle_fn, got_fn, work, unit, sample):
        """Time the oracle on a bounded sample (host arrays are prepared by the caller, outside
        the clock) and compare the timed GPU output on the same sample."""
        if not cpu:
            return
        t0 = time.perf_counter()
        ref = oracle_fn()
        sec = time.perf_counter() - t0
        r["cpu_baseline"] = {"value": work / sec / 1e9, "unit": unit, "cores": cores, "kind": "oracle",
                             "seconds": sec, "sample": sample}
        got = got_fn()
        if np.ndim(ref) == 0:
            r["sample_normwise_err"] = abs(float(got) - float(ref)) / (abs(float(ref)) or 1.0)
        else:
            r["sample_normwise_err"] = sample_err(got, ref)

    def h(t):
        return np.ascontiguousarray(t.cpu().numpy())

    # ---------------------------------------------------------------- GEMM (configs[1]) and its relatives
    gemm_rows = [n for n in ("gemm_f64", "gemm_f32") if n in want]
    for name in gemm_rows:
        npdt = np.float64 if name == "gemm_f64" else np.float32
        n = 8192
        dt = dname(npdt)
        log(f"[bench] {name}: generating operands")
        A = operand(1, 0, (n, n), npdt)
        B = operand(1, 1, (n, n), npdt)
        C = torch.zeros((n, n), dtype=tdt(npdt), device=dev)
        r = finish(name, f"C(i,j)=sum_k A(i,k)B(k,j), M=N=K={n}, {dt}, uniform[-1,1) seed 1", dt,
                   lambda: binding.distal_gemm(A, B, C), 2.0 * n ** 3, 3.0 * n * n * np.dtype(npdt).itemsize,
                   "mfma")
        if cpu:
            m_s = 96 if name == "gemm_f64" else 24
            idx = torch.from_numpy(np.linspace(0, n - 1, m_s).astype(np.int64)).to(dev)
            hA, hB = h(A[idx]), h(B)
            baseline(r, lambda: oracle.gemm(hA, hB), lambda: h(C[idx]), 2.0 * m_s * n * n, "GFLOP/s",
                     f"{m_s} evenly spaced rows of C (all {n} columns, full K={n})")
            del hA, hB

        if "summa" in want:
            # the leaf one processor issues per k-step of SUMMA / Cannon: C += A(:, chunk) B(chunk, :)
            for chunk in [int(c) for c in args.summa_chunks.split(",") if c]:
                C.zero_()
                r = finish(f"{name}_summa_chunk{chunk}",
                           f"C += A(:, 0:{chunk}) B(0:{chunk}, :), M=N={n}, {dt}: one k-step of a SUMMA schedule", dt,
                           lambda: binding.distal_gemm(A[:, 0:chunk], B[0:chunk, :], C, accumulate=True),
                           2.0 * n * n * chunk, np.dtype(npdt).itemsize * (2.0 * n * chunk + 2 * n * n), "mfma")
                if cpu:
                    # after W + K accumulating launches C holds (launches) x the chunk product: check one launch's worth
                    C.zero_()
                    binding.distal_gemm(A[:, 0:chunk], B[0:chunk, :], C, accumulate=True)
                    idx = torch.from_numpy(np.linspace(0, n - 1, 16).astype(np.int64)).to(dev)
                    hA, hB = h(A[idx][:, 0:chunk]), h(B[0:chunk, :])
                    baseline(r, lambda: oracle.gemm(hA, hB), lambda: h(C[idx]), 2.0 * 16 * n * chunk, "GFLOP/s",
                             f"16 evenly spaced rows of one k-step's product")
        if "summa_schedule" in want:
            # the whole schedule of one processor's share: K / 512 accumulating k-steps through the
            # schedule driver (one "launch" of this row is the sequence of all of them)
            from paper_2203_08069_amd import schedules
            chunk = 512
            C.zero_()
            r = finish(f"{name}_summa_schedule_chunk{chunk}",
                       f"SUMMA on a 1 x 1 grid, M=N=K={n}, {dt}: {n // chunk} accumulating k-steps of {chunk} "
                       f"issued by the schedule driver, timed as one unit", dt,
                       lambda: schedules.summa(A, B, C, 1, 1, chunk), 2.0 * n ** 3,
                       np.dtype(npdt).itemsize * (2.0 * n * n + (n // chunk) * 2.0 * n * n), "mfma")
            r["launches_per_step"] = n // chunk
            if cpu:
                C.zero_()
                schedules.summa(A, B, C, 1, 1, chunk)
                idx = torch.from_numpy(np.linspace(0, n - 1, 8).astype(np.int64)).to(dev)
                hA, hB = h(A[idx]), h(B)
                baseline(r, lambda: oracle.gemm(hA, hB), lambda: h(C[idx]), 2.0 * 8 * n * n, "GFLOP/s",
                         f"8 evenly spaced rows of C after one run of the schedule from C = 0")
                del hA, hB
        if "gemm_shapes" in want:
            # shapes off the benchmark's grid: two or three rounds of tiles, an odd extent, a misaligned view
            cases = [("3000", 3000, 3000, 3000, 0), ("2000", 2000, 2000, 2000, 0), ("n8191", 8192, 8191, 8192, 0),
                     ("view_off1", 8192, 8188, 8192, 1)]
            for tag, M, N, K, off in cases:
                Av, Bv = A[:M, :K], B[:K, off:off + N]
                Cv = C[:M, off:off + N]
                r = finish(f"{name}_{tag}",
                           f"C = A B on views of the 8192^2 operands: M={M}, N={N}, K={K}, column offset {off}, {dt}", dt,
                           lambda: binding.distal_gemm(Av, Bv, Cv), 2.0 * M * N * K,
                           np.dtype(npdt).itemsize * (M * K + K * N + M * N), "mfma")
                if cpu:
                    idx = torch.from_numpy(np.linspace(0, M - 1, 8).astype(np.int64)).to(dev)
                    hA, hB = h(Av[idx]), h(Bv)
                    baseline(r, lambda: oracle.gemm(hA, hB), lambda: h(Cv[idx]), 2.0 * 8 * N * K, "GFLOP/s",
                             "8 evenly spaced rows of C")
            # a small output with a long contracted index (the operands viewed as 512 x 131072 and
            # 131072 x 512): 64 tiles for 256 compute units unless the product is cut along k
            Mt, Kt = 512, n * n // 512
            At, Bt, Ct = A.view(Mt, Kt), B.view(Kt, Mt), C[:Mt, :Mt]
            for tag, fn in (("tallk", lambda: binding.distal_gemm(At, Bt, Ct)), ("tallk_ws", lambda: binding.distal_gemm_ws(At, Bt, Ct))):
                r = finish(f"{name}_{tag}",
                           f"C = A B, M=N={Mt}, K={Kt}, {dt}" + (", cut along k with scratch memory (distal_gemm_ws)" if tag.endswith("ws") else ""),
                           dt, fn, 2.0 * Mt * Mt * Kt, np.dtype(npdt).itemsize * (2.0 * Mt * Kt + Mt * Mt), "mfma")
                if cpu:
                    idx = torch.from_numpy(np.linspace(0, Mt - 1, 4).astype(np.int64)).to(dev)
                    hA, hB = h(At[idx]), h(Bt)
                    baseline(r, lambda: oracle.gemm(hA, hB), lambda: h(Ct[idx]), 2.0 * 4 * Mt * Kt, "GFLOP/s",
                             "4 evenly spaced rows of C")
                    del hA, hB
        del A, B, C

    # ---------------------------------------------------------------- TTV + innerprod (configs[2]), all modes, both dtypes
    for npdt in (np.float32, np.float64):
        sfx = "" if npdt == np.float32 else "_f64"
        dt, esz = dname(npdt), np.dtype(npdt).itemsize
        names = {"ttv" + sfx, "innerprod" + sfx} | ({"ttv_mode0", "ttv_mode1"} if npdt == np.float32 else set())
        if not (want & names):
            continue
        I = J = K = 1024
        log(f"[bench] ttv/innerprod {dt}: generating operands")
        B = operand(2, 0, (I, J, K), npdt)
        c = operand(2, 1, (K,), npdt)
        if "ttv" + sfx in want:
            A = torch.empty((I, J), dtype=tdt(npdt), device=dev)
            r = finish("ttv" + sfx, f"A(i,j)=sum_k B(i,j,k)c(k), B {I}x{J}x{K} {dt}, seed 2", dt,
                       lambda: binding.distal_ttv(B, c, A), 2.0 * I * J * K, esz * (I * J * K + K + I * J), "hbm")
            if cpu:
                i_s = 256 if npdt == np.float32 else 128
                hB, hc = h(B[:i_s]), h(c)
                baseline(r, lambda: oracle.ttv(hB, hc), lambda: h(A[:i_s]), esz * (i_s * J * K + K + i_s * J),
                         "GB/s", f"first {i_s} of {I} i-slices of B")
                del hB
            del A
        for mode in (0, 1):
            if npdt != np.float32 or f"ttv_mode{mode}" not in want:
                continue
            A = torch.empty((I, J), dtype=tdt(npdt), device=dev)      # I = J = K: the vector fits every mode
            r = finish(f"ttv_mode{mode}", f"TTV along mode {mode}, B {I}x{J}x{K} {dt}, seed 2", dt,
                       lambda: binding.distal_ttv_mode(mode, B, c, A), 2.0 * I * J * K,
                       esz * (I * J * K + K + I * J), "hbm")
            if cpu:
                # a block of outputs depends on the matching block of B only
                hB, hc = h(B[:, :4, :] if mode == 0 else B[:4]), h(c)
                baseline(r, lambda: oracle.ttv_mode(mode, hB, hc), lambda: h(A[:4]), float(hB.nbytes), "GB/s",
                         "4 of 1024 slices of B along mode %d" % (1 - mode))
            del A
        if "innerprod" + sfx in want:
            C = operand(2, 2, (I, J, K), npdt)
            a = torch.empty(1, dtype=tdt(npdt), device=dev)
            r = finish("innerprod" + sfx, f"a=sum_ijk B(i,j,k)C(i,j,k), B,C {I}x{J}x{K} {dt}, seed 2", dt,
                       lambda: binding.distal_innerprod(B, C, a), 2.0 * I * J * K, 2.0 * esz * I * J * K, "hbm")
            if cpu:
                n_s = (1 << 28) if npdt == np.float32 else (1 << 27)
                fB, fC = B.view(-1)[:n_s].view(1, 1, n_s), C.view(-1)[:n_s].view(1, 1, n_s)
                hB, hC = h(fB), h(fC)
                a2 = torch.empty(1, dtype=tdt(npdt), device=dev)
                binding.distal_innerprod(fB, fC, a2)
                baseline(r, lambda: oracle.innerprod(hB, hC), lambda: float(a2.item()), 2.0 * esz * n_s, "GB/s",
                         f"first 2^{n_s.bit_length() - 1} of 2^30 elements of B and C")
                del hB, hC
            del C, a
        del B, c

    # ---------------------------------------------------------------- TTM (configs[3]), all modes, rank 32, both dtypes
    for npdt in (np.float32, np.float64):
        sfx = "" if npdt == np.float32 else "_f64"
        dt, esz = dname(npdt), np.dtype(npdt).itemsize
        names = {"ttm" + sfx, "ttm_rank32"} | ({"ttm_mode0", "ttm_mode1"} if npdt == np.float32 else set())
        if not (want & names):
            continue
        I = J = K = 1024
        L = 256
        log(f"[bench] ttm {dt}: generating operands")
        B = operand(3, 0, (I, J, K), npdt)
        C = operand(3, 1, (K, L), npdt)                   # I = J = K: one factor serves every mode
        hC = h(C)
        if "ttm" + sfx in want:
            A = torch.empty((I, J, L), dtype=tdt(npdt), device=dev)
            r = finish("ttm" + sfx, f"A(i,j,l)=sum_k B(i,j,k)C(k,l), B {I}x{J}x{K}, C {K}x{L} {dt}, seed 3", dt,
                       lambda: binding.distal_ttm(B, C, A), 2.0 * I * J * K * L,
                       esz * (I * J * K + K * L + I * J * L), "mfma")
            if cpu:
                i_s = 16 if npdt == np.float32 else 8
                hB = h(B[:i_s])
                baseline(r, lambda: oracle.ttm(hB, hC), lambda: h(A[:i_s]), 2.0 * i_s * J * K * L, "GFLOP/s",
                         f"first {i_s} of {I} i-slices")
            del A
        for rank, tag, bound in ((L, "ttm_mode%d", "mfma"), (32, "ttm_rank32_mode%d", "hbm")):
            for mode in ((0, 1) if rank == L else (2, 0, 1)):
                row = tag % mode + ("" if npdt == np.float32 else "_f64")
                # binary64: the rank-32 product along the last mode only (the kernel that holds the factor in registers)
                if (npdt != np.float32 and (rank == L or mode != 2)) or (tag % mode if rank == L else "ttm_rank32") not in want:
                    continue
                Cr = C if rank == L else C[:, :rank].contiguous()
                shape = [I, J, K]
                shape[mode] = rank
                A = torch.empty(shape, dtype=tdt(npdt), device=dev)
                r = finish(row, f"TTM along mode {mode}, B {I}x{J}x{K}, C {K}x{rank} {dt}, seed 3"
                           + (" (16 flop/B: HBM-bound)" if rank == 32 else ""), dt,
                           lambda: binding.distal_ttm_mode(mode, B, Cr, A), 2.0 * I * J * K * rank,
                           esz * (I * J * K + K * rank + I * J * rank), bound)
                if cpu:
                    # outputs that depend on one slice of B only: mode 0 -> A(:, j, :), modes 1, 2 -> A(i, :, :)
                    n_s = 8
                    hB = h(B[:, :n_s, :]) if mode == 0 else h(B[:n_s])
                    hCr = h(Cr)
                    baseline(r, lambda: oracle.ttm_mode(mode, hB, hCr),
                             lambda: h(A[:, :n_s, :]) if mode == 0 else h(A[:n_s]), 2.0 * n_s * J * K * rank,
                             "GFLOP/s", f"{n_s} of 1024 slices of the output")
                del A
        del B, C

    # ---------------------------------------------------------------- MTTKRP (configs[4]), all modes, rank 64, both dtypes
    for npdt in (np.float32, np.float64):
        sfx = "" if npdt == np.float32 else "_f64"
        dt, esz = dname(npdt), np.dtype(npdt).itemsize
        names = {"mttkrp" + sfx} | ({"mttkrp_floor", "mttkrp_rank64", "mttkrp_mode1", "mttkrp_mode2"}
                                    if npdt == np.float32 else set())
        if not (want & names):
            continue
        I = J = K = 1024
        log(f"[bench] mttkrp {dt}: generating operands")
        B = operand(4, 0, (I, J, K), npdt)
        C64 = operand(4, 1, (J, 64), npdt)                 # I = J = K: the factors fit every mode
        D64 = operand(4, 2, (K, 64), npdt)
        cases = [("mttkrp" + sfx, 0, 32)]
        if npdt == np.float32:
            cases += [("mttkrp_mode1", 1, 32), ("mttkrp_mode2", 2, 32), ("mttkrp_rank64", 0, 64)]
        for row, mode, L in cases:
            if row not in want:
                continue
            # the rank-32 factors are the seeded J x 32 tensors of configs[4]; rank 64 uses a J x 64 one
            C = operand(4, 1, (J, L), npdt) if L == 32 else C64
            D = operand(4, 2, (K, L), npdt) if L == 32 else D64
            A = torch.empty((I, L), dtype=tdt(npdt), device=dev)
            flops = 2.0 * I * J * K * L + 2.0 * I * J * L       # factored form: matrix products, then the reduction
            bytes_ = esz * (I * J * K + J * L + K * L + I * L)
            bound = "mfma" if L == 64 else "hbm"
            r = finish(row, f"MTTKRP along mode {mode}, B {I}x{J}x{K}, rank {L} {dt}, seed 4", dt,
                       lambda: binding.distal_mttkrp_mode(mode, B, C, D, A), flops, bytes_, bound)
            r["mfma_frac"] = flops / r["ms_kernel_avg"] / 1e9 / PEAK_TFLOPS[dt]
            r["hbm_frac"] = bytes_ / r["ms_kernel_avg"] / 1e6 / PEAK_HBM_GBS
            if cpu:
                # output row x depends only on the slice of B with that mode fixed at x
                n_s = 16 if npdt == np.float32 else 8
                hB = h((B[:n_s], B[:, :n_s, :], B[:, :, :n_s])[mode])
                hC, hD = h(C), h(D)
                baseline(r, lambda: oracle.mttkrp_mode(mode, hB, hC, hD), lambda: h(A[:n_s]),
                         3.0 * n_s * J * K * L, "GFLOP/s",
                         f"first {n_s} of 1024 output rows (3 flop per term: the oracle sums the literal triple product)")
            del A
        if npdt == np.float32 and "mttkrp_floor" in want:
            # Not a row of the method: a synthetic kernel with the MTTKRP kernel's load stream and MFMA count
            # and none of its bookkeeping, on the same tensor and on zeros (the duration follows the data:
            # the part is power-limited when HBM and the matrix pipe are loaded together).
            from paper_2203_08069_amd import probe
            F = operand(4, 1, (1024,), np.float32)
            out = torch.empty(probe.out_bytes(I, J, K) // 4, dtype=torch.float32, device=dev)
            flops, bytes_ = 2.0 * I * J * K * 32, 4.0 * I * J * K
            for tag, T, lds in (("lds", B, True), ("nolds", B, False), ("lds_zeros", None, True)):
                if T is None:
                    T = torch.zeros((I, J, K), dtype=torch.float32, device=dev)
                r = finish(f"mttkrp_floor_{tag}",
                           "synthetic: one pass over a 1024^3 f32 tensor with the MTTKRP kernel's access pattern, "
                           "32 MFMA 32x32x2 per 8 KiB block, " + ("through an LDS patch" if lds else "operands from the load registers")
                           + ("; tensor of zeros" if tag.endswith("zeros") else "; the seed-4 tensor"),
                           "f32", lambda: probe.stream_mfma(T, F, out, lds), flops, bytes_, "hbm")
                r["mfma_frac"] = flops / r["ms_kernel_avg"] / 1e9 / PEAK_TFLOPS["f32"]
                r["synthetic"] = True
                del T
            del F, out
        del B, C64, D64

    if "mfma_peak" in want:
        # Not a row of the method: matrix instructions on registers alone, the on-device check of the
        # peak denominators (clock under that load x pipe width)
        from paper_2203_08069_amd import probe
        for f64 in (True, False):
            dt = "f64" if f64 else "f32"
            out = torch.empty(probe.mfma_peak_out_bytes(f64) // (8 if f64 else 4),
                              dtype=torch.float64 if f64 else torch.float32, device=dev)
            iters = 3000
            r = finish(f"mfma_peak_{dt}",
                       f"synthetic: 2048 workgroups x 4 wavefronts x {iters} rounds of 8 independent "
                       + ("v_mfma_f64_16x16x4_f64" if f64 else "v_mfma_f32_32x32x2_f32") + " on registers, no memory traffic",
                       dt, lambda: probe.mfma_peak(f64, iters, out), probe.mfma_peak_flops(f64, iters), float(out.numel() * out.element_size()),
                       "mfma")
            r["synthetic"] = True
            del out

    if "hbm_peak" in want:
        # Not a row of the method: a kernel that only reads 4 GiB, the on-device check of what HBM
        # delivers (the ceiling of the TTV and inner-product rows) for three launch shapes
        from paper_2203_08069_amd import probe
        src = operand(2, 0, (1 << 30,), np.float32)
        for blocks, in_flight in ((256, 8), (1024, 8), (2048, 16)):
            out = torch.empty(probe.hbm_read_out_bytes(blocks) // 4, dtype=torch.float32, device=dev)
            r = finish(f"hbm_read_{blocks}x{in_flight}",
                       f"synthetic: one read of a 4 GiB f32 array, {blocks} workgroups each on its own contiguous range, "
                       f"{in_flight} 16-byte non-temporal loads per lane in flight, nothing else",
                       "f32", lambda: probe.hbm_read(src, blocks, in_flight, out), 2.0 ** 30, 4.0 * 2 ** 30, "hbm")
            r["synthetic"] = True
            del out
        del src

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
