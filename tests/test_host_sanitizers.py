"""Host code under the address and undefined-behaviour sanitizers (no GPU involved).

  * the CPU oracle: its C file is compiled into a driver program with
    -fsanitize=address,undefined and run on cases whose operands sit in heap buffers of exactly
    their size (strided GEMM operands, every mode, empty extents); the results must equal the
    ordinary build's bit for bit, so the oracle the parity tests trust reads nothing it should not.
  * the library's launch planning (tile choice, the cut into two launches, MTTKRP ranges and
    workspace rows, the streaming kernels' ranges, the block-id -> tile map): a host-only header
    compiled the same way into tests/host_plan_check.cpp, which fuzzes the extents.
The sanitizer runtimes are linked statically, so nothing has to be preloaded.
"""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

from paper_2203_08069_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def compile_or_skip(cmd, exe):
    if shutil.which(cmd[0]) is None:
        pytest.skip(f"{cmd[0]} not available")
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "sanitize" in r.stderr and "cannot find" in r.stderr:
        pytest.skip("sanitizer runtimes are not installed: " + r.stderr.strip().splitlines()[-1])
    assert r.returncode == 0, r.stderr
    return exe


def test_launch_planning_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_plan_check")
    compile_or_skip(["g++", "-std=c++17", "-Wall", "-Werror"] + SAN +
                    [os.path.join(ROOT, "tests", "host_plan_check.cpp"), "-o", exe], exe)
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "host_plan_check: ok" in r.stdout


def cases():
    """(header, operands, oracle call) for every oracle function, both dtypes, awkward shapes."""
    out = []
    for di, dtype in enumerate((np.float32, np.float64)):
        t = lambda o, shape: inputs.tensor(80 + di, o, shape, dtype)
        # gemm: dense, sub-blocks of larger matrices with accumulate, empty sum
        A, B = t(0, (5, 7)), t(1, (7, 3))
        out.append(((0, di, 0, 5, 3, 7, 0, 7, 3, 0, 0), [A, B], lambda o, A=A, B=B: o.gemm(A, B)))
        bigA, bigB, bigC = t(2, (6, 11)), t(3, (9, 8)), t(4, (7, 9))
        As, Bs, Cs = bigA[1:5, 2:9], bigB[1:8, 3:7], bigC[2:6, 4:8]
        def window(v):
            """The (rows-1)*ld + cols elements of the parent buffer that a strided view spans."""
            ld = v.strides[0] // v.itemsize
            start = (v.__array_interface__['data'][0] - v.base.__array_interface__['data'][0]) // v.itemsize
            return v.base.reshape(-1)[start:start + (v.shape[0] - 1) * ld + v.shape[1]].copy(), ld
        (wa, lda), (wb, ldb), (wc, ldc) = window(As), window(Bs), window(Cs)
        out.append(((0, di, 0, 4, 4, 7, 0, lda, ldb, ldc, 1), [wa, wb, wc], lambda o, As=As, Bs=Bs, Cs=Cs: o.gemm(As, Bs, init=Cs)))
        out.append(((0, di, 0, 3, 2, 0, 0, 1, 2, 0, 0), [np.empty(0, dtype), np.empty(0, dtype)],
                    lambda o, dtype=dtype: o.gemm(np.empty((3, 0), dtype), np.empty((0, 2), dtype))))
        T, T2 = t(5, (3, 4, 5)), t(6, (3, 4, 5))
        c5, C54, C43, D54 = t(7, (5,)), t(8, (5, 4)), t(9, (4, 4)), t(10, (5, 4))
        out.append(((1, di, 0, 3, 4, 5, 0, 0, 0, 0, 0), [T, c5], lambda o, T=T, c5=c5: o.ttv(T, c5)))
        out.append(((2, di, 0, 3, 4, 5, 0, 0, 0, 0, 0), [T, T2], lambda o, T=T, T2=T2: np.array([o.innerprod(T, T2)])))
        n = (1 << 20) + 77                         # crosses the oracle's fixed summation blocks
        X, Y = t(11, (1, 1, n)), t(12, (1, 1, n))
        out.append(((2, di, 0, 1, 1, n, 0, 0, 0, 0, 0), [X, Y], lambda o, X=X, Y=Y: np.array([o.innerprod(X, Y)])))
        out.append(((3, di, 0, 3, 4, 5, 4, 0, 0, 0, 0), [T, C54], lambda o, T=T, C54=C54: o.ttm(T, C54)))
        out.append(((4, di, 0, 3, 4, 5, 4, 0, 0, 0, 0), [T, C43, D54], lambda o, T=T, C43=C43, D54=D54: o.mttkrp(T, C43, D54)))
        for mode in (0, 1, 2):
            Cm = t(13 + mode, (T.shape[mode], 6))
            out.append(((5, di, mode, 3, 4, 5, 6, 0, 0, 0, 0), [T, Cm], lambda o, T=T, Cm=Cm, mode=mode: o.ttm_mode(mode, T, Cm)))
            a, b = [m for m in (0, 1, 2) if m != mode]
            Fa, Fb = t(16 + mode, (T.shape[a], 3)), t(19 + mode, (T.shape[b], 3))
            out.append(((6, di, mode, 3, 4, 5, 3, 0, 0, 0, 0), [T, Fa, Fb],
                        lambda o, T=T, Fa=Fa, Fb=Fb, mode=mode: o.mttkrp_mode(mode, T, Fa, Fb)))
            cm = t(22 + mode, (T.shape[mode],))
            out.append(((7, di, mode, 3, 4, 5, 0, 0, 0, 0, 0), [T, cm], lambda o, T=T, cm=cm, mode=mode: o.ttv_mode(mode, T, cm)))
        E = np.empty((2, 0, 5), dtype)             # an empty tensor: outputs exist and are zero, or are empty
        out.append(((1, di, 0, 2, 0, 5, 0, 0, 0, 0, 0), [E, c5], lambda o, E=E, c5=c5: o.ttv(E, c5)))
        out.append(((4, di, 0, 2, 0, 5, 4, 0, 0, 0, 0), [E, np.empty((0, 4), dtype), D54],
                    lambda o, E=E, D54=D54, dtype=dtype: o.mttkrp(E, np.empty((0, 4), dtype), D54)))
    return out


def test_oracle_under_sanitizers(tmp_path, oracle):
    exe = str(tmp_path / "oracle_asan_driver")
    compile_or_skip(["gcc", "-std=c11", "-Wall", "-fopenmp", "-ffp-contract=off"] + SAN +
                    [os.path.join(ROOT, "oracle", "distal_oracle.c"), os.path.join(ROOT, "tests", "oracle_asan_driver.c"),
                     "-o", exe, "-lm"], exe)
    cs = cases()
    want = []
    with open(tmp_path / "cases.bin", "wb") as f:
        for header, operands, call in cs:
            f.write(struct.pack("<11q", *header))
            for a in operands:
                f.write(np.ascontiguousarray(a).tobytes())
            want.append(np.asarray(call(oracle), dtype=np.float64).reshape(-1))
    env = dict(ENV, OMP_NUM_THREADS="3")
    r = subprocess.run([exe, str(tmp_path / "cases.bin"), str(tmp_path / "results.bin")], capture_output=True,
                       text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert f"{len(cs)} cases ok" in r.stdout
    got = np.fromfile(tmp_path / "results.bin", dtype=np.float64)
    ref = np.concatenate(want)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref)
