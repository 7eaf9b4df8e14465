"""Build the HIP leaf-kernel library for gfx950 (MI355X) with hipcc.

    python -m paper_2203_08069_amd.build

hipcc cross-compiles without a GPU.  The shared object is written next to this
file (``libdistal.so``) so that it travels with the source tree.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdistal.so")
SOURCES = ["distal_api.hip"]
HEADERS = ["gemm_kernel.hpp", "mttkrp_kernel.hpp", "stream_kernels.hpp", "host_plan.hpp", "tile_map.hpp"]
# the measurement aid of include/distal_probe.h: a library of its own, never loaded by the binding
PROBE_LIB = os.path.join(HERE, "libdistal_probe.so")
PROBE_SOURCES = ["roofline_probe.hip"]

# Packed-FP32 VALU forms are switched off for every kernel of this library.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library cannot be built")
    return exe


def build_library(force: bool = True, extra_flags=()) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS] + \
        [os.path.join(os.path.dirname(HERE), "include", "distal.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc()] + HIPCC_FLAGS + list(extra_flags) + ["-o", tmp] + srcs
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    build_probe(force=force)
    return LIB


def build_probe(force: bool = True) -> str:
    srcs = [os.path.join(CSRC, s) for s in PROBE_SOURCES]
    deps = srcs + [os.path.join(os.path.dirname(HERE), "include", "distal_probe.h")]
    if not force and os.path.exists(PROBE_LIB) and all(os.path.getmtime(PROBE_LIB) >= os.path.getmtime(d) for d in deps):
        return PROBE_LIB
    tmp = PROBE_LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([hipcc()] + HIPCC_FLAGS + ["-o", tmp] + srcs)
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


if __name__ == "__main__":
    print(build_library(force=True, extra_flags=sys.argv[1:]))
