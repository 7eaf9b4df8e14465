"""Host-only checks of the C-ABI library: it loads, exports every symbol that
include/distal.h declares, and turns bad arguments into status codes before
anything is launched (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2203_08069_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "distal.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(distal_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    from paper_2203_08069_amd import binding
    assert declared_symbols() == sorted(binding.EXPORTS)


def test_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert lib.distal_version() >= 100
    seen = set()
    for code in range(0, 9):
        s = lib.distal_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert lib.distal_status_string(99).decode() == "unknown status"


P = ctypes.c_void_p
FAKE = 0x1000   # never dereferenced: every call below must fail validation first


def test_gemm_argument_errors(lib):
    g = lib.distal_gemm
    assert g(7, 4, 4, 4, P(FAKE), 4, P(FAKE + 256), 4, P(FAKE + 512), 4, 0, None) == 3
    assert g(0, -1, 4, 4, P(FAKE), 4, P(FAKE + 256), 4, P(FAKE + 512), 4, 0, None) == 2
    assert g(0, 1 << 40, 1 << 40, 4, P(FAKE), 4, P(FAKE + 256), 1 << 40, P(FAKE + 512), 1 << 40, 0, None) == 2
    assert g(0, 4, 4, 4, P(FAKE), 3, P(FAKE + 256), 4, P(FAKE + 512), 4, 0, None) == 4
    assert g(0, 4, 4, 4, P(FAKE), 4, P(FAKE + 256), 3, P(FAKE + 512), 4, 0, None) == 4
    assert g(0, 4, 4, 4, P(FAKE), 4, P(FAKE + 256), 4, P(FAKE + 512), 2, 0, None) == 4
    assert g(1, 4, 4, 4, None, 4, P(FAKE + 256), 4, P(FAKE + 512), 4, 0, None) == 1
    assert g(1, 4, 4, 4, P(FAKE), 4, P(FAKE + 256), 4, None, 4, 0, None) == 1
    assert g(1, 4, 4, 4, P(FAKE), 4, P(FAKE + 256), 4, P(FAKE), 4, 1, None) == 5
    # empty output: nothing to do, pointers are not needed
    assert g(1, 0, 4, 4, None, 4, None, 4, None, 4, 0, None) == 0
    assert g(1, 4, 0, 4, None, 4, None, 1, None, 1, 0, None) == 0


def test_tensor_call_argument_errors(lib):
    a, b, c, d, w = (P(FAKE + 256 * i) for i in range(5))
    assert lib.distal_ttm(2, 2, 2, 2, 2, a, b, c, None) == 3
    assert lib.distal_ttm(0, 2, -2, 2, 2, a, b, c, None) == 2
    assert lib.distal_ttm(0, 1 << 31, 1 << 31, 1 << 31, 2, a, b, c, None) == 2
    assert lib.distal_ttm(0, 2, 2, 2, 2, None, b, c, None) == 1
    assert lib.distal_ttm(0, 2, 2, 2, 2, a, b, a, None) == 5
    assert lib.distal_ttv(0, 2, 2, 2, a, None, c, None) == 1
    assert lib.distal_ttv(0, 2, 2, -1, a, b, c, None) == 2
    assert lib.distal_ttv(1, 2, 2, 2, a, b, b, None) == 5
    assert lib.distal_ttv(5, 2, 2, 2, a, b, c, None) == 3
    assert lib.distal_ttv(0, 0, 2, 2, None, None, None, None) == 0
    assert lib.distal_mttkrp(0, 2, 2, 2, 2, a, b, c, None, w, 1 << 20, None) == 1
    assert lib.distal_mttkrp(0, 2, 2, 2, 2, a, b, c, a, w, 1 << 20, None) == 5
    assert lib.distal_mttkrp(0, 2, 2, 2, -2, a, b, c, d, w, 1 << 20, None) == 2
    assert lib.distal_mttkrp(9, 2, 2, 2, 2, a, b, c, d, w, 1 << 20, None) == 3
    # the sum over j is split into ranges: workspace is then mandatory, big enough and aligned
    need = lib.distal_mttkrp_workspace_bytes(0, 4, 1000, 8, 32)
    # I rows x 500 ranges of two j x 1 k-slice x L partial sums, in floats
    assert need == (4 * 500 * 32) * 4
    # one j and one k-slice: the only partial row of an i is the output row, no workspace
    assert lib.distal_mttkrp_workspace_bytes(0, 4, 1, 8, 32) == 0
    assert lib.distal_mttkrp(0, 4, 1000, 8, 32, a, b, c, d, None, 0, None) == 6
    assert lib.distal_mttkrp(0, 4, 1000, 8, 32, a, b, c, d, w, need - 1, None) == 6
    assert lib.distal_mttkrp(0, 4, 1000, 8, 32, a, b, c, d, P(FAKE + 8), need, None) == 6
    assert lib.distal_mttkrp(0, 0, 1000, 8, 32, None, None, None, None, None, 0, None) == 0
    need = lib.distal_innerprod_workspace_bytes(0, 2, 2, 2)
    assert need > 0 and need % 8 == 0
    assert lib.distal_innerprod(0, 2, 2, 2, a, b, None, w, need, None) == 1
    assert lib.distal_innerprod(0, 2, 2, 2, a, b, a, w, need, None) == 5
    assert lib.distal_innerprod(0, 2, 2, 2, a, b, c, None, 0, None) == 6
    assert lib.distal_innerprod(0, 2, 2, 2, a, b, c, w, need - 8, None) == 6
    assert lib.distal_innerprod(0, 2, 2, 2, a, b, c, P(FAKE + 4), need, None) == 6
    assert lib.distal_innerprod(0, 2, 2, 2, a, b, c, c, need, None) == 5
    assert lib.distal_innerprod(0, 2, -2, 2, a, b, c, w, need, None) == 2
    assert lib.distal_innerprod(3, 2, 2, 2, a, b, c, w, need, None) == 3
    assert lib.distal_mttkrp_workspace_bytes(7, 1, 1, 1, 1) == 0
    assert lib.distal_innerprod_workspace_bytes(0, -1, 1, 1) == 0


def test_binding_refuses_host_tensors():
    import torch
    from paper_2203_08069_amd import binding
    x = torch.zeros(2, 2)
    with pytest.raises((ValueError, TypeError)):
        binding.distal_gemm(x, x, torch.zeros(2, 2))
    with pytest.raises(TypeError):
        binding._dtype_code(torch.zeros(2, dtype=torch.int32))


def test_missing_library_is_an_error(tmp_path):
    from paper_2203_08069_amd import binding
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library(str(tmp_path / "libdistal.so"))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2203_08069_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "distal_oracle" not in text, f
    otext = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + \
        open(os.path.join(ROOT, "oracle", "distal_oracle.c")).read()
    assert "paper_2203_08069_amd" not in otext and "distal.h" not in otext


def test_mode_call_argument_errors(lib):
    a, b, c = (P(FAKE + 256 * i) for i in range(3))
    t = lib.distal_ttm_mode
    assert t(0, 3, 2, 2, 2, 2, a, b, c, None) == 8
    assert t(0, -1, 2, 2, 2, 2, a, b, c, None) == 8
    assert t(5, 1, 2, 2, 2, 2, a, b, c, None) == 3
    for mode in (0, 1, 2):
        assert t(0, mode, 2, -2, 2, 2, a, b, c, None) == 2
        assert t(0, mode, 1 << 31, 1 << 31, 1 << 31, 2, a, b, c, None) == 2
        assert t(0, mode, 2, 2, 2, 2, None, b, c, None) == 1
        assert t(0, mode, 2, 2, 2, 2, a, None, c, None) == 1
        assert t(0, mode, 2, 2, 2, 2, a, b, None, None) == 1
        assert t(0, mode, 2, 2, 2, 2, a, b, a, None) == 5
        assert t(1, mode, 2, 2, 2, 0, None, None, None, None) == 0      # empty output


def test_ttv_mode_argument_errors(lib):
    a, b, c = (P(FAKE + 256 * i) for i in range(3))
    t = lib.distal_ttv_mode
    assert t(0, 3, 2, 2, 2, a, b, c, None) == 8
    assert t(6, 0, 2, 2, 2, a, b, c, None) == 3
    for mode in (0, 1, 2):
        assert t(0, mode, 2, 2, -1, a, b, c, None) == 2
        assert t(0, mode, 1 << 31, 1 << 31, 1 << 31, a, b, c, None) == 2
        assert t(0, mode, 2, 2, 2, None, b, c, None) == 1
        assert t(0, mode, 2, 2, 2, a, None, c, None) == 1
        assert t(0, mode, 2, 2, 2, a, b, None, None) == 1
        assert t(0, mode, 2, 2, 2, a, b, a, None) == 5
    assert t(1, 0, 3, 0, 2, None, None, None, None) == 0          # empty output
    assert t(1, 1, 0, 3, 2, None, None, None, None) == 0


def test_mttkrp_mode_argument_errors(lib):
    a, b, c, d, w = (P(FAKE + 256 * i) for i in range(5))
    m = lib.distal_mttkrp_mode
    assert m(0, 3, 2, 2, 2, 2, a, b, c, d, w, 1 << 20, None) == 8
    assert m(4, 1, 2, 2, 2, 2, a, b, c, d, w, 1 << 20, None) == 3
    for mode in (0, 1, 2):
        assert m(0, mode, 2, 2, -2, 2, a, b, c, d, w, 1 << 20, None) == 2
        assert m(0, mode, 2, 2, 2, 2, a, b, c, None, w, 1 << 20, None) == 1
        assert m(0, mode, 2, 2, 2, 2, None, b, c, d, w, 1 << 20, None) == 1
        assert m(0, mode, 2, 2, 2, 2, a, b, c, a, w, 1 << 20, None) == 5
        assert m(0, mode, 0, 0, 0, 4, None, None, None, None, None, 0, None) == 0
    # several ranges of i: one partial row per (range, k-slice) resp. (range, group of 64 j)
    lib.distal_mttkrp_mode_workspace_bytes.restype = ctypes.c_size_t
    need1 = lib.distal_mttkrp_mode_workspace_bytes(0, 1, 10, 32, 64, 32)
    assert need1 == 32 * 10 * 32 * 4          # J rows x 10 ranges x 1 slice x L floats
    need2 = lib.distal_mttkrp_mode_workspace_bytes(0, 2, 10, 32, 128, 32)
    assert need2 == 128 * 10 * 32 * 4         # K rows x 10 ranges x 1 group x L floats
    assert lib.distal_mttkrp_mode_workspace_bytes(0, 1, 1, 32, 64, 32) == 0
    assert lib.distal_mttkrp_mode_workspace_bytes(0, 0, 4, 1000, 8, 32) == lib.distal_mttkrp_workspace_bytes(0, 4, 1000, 8, 32)
    assert m(0, 1, 10, 32, 64, 32, a, b, c, d, None, 0, None) == 6
    assert m(0, 1, 10, 32, 64, 32, a, b, c, d, w, need1 - 1, None) == 6
    assert m(0, 2, 10, 32, 128, 32, a, b, c, d, P(FAKE + 8), need2, None) == 6


def test_gemm_plan_choice(lib):
    """The host-side tile choice for the shapes the benchmark rows and the schedules issue, for
    narrow rank-sized outputs, ragged shapes (padding and the last round of tiles count) and
    small problems; and its argument checks."""
    from paper_2203_08069_amd import binding
    F32, F64 = 0, 1
    tile, plan = binding.gemm_tile, binding.gemm_plan
    # the headline product in both types, and the benchmark's tensor-times-matrix shape along modes 2, 0, 1
    assert tile(F64, False, 8192, 8192, 8192) == (128, 128, 16)
    assert tile(F32, False, 8192, 8192, 8192) == (128, 128, 16)
    assert tile(F32, False, 1 << 20, 256, 1024) == (128, 128, 16)
    assert tile(F32, True, 256, 1 << 20, 1024) == (128, 128, 16)
    assert tile(F32, True, 256, 1024, 1024, batch=1024) == (128, 128, 16)
    assert tile(F64, False, 1 << 20, 256, 1024) == (128, 128, 16)
    # SUMMA k-chunks
    for K in (256, 512, 1024, 2048):
        assert tile(F64, False, 8192, 8192, K) == (128, 128, 16)
    for K in (128, 256, 512, 1040):
        assert tile(F32, False, 8192, 8192, K) == (128, 128, 16)
    assert tile(F32, False, 4096, 4096, 4096) == (128, 256, 16)     # two tiles per compute unit
    assert tile(F32, False, 1 << 20, 128, 1024) == (128, 128, 16)
    # rank-sized outputs: a 32- or 64-wide short side on the narrow operand's side
    assert tile(F32, False, 1 << 20, 32, 1024) == (128, 32, 32)
    assert tile(F32, False, 1 << 20, 64, 1024) == (128, 64, 32)
    assert tile(F32, True, 32, 1 << 20, 1024) == (32, 256, 32)
    assert tile(F64, False, 1 << 19, 16, 1024) == (128, 32, 16)
    assert tile(F64, True, 64, 1 << 19, 1024) == (64, 128, 16)
    # ragged: 8200 rows are 16.25 rounds of 128 x 128 tiles: the first 8192 rows are sixteen whole rounds
    # of them (the tile reported), the other 8 rows a second launch of small tiles
    assert tile(F64, False, 8200, 8192, 8192) == (128, 128, 16)
    # 8000^3: 3969 tiles of 128 x 128 pad the output by 1.6 %, 7875 of 64 x 128 by 0.8 %
    assert tile(F64, False, 8000, 8000, 8000) == (64, 128, 16)
    # 3000^3: 576 tiles of 128 x 128 are 2.25 rounds of one or two tiles per compute unit, where that
    # tile runs below its speed; 2209 tiles of 64 x 64 are nine rounds at full speed
    assert plan(F64, False, 3000, 3000, 3000) == ((64, 64, 16), 0, 0, (0, 0, 0))
    # binary32: 64 x 64 tiles take 32-deep slabs from K = 256 on
    assert plan(F32, False, 3000, 3000, 3000) == ((128, 128, 16), 1, 2688, (64, 64, 32))
    assert plan(F32, False, 3500, 3500, 3500) == ((64, 64, 32), 0, 0, (0, 0, 0))
    # 2000^3: two 128 x 64 tiles per compute unit
    assert plan(F32, False, 2000, 2000, 2000) == ((128, 64, 32), 0, 0, (0, 0, 0))
    assert plan(F32, False, 2000, 2000, 200) == ((128, 64, 32), 0, 0, (0, 0, 0))
    assert plan(F32, False, 3000, 2040, 100) == ((64, 128, 32), 0, 0, (0, 0, 0))
    assert plan(F64, False, 2048, 2048, 2048) == ((64, 128, 16), 0, 0, (0, 0, 0))      # two per compute unit
    assert tile(F32, False, 1024, 1024, 128) == (64, 64, 16)
    assert plan(F32, False, 4000, 2040, 100) == ((128, 128, 16), 0, 0, (0, 0, 0))
    # small problems: quarter-size tiles
    assert tile(F32, False, 1024, 1024, 1024) == (64, 64, 32)
    assert tile(F64, False, 300, 200, 100) == (64, 64, 16)
    # the two-launch plans: whole rounds of large tiles first, the rest on small tiles
    assert plan(F64, False, 8192, 8192, 8192) == ((128, 128, 16), 0, 0, (0, 0, 0))
    assert plan(F64, False, 8200, 8192, 8192) == ((128, 128, 16), 1, 8192, (64, 64, 16))
    assert plan(F64, False, 8192, 8200, 8192) == ((128, 128, 16), 2, 8192, (64, 64, 16))
    assert plan(F64, False, 5000, 5000, 5000) == ((128, 128, 16), 1, 4864, (64, 64, 16))
    assert plan(F32, False, 4200, 4096, 1024) == ((128, 256, 16), 1, 4096, (64, 64, 32))
    assert plan(F32, False, 8200, 8192, 8192) == ((128, 128, 16), 1, 8192, (64, 64, 32))
    tile3, rest3 = (ctypes.c_int * 3)(), (ctypes.c_int * 3)()
    split, cut = ctypes.c_int(), ctypes.c_int64()
    refs = (tile3, ctypes.byref(split), ctypes.byref(cut), rest3)
    assert lib.distal_gemm_plan(7, 0, 8, 8, 8, 1, 0, *refs) == 3
    assert lib.distal_gemm_plan(0, 0, 0, 8, 8, 1, 0, *refs) == 2
    assert lib.distal_gemm_plan(0, 0, 8, 8, 8, 0, 0, *refs) == 2
    assert lib.distal_gemm_plan(0, 0, 8, 8, 8, 1, 0, None, None, None, None) == 1
    # added onto an old C, binary32 takes the 128 x 128 tile from K = 512 on and 64 x 128 tiles for thinner
    # steps; binary64 changes tile only for steps of at most 128 terms
    for K in (512, 1024, 4096):
        assert tile(F32, False, 8192, 8192, K, accumulate=True) == (128, 128, 16)
    assert tile(F32, False, 8192, 8192, 256, accumulate=True) == (64, 128, 32)      # thin and bound by C's traffic
    for K in (256, 1024, 8192):
        assert plan(F64, False, 8192, 8192, K, accumulate=True) == plan(F64, False, 8192, 8192, K)
    assert tile(F64, False, 8192, 8192, 128, accumulate=True) == (64, 128, 16)      # bound by C's traffic
    assert tile(F64, False, 8192, 8192, 128) == (128, 128, 16)


def test_gemm_peeled_columns(lib):
    """Rows of the right operand that end inside a 16-byte piece: a narrow output stays whole (a second
    pass over the left operand would double the time), a wide one has its trailing columns peeled
    off (that pass costs a percent and the rest runs on whole pieces); fewer columns than one
    piece all go to the streaming kernel."""
    from paper_2203_08069_amd import binding
    peeled = binding.gemm_peeled_columns
    F32, F64 = 0, 1
    for dt, vec in ((F32, 4), (F64, 2)):
        for N in (vec, 32, 8192):
            assert peeled(dt, False, 8192, N, 8192) == 0
        for N in range(1, vec):
            assert peeled(dt, False, 1 << 20, N, 1000) == N
        for N in (vec + 1, 31, 33):
            assert peeled(dt, False, 1000000, N, 1000) == 0, (dt, N)         # rank-sized outputs of TTM
        for N in (4097, 8191):
            assert peeled(dt, False, 8192, N, 8192) == N % vec, (dt, N)
        assert peeled(dt, True, 256, 1000 * 1000 + 1, 1000) in (0, 1)
    assert peeled(7, False, 8, 8, 8) == -1 and peeled(F32, False, 0, 8, 8) == -1 and peeled(F32, False, 8, 8, 8, batch=0) == -1
    assert peeled(F32, False, 1 << 40, 1 << 40, 8) == -1


def test_ttm_slices_plan(lib):
    """Where the last-mode TTM keeps its factor in registers: at most 32 columns, at least 65536 rows
    of whole 16-byte pieces, at most 32 slices of 256 bytes of which at least seven eighths are used;
    three and four slices per wavefront only on whole slices."""
    from paper_2203_08069_amd import binding
    ns = binding.ttm_slices_per_wave
    F32, F64 = 0, 1
    R = 1 << 20
    assert [ns(F32, R, K, 32) for K in (512, 1024, 1536, 2048, 1000, 960, 448)] == [1, 2, 3, 4, 2, 2, 1]
    assert [ns(F64, R, K, 32) for K in (256, 512, 768, 1024, 500, 480, 224)] == [1, 2, 3, 4, 2, 2, 1]
    assert ns(F32, R, 1024, 1) == 2 and ns(F32, R, 1024, 33) == 0 and ns(F32, R, 1024, 0) == 0
    assert ns(F32, R, 768, 32) == 0 and ns(F32, R, 256, 32) == 0        # too many idle wavefronts
    assert ns(F32, R, 4096, 32) == 0 and ns(F64, R, 2048, 32) == 0      # the factor does not fit the registers
    assert ns(F32, R, 1022, 32) == 0 and ns(F64, R, 511, 32) == 0       # rows are not whole 16-byte pieces
    assert ns(F32, R, 2000, 32) == 0 and ns(F64, R, 1000, 32) == 0      # four slices: whole slices only
    assert ns(F32, R, 1500, 32) == 0 and ns(F64, R, 760, 32) == 0       # and three
    assert ns(F32, R - 1, 2048, 32) == 4 and ns(F32, R - 1, 1536, 32) == 3     # rows beyond whole blocks are no obstacle
    assert ns(F32, 65535, 1024, 32) == 0 and ns(F32, 65536, 1024, 32) == 2
    assert ns(7, R, 1024, 32) == 0 and ns(F32, -1, 1024, 32) == 0


def test_gemm_plan_invariants_on_random_extents(lib):
    """Whatever the extents: tiles come from the dtype's set, narrow tiles only serve narrow outputs,
    slabs are no deeper than K allows the kernels to start (K >= BK or the guarded kernel is used),
    a cut is a positive multiple of the first tile inside the extent it cuts."""
    import random
    from paper_2203_08069_amd import binding
    rng = random.Random(5)
    tiles = {0: {(256, 256), (256, 128), (128, 256), (128, 128), (64, 64), (128, 64), (64, 128), (256, 64), (128, 32), (64, 256), (32, 256)},
             1: {(256, 128), (128, 128), (64, 64), (128, 64), (128, 32), (64, 128), (32, 256)}}
    pick = lambda: rng.choice([1, 4, 8, 16, 24, 32, 48, 64, 100, 128, 250, 256, 512, 1000, 1024, 3000, 4096, 5000, 8192, 8200,
                               65536, 1 << 20]) + rng.choice([0, 0, 0, 4, -4 if rng.random() < .5 else 8])
    for _ in range(3000):
        dt, ta = rng.randrange(2), rng.randrange(2)
        M, N, K = max(1, pick()), max(1, pick()), max(16, pick())
        batch = rng.choice([1, 1, 1, 7, 1024])
        if M * N * batch > 1 << 44:
            continue
        tile, split, cut, rest = binding.gemm_plan(dt, bool(ta), M, N, K, batch)
        assert binding.gemm_plan(dt, bool(ta), M, N, K, batch) == (tile, split, cut, rest)

        def ok(t, m, n):
            assert (t[0], t[1]) in tiles[dt], (t, dt)
            assert t[2] in (16, 32) and t[2] <= max(K, 16), (t, K)
            if t[1] < 64 or (t[1] == 64 and t[0] == 256):
                assert n <= 64, (t, n)              # a narrow N side only for a narrow N
            if t[0] < 64 or (t[0] == 64 and t[1] == 256):
                assert m <= 64, (t, m)
        if split == 0:
            ok(tile, M, N)
            assert cut == 0 and rest == (0, 0, 0)
        elif split == 1:
            assert 0 < cut < M and cut % tile[0] == 0
            ok(tile, M, N), ok(rest, M - cut, N)
        else:
            assert split == 2 and 0 < cut < N and cut % tile[1] == 0
            ok(tile, M, N), ok(rest, M, N - cut)


def test_binding_refuses_views_whose_rows_overlap():
    """A row stride below the row length (expand(), overlapping as_strided) must raise in the
    binding instead of reaching the kernels with a leading dimension that was silently raised."""
    import torch
    from paper_2203_08069_amd import binding
    row = torch.zeros(1, 8)
    with pytest.raises(ValueError):
        binding._row_stride(row.expand(5, 8), "A")                     # stride(0) == 0
    with pytest.raises(ValueError):
        binding._row_stride(torch.zeros(64).as_strided((5, 8), (4, 1)), "A")   # rows overlap
    with pytest.raises(ValueError):
        binding._row_stride(torch.zeros(8, 8).t(), "A")                # columns not contiguous
    assert binding._row_stride(torch.zeros(5, 8), "A") == 8
    assert binding._row_stride(torch.zeros(5, 16)[:, 3:11], "A") == 16     # a column slice keeps its stride
    assert binding._row_stride(row, "A") == 8                          # one row: the row length
    assert binding._row_stride(torch.zeros(64).as_strided((5, 8), (8, 1)), "A") == 8


def test_noalloc_argument_errors(lib):
    """The allocation-free entry point validates on the host before it touches the device."""
    a, b, c = (P(FAKE + 256 * i) for i in range(3))
    f = lib.distal_innerprod_noalloc
    assert f(9, 2, 2, 2, a, b, c, None) == 3
    assert f(0, 2, -2, 2, a, b, c, None) == 2
    assert f(0, 1 << 31, 1 << 31, 1 << 31, a, b, c, None) == 2
    assert f(0, 2, 2, 2, None, b, c, None) == 1
    assert f(0, 2, 2, 2, a, b, None, None) == 1
    assert f(1, 2, 2, 2, a, b, a, None) == 5


def test_gemm_tiled_argument_errors(lib):
    """The caller-chosen-tile product validates tile, extents, strides and pointers on the host."""
    a, b, c = (P(FAKE + 256 * i) for i in range(3))
    f = lib.distal_gemm_tiled
    ok = (64, 64, 64, a, 64, b, 64, c, 64, 0, None)
    assert f(9, 0, 64, 64, *ok) == 3
    for dt, bm, bn in ((1, 256, 256), (1, 256, 64), (1, 64, 256), (0, 48, 48), (0, 0, 0), (0, 64, 32), (1, 256, 32)):
        assert f(dt, 0, bm, bn, *ok) == 2, (dt, bm, bn)          # no kernel of that tile for the dtype
    assert f(0, 0, 64, 64, -1, 64, 64, a, 64, b, 64, c, 64, 0, None) == 2
    assert f(0, 0, 64, 64, 64, 64, 64, a, 63, b, 64, c, 64, 0, None) == 4
    assert f(0, 1, 64, 64, 128, 64, 64, a, 64, b, 64, c, 64, 0, None) == 4      # stored K x M: lda >= M
    assert f(0, 0, 64, 64, 64, 64, 64, a, 64, b, 63, c, 64, 0, None) == 4
    assert f(0, 0, 64, 64, 64, 64, 64, a, 64, b, 64, c, 63, 0, None) == 4
    assert f(0, 0, 64, 64, 64, 64, 64, None, 64, b, 64, c, 64, 0, None) == 1
    assert f(0, 0, 64, 64, 64, 64, 64, a, 64, b, 64, None, 64, 0, None) == 1
    assert f(0, 0, 64, 64, 64, 64, 64, a, 64, b, 64, a, 64, 0, None) == 5
    assert f(1, 1, 128, 64, 0, 64, 64, None, 64, None, 64, None, 64, 0, None) == 0   # empty output: nothing to do


def test_gemm_ws_workspace_sizes_and_argument_errors(lib):
    """The product that is cut along k: which extents are cut (and into how many M x N slabs), and
    the host-side checks of the call; extents that are not cut behave as distal_gemm and ignore
    the workspace."""
    F32, F64 = 0, 1
    wb, f = lib.distal_gemm_workspace_bytes, lib.distal_gemm_ws
    assert wb(F64, 512, 512, 8192) == 8 * 512 * 512 * 8            # 64 tiles of 64 x 64: eight parts of 1024
    assert wb(F64, 512, 512, 65536) == 32 * 512 * 512 * 8          # deep enough for 16 tiles of 128 x 128 in 32 parts
    assert wb(F32, 256, 256, 1 << 20) == 64 * 256 * 256 * 4        # the cap of 64 parts
    assert wb(F64, 64, 64, 1 << 20) == 64 * 64 * 64 * 8            # one tile: 64 parts
    assert wb(F64, 100, 100, 3000) == 2 * 100 * 100 * 8            # parts stay at least 1024 deep
    assert wb(F64, 1024, 1024, 8192) == 0                          # every compute unit has a tile already
    assert wb(F64, 512, 512, 2047) == 0 and wb(F64, 512, 512, 0) == 0 and wb(F64, 0, 512, 8192) == 0
    assert wb(7, 512, 512, 8192) == 0 and wb(F64, -1, 512, 8192) == 0
    a, b, c, w = (P(FAKE + 256 * i) for i in range(4))
    big = 1 << 40
    cut = (512, 512, 8192)
    assert f(F64, *cut, a, 8192, b, 512, c, 512, 0, None, 0, None) == 6
    assert f(F64, *cut, a, 8192, b, 512, c, 512, 0, w, wb(F64, *cut) - 1, None) == 6
    assert f(F64, *cut, a, 8192, b, 512, c, 512, 0, P(FAKE + 8), big, None) == 6          # misaligned
    assert f(F64, *cut, a, 8192, b, 512, c, 512, 0, a, big, None) == 5
    assert f(F64, *cut, a, 8192, b, 512, a, 512, 0, w, big, None) == 5
    assert f(F64, *cut, None, 8192, b, 512, c, 512, 0, w, big, None) == 1
    assert f(F64, *cut, a, 8191, b, 512, c, 512, 0, w, big, None) == 4
    assert f(F64, *cut, a, 8192, b, 511, c, 512, 0, w, big, None) == 4
    assert f(9, *cut, a, 8192, b, 512, c, 512, 0, w, big, None) == 3
    # not cut: distal_gemm's checks, no workspace needed
    assert f(F64, 64, 64, -1, a, 64, b, 64, c, 64, 0, None, 0, None) == 2
    assert f(F64, 64, 64, 64, a, 63, b, 64, c, 64, 0, None, 0, None) == 4
    assert f(F64, 0, 64, 64, None, 64, None, 64, None, 64, 0, None, 0, None) == 0


def test_probe_library_exports_and_argument_errors():
    """The measurement aid (include/distal_probe.h) is a library of its own: it loads, exports what
    its header declares and validates on the host before launching."""
    from paper_2203_08069_amd import build, probe
    if not os.path.exists(probe.LIB_PATH):
        build.build_probe()
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "distal_probe.h")).read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(distal_probe_[a-z_]+)\s*\(", text)))
    assert declared == sorted(probe.EXPORTS)
    lib = probe.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    f = lib.distal_probe_stream_mfma
    a, b, c = (P(FAKE + 256 * i) for i in range(3))
    assert lib.distal_probe_out_bytes(1024, 1024, 1024) == 768 * 256 * 16 * 4
    assert lib.distal_probe_out_bytes(1000, 1024, 1024) == 0
    assert f(1000, 8, 256, a, b, 1, c, 1 << 30, None) == 2          # I not a multiple of 32
    assert f(32, 8, 100, a, b, 1, c, 1 << 30, None) == 2            # K not a multiple of 256
    assert f(32, 8, 256, None, b, 1, c, 1 << 30, None) == 1
    assert f(32, 8, 256, P(FAKE + 4), b, 1, c, 1 << 30, None) == 4
    assert f(32, 8, 256, a, b, 1, c, 16, None) == 6
    g = lib.distal_probe_mfma_peak
    assert lib.distal_probe_mfma_peak_out_bytes(1) == 2048 * 256 * 8 and lib.distal_probe_mfma_peak_out_bytes(0) == 2048 * 256 * 4
    assert lib.distal_probe_mfma_peak_flops(1, 10) == 2048 * 4 * 10 * 8 * 2048.0      # 16x16x4: 2048 flop per instruction
    assert lib.distal_probe_mfma_peak_flops(0, 10) == 2048 * 4 * 10 * 8 * 4096.0      # 32x32x2: 4096
    assert g(1, 0, c, 1 << 30, None) == 2
    assert g(1, 10, None, 1 << 30, None) == 1
    assert g(0, 10, c, 16, None) == 6
    r = lib.distal_probe_hbm_read
    assert lib.distal_probe_hbm_read_out_bytes(256) == 256 * 256 * 4 and lib.distal_probe_hbm_read_out_bytes(0) == 0
    big = 1 << 30
    assert r(None, 1 << 20, 256, 8, c, big, None) == 1 and r(c, 1 << 20, 256, 8, None, big, None) == 1
    assert r(c, 24, 256, 8, c, big, None) == 2 and r(c, 0, 256, 8, c, big, None) == 2      # not whole 16-byte pieces
    assert r(c, 1 << 20, 0, 8, c, big, None) == 2 and r(c, 1 << 20, 256, 5, c, big, None) == 2
    assert r(ctypes.c_void_p(FAKE + 4), 1 << 20, 256, 8, c, big, None) == 4
    assert r(c, 1 << 20, 256, 8, c, 1024, None) == 6


def test_package_and_library_versions_agree(lib):
    import paper_2203_08069_amd as pkg
    major, minor, patch = (int(x) for x in pkg.__version__.split()[0].strip('"').split("."))
    assert lib.distal_version() == major * 10000 + minor * 100 + patch
