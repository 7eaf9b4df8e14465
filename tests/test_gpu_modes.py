"""GPU parity for the contractions along the other modes of the tensor (TTM and MTTKRP
along mode 0, 1 and 2), against the CPU oracle on the same seeded inputs.  Small and
ragged shapes are compared element by element; shapes large enough to reach the
big-tile launch configurations are compared on slices of the output that depend on a
slice of the input only, which the oracle recomputes from that slice."""
import numpy as np
import pytest

from paper_2203_08069_amd import inputs

import _util as U

pytestmark = pytest.mark.gpu

DT = [np.float32, np.float64]
KINDS = [inputs.UNIFORM, inputs.SMALLINT]


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2203_08069_amd import binding
    binding.load_library()          # raises if the HIP library was not built
    return binding


def empty(shape, dtype):
    import torch
    return torch.full(tuple(shape), float("nan"), dtype=getattr(torch, np.dtype(dtype).name), device="cuda:0")


def compare(got, ref, dtype, kind, klen, absref=None):
    """absref: a callable giving the oracle's result on the absolute values of the inputs, for
    the element-by-element bound (uniform inputs only; integer inputs must match exactly)."""
    if kind == inputs.SMALLINT:
        U.assert_exact(got, ref)
    else:
        U.assert_close(got, ref, dtype, klen)
        if absref is not None:
            U.assert_componentwise(got, ref, absref(), dtype, klen)


def out_shape(shape, mode, R):
    s = list(shape)
    s[mode] = R
    return tuple(s)


# ------------------------------------------------------------------ ttm along a mode

# (I, J, K, R): ragged, extent-1 modes, and shapes made of whole 128 x 128 tiles in each mode's
# matrix form (mode 0: R x JK over I; mode 1: per i, R x K over J)
TTM_MODE_SHAPES = [(3, 5, 7, 4), (17, 9, 33, 130), (32, 8, 32, 128), (130, 3, 44, 5), (1, 1, 1, 1),
                   (5, 40, 3, 1), (16, 128, 128, 128), (48, 2, 64, 256), (2, 19, 520, 36),
                   (70000, 2, 4, 3),           # mode 1: more problems in the batch than one grid dimension holds
                   # aligned pieces with a contracted extent that leaves trailing terms (37 is no multiple
                   # of the vector either: fine under a transposed left operand, a second pass along mode 2)
                   (37, 12, 20, 8), (21, 16, 24, 12), (8, 6, 37, 8)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("I,J,K,R", TTM_MODE_SHAPES)
def test_ttm_mode(lib, oracle, dtype, kind, mode, I, J, K, R):
    shape = (I, J, K)
    B, C = U.gen(40 + mode, 0, shape, dtype, kind), U.gen(40 + mode, 1, (shape[mode], R), dtype, kind)
    A = empty(out_shape(shape, mode, R), dtype)
    lib.distal_ttm_mode(mode, U.dev(B), U.dev(C), A)
    compare(U.host(A), oracle.ttm_mode(mode, B, C), dtype, kind, shape[mode],
            lambda: oracle.ttm_mode(mode, np.abs(B), np.abs(C)))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_ttm_mode_identity_and_permutation(lib, dtype, mode):
    shape = (24, 40, 56)
    B = U.gen(43, 0, shape, dtype)
    n = shape[mode]
    A = empty(shape, dtype)
    lib.distal_ttm_mode(mode, U.dev(B), U.dev(np.eye(n, dtype=dtype)), A)
    assert np.array_equal(U.host(A), B)
    perm = np.roll(np.arange(n), 3)
    lib.distal_ttm_mode(mode, U.dev(B), U.dev(np.ascontiguousarray(np.eye(n, dtype=dtype)[:, perm])), A)
    assert np.array_equal(U.host(A), np.take(B, perm, axis=mode))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
def test_ttm_mode1_many_batches_big_tiles(lib, oracle, dtype, kind):
    """mode 1 as a batch of I products R x K over J: 256 problems of one 256 x 256 tile each
    (the binary32 big-tile configuration); a few i are checked in full."""
    I, J, K, R = 256, 48, 256, 256
    B, C = U.gen(44, 0, (I, J, K), dtype, kind), U.gen(44, 1, (J, R), dtype, kind)
    A = empty((I, R, K), dtype)
    lib.distal_ttm_mode(1, U.dev(B), U.dev(C), A)
    got = U.host(A)
    assert np.all(np.isfinite(got))
    for i in (0, 1, 100, 255):
        compare(got[i:i + 1], oracle.ttm_mode(1, B[i:i + 1], C), dtype, kind, J)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
def test_ttm_mode0_wide_big_tiles(lib, oracle, dtype, kind):
    """mode 0 as one product R x JK over I with JK = 65536 (256 tiles of 256 x 256 in binary32);
    some j-slices are checked in full (A(:, j, :) depends on B(:, j, :) only)."""
    I, J, K, R = 32, 256, 256, 256
    B, C = U.gen(45, 0, (I, J, K), dtype, kind), U.gen(45, 1, (I, R), dtype, kind)
    A = empty((R, J, K), dtype)
    lib.distal_ttm_mode(0, U.dev(B), U.dev(C), A)
    got = U.host(A)
    assert np.all(np.isfinite(got))
    for j in (0, 77, 255):
        compare(got[:, j:j + 1, :], oracle.ttm_mode(0, np.ascontiguousarray(B[:, j:j + 1, :]), C), dtype, kind, I)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("I,J,K,R", [(200, 50, 40, 4080), (1028, 60, 68, 4000), (4100, 60, 68, 4000), (520, 60, 68, 4000),
                                     (1028, 60, 70, 4096), (1024, 64, 64, 4200)])
def test_ttm_mode0_ragged_edge_tiles(lib, oracle, dtype, kind, I, J, K, R):
    """mode 0 with R and J*K that are not whole tiles and a contracted extent with trailing terms:
    the transposed-left-operand kernels in their edge-clamping form (128 x 256 and 128 x 128 binary32 tiles;
    128 x 128 binary64 tiles); the last two shapes run as two launches in
    binary32, cut along the columns and along the rows.  Some j-slices are checked in full."""
    want = {(200, 4080): ((128, 128, 16), (128, 128, 16)), (1028, 4000): ((128, 256, 16), (128, 128, 16)),
            (4100, 4000): ((128, 256, 16), (128, 128, 16)), (520, 4000): ((128, 256, 16), (128, 128, 16)),
            (1028, 4096): ((128, 256, 16), None),
            (1024, 4200): ((128, 256, 16), None)}[(I, R)][int(dtype == np.float64)]
    plan = lib.gemm_plan(int(dtype == np.float64), True, R, J * K, I)
    assert want is None or plan[0] == want
    if dtype == np.float32 and (J, K) in ((60, 70), (64, 64)):
        assert plan[1] == (2 if R == 4096 else 1)
    B, C = U.gen(46, 0, (I, J, K), dtype, kind), U.gen(46, 1, (I, R), dtype, kind)
    A = empty((R, J, K), dtype)
    lib.distal_ttm_mode(0, U.dev(B), U.dev(C), A)
    got = U.host(A)
    assert np.all(np.isfinite(got))
    for j in (0, J // 2, J - 1):
        compare(got[:, j:j + 1, :], oracle.ttm_mode(0, np.ascontiguousarray(B[:, j:j + 1, :]), C), dtype, kind, I)


# (mode, I, J, K, R) with a rank-sized R and enough of the other side to fill the part: the tiles with a
# 32- or 64-wide short side (N side for mode 2, M side under a transposed left operand for modes 0
# and 1, there also as a batch), whole and in their edge-clamping form, with trailing K terms
NARROW_TTM = [(2, 256, 256, 64, 32), (2, 256, 255, 72, 24), (2, 256, 256, 64, 64),
              (0, 64, 256, 256, 32), (0, 60, 250, 260, 24), (0, 64, 256, 256, 64),
              (1, 128, 64, 512, 32), (1, 256, 72, 256, 64),
              # a rank or a kept extent that is not a multiple of the 16-byte vector: the trailing rows of
              # the transposed form go to the bounds-checked kernel, the trailing columns to the streaming one
              (0, 64, 256, 256, 33), (1, 128, 64, 512, 31), (1, 64, 64, 257, 32), (0, 64, 15, 17, 34), (2, 64, 250, 66, 29)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("mode,I,J,K,R", NARROW_TTM)
def test_ttm_mode_narrow_rank_tiles(lib, oracle, dtype, kind, mode, I, J, K, R):
    shape = (I, J, K)
    B, C = U.gen(48, 0, shape, dtype, kind), U.gen(48, 1, (shape[mode], R), dtype, kind)
    A = empty(out_shape(shape, mode, R), dtype)
    lib.distal_ttm_mode(mode, U.dev(B), U.dev(C), A)
    compare(U.host(A), oracle.ttm_mode(mode, B, C), dtype, kind, shape[mode],
            lambda: oracle.ttm_mode(mode, np.abs(B), np.abs(C)))


@pytest.mark.parametrize("dtype", DT)
def test_ttm_mode0_k_chunk_tiles(lib, oracle, dtype):
    """mode 0 with a contracted extent of 512 and 256 tiles of 256 x 128 (the binary32 k-chunk
    configuration with a transposed left operand)."""
    I, J, K, R = 512, 128, 256, 256
    B, C = U.gen(47, 0, (I, J, K), dtype), U.gen(47, 1, (I, R), dtype)
    A = empty((R, J, K), dtype)
    lib.distal_ttm_mode(0, U.dev(B), U.dev(C), A)
    got = U.host(A)
    assert np.all(np.isfinite(got))
    for j in (0, 64, 127):
        U.assert_close(got[:, j:j + 1, :], oracle.ttm_mode(0, np.ascontiguousarray(B[:, j:j + 1, :]), C), dtype, I)


def test_ttm_mode0_deep_binary64_big_tiles(lib, oracle):
    """binary64, contracted extent 4096 and 256 tiles of 256 x 128: the deep big-tile configuration."""
    dtype = np.float64
    I, J, K, R = 4096, 64, 512, 256
    B, C = U.gen(46, 0, (I, J, K), dtype), U.gen(46, 1, (I, R), dtype)
    A = empty((R, J, K), dtype)
    lib.distal_ttm_mode(0, U.dev(B), U.dev(C), A)
    got = U.host(A)
    assert np.all(np.isfinite(got))
    for j, k0 in ((0, 0), (31, 200), (63, 504)):
        ref = oracle.ttm_mode(0, np.ascontiguousarray(B[:, j:j + 1, k0:k0 + 8]), C)
        U.assert_close(got[:, j:j + 1, k0:k0 + 8], ref, dtype, I)


@pytest.mark.parametrize("dtype", DT)
def test_ttm_mode_zero_extents(lib, dtype):
    import torch
    tdt = getattr(torch, np.dtype(dtype).name)
    z = lambda *s: torch.zeros(s, dtype=tdt, device="cuda:0")
    A = empty((4, 3, 5), dtype)
    lib.distal_ttm_mode(0, z(0, 3, 5), z(0, 4), A)          # empty sum -> zeros
    assert np.array_equal(U.host(A), np.zeros((4, 3, 5)))
    A = empty((2, 4, 5), dtype)
    lib.distal_ttm_mode(1, z(2, 0, 5), z(0, 4), A)
    assert np.array_equal(U.host(A), np.zeros((2, 4, 5)))
    lib.distal_ttm_mode(1, z(2, 3, 0), z(3, 4), z(2, 4, 0))  # empty output: a no-op
    lib.distal_ttm_mode(0, z(2, 3, 5), z(2, 0), z(0, 3, 5))


# ------------------------------------------------------------------ ttv along a mode

TTV_MODE_SHAPES = [(3, 5, 7), (17, 9, 36), (64, 33, 128), (1, 1, 1), (300, 4, 8), (5, 700, 3), (40, 50, 1024),
                   (1000, 16, 64), (2, 1000, 260),
                   # few outputs and many rows to add: the kernels that split the rows inside a workgroup
                   # (16 or 8 lanes per run of a row; ragged runs; a batch of short walks along mode 1)
                   (200, 40, 300), (1030, 100, 100), (77, 1, 4100),
                   # odd output rows: element-aligned 16-byte accesses with an overlapping last piece
                   (300, 33, 101), (1000, 3, 4097), (50, 20, 33333), (70, 5, 5), (2, 66, 9),
                   # >= 256 spans of 16 KiB per row: the one-span-per-workgroup kernel, with a leftover row
                   # (mode 0: N = J*K = 2^20; mode 1: N = K, batch I)
                   (5, 1024, 1024), (9, 5, 262144)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("I,J,K", TTV_MODE_SHAPES)
def test_ttv_mode(lib, oracle, dtype, kind, mode, I, J, K):
    shape = (I, J, K)
    B, c = U.gen(48 + mode, 0, shape, dtype, kind), U.gen(48 + mode, 1, (shape[mode],), dtype, kind)
    A = empty([n for m, n in enumerate(shape) if m != mode], dtype)
    lib.distal_ttv_mode(mode, U.dev(B), U.dev(c), A)
    compare(U.host(A), oracle.ttv_mode(mode, B, c), dtype, kind, shape[mode],
            lambda: oracle.ttv_mode(mode, np.abs(B), np.abs(c)))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("mode", [0, 1])
def test_ttv_mode_closed_forms_and_zero_extents(lib, dtype, mode):
    import torch
    shape = (12, 20, 48)
    B = U.gen(49, 0, shape, dtype)
    n = shape[mode]
    keep = [x for m, x in enumerate(shape) if m != mode]
    A = empty(keep, dtype)
    e = np.zeros(n, dtype=dtype)
    e[n - 3] = 1
    lib.distal_ttv_mode(mode, U.dev(B), U.dev(e), A)
    assert np.array_equal(U.host(A), np.take(B, n - 3, axis=mode))
    lib.distal_ttv_mode(mode, U.dev(B), U.dev(np.ones(n, dtype=dtype)), A)
    U.assert_close(U.host(A), B.astype(np.float64).sum(axis=mode), dtype, n)
    tdt = getattr(torch, np.dtype(dtype).name)
    z = lambda *s: torch.zeros(s, dtype=tdt, device="cuda:0")
    if mode == 0:
        A = empty((3, 4), dtype)
        lib.distal_ttv_mode(0, z(0, 3, 4), z(0), A)
        assert np.array_equal(U.host(A), np.zeros((3, 4)))
        lib.distal_ttv_mode(0, z(2, 0, 4), z(2), z(0, 4))
    else:
        A = empty((2, 4), dtype)
        lib.distal_ttv_mode(1, z(2, 0, 4), z(0), A)
        assert np.array_equal(U.host(A), np.zeros((2, 4)))
        lib.distal_ttv_mode(1, z(2, 3, 0), z(3), z(2, 0))


# ------------------------------------------------------------------ mttkrp along a mode

def factor_shapes(shape, mode, L):
    a, b = [m for m in (0, 1, 2) if m != mode]
    return (shape[a], L), (shape[b], L)


# (I, J, K, L): ragged and tiny shapes (guarded kernels), shapes of whole blocks (vector kernels),
# several column tiles, one-i-per-range and several-i-per-range splits (odd and even counts)
MTTKRP_MODE_SHAPES = [(3, 5, 7, 4), (9, 33, 129, 5), (2, 70, 256, 32), (1, 1, 1, 1), (4, 16, 128, 32),
                      (6, 64, 128, 32), (40, 32, 256, 64), (50, 32, 64, 32), (7, 48, 200, 40),
                      (100, 256, 512, 32),
                      # whole aligned k-slices, ragged everything else: the vector kernels' ragged variants
                      (5, 37, 128, 33), (33, 50, 256, 16), (100, 17, 128, 48),
                      # ranks above 32: two column tiles per wavefront, whole (128) and ragged (96)
                      (6, 64, 128, 128), (5, 37, 128, 96),
                      # K a multiple of the 16-byte vector but not of a k-slice: vector kernels with a short
                      # last slice (one slice only; several; with two column tiles; binary64 only for 130)
                      (33, 50, 72, 16), (20, 40, 1000, 32), (12, 20, 132, 40), (6, 10, 1028, 64), (9, 21, 130, 8)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("I,J,K,L", MTTKRP_MODE_SHAPES)
def test_mttkrp_mode(lib, oracle, dtype, kind, mode, I, J, K, L):
    shape = (I, J, K)
    cs, ds = factor_shapes(shape, mode, L)
    B = U.gen(50 + mode, 0, shape, dtype, kind, 2)
    C, D = U.gen(50 + mode, 1, cs, dtype, kind, 2), U.gen(50 + mode, 2, ds, dtype, kind, 2)
    A = empty((shape[mode], L), dtype)
    lib.distal_mttkrp_mode(mode, U.dev(B), U.dev(C), U.dev(D), A)
    compare(U.host(A), oracle.mttkrp_mode(mode, B, C, D), dtype, kind, cs[0] * ds[0],
            lambda: oracle.mttkrp_mode(mode, np.abs(B), np.abs(C), np.abs(D)))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("mode", [1, 2])
def test_mttkrp_mode_selection_and_rank1(lib, dtype, mode):
    shape = (12, 32, 128)
    a, b = [m for m in (0, 1, 2) if m != mode]
    B = U.gen(53, 0, shape, dtype)
    L = 32
    C, D = np.zeros((shape[a], L), dtype=dtype), np.zeros((shape[b], L), dtype=dtype)
    for l in range(L):
        C[(3 * l + 1) % shape[a], l] = 1
        D[(5 * l + 2) % shape[b], l] = 1
    A = empty((shape[mode], L), dtype)
    lib.distal_mttkrp_mode(mode, U.dev(B), U.dev(C), U.dev(D), A)
    got = U.host(A)
    for l in range(L):
        idx = [slice(None)] * 3
        idx[a], idx[b] = (3 * l + 1) % shape[a], (5 * l + 2) % shape[b]
        assert np.array_equal(got[:, l], B[tuple(idx)])
    # all-ones rank-1 factors: sums over the two other modes
    A1 = empty((shape[mode], 1), dtype)
    lib.distal_mttkrp_mode(mode, U.dev(B), U.dev(np.ones((shape[a], 1), dtype)), U.dev(np.ones((shape[b], 1), dtype)), A1)
    ref = B.astype(np.float64).sum(axis=(a, b))
    U.assert_close(U.host(A1)[:, 0], ref, dtype, shape[a] * shape[b])


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("mode", [1, 2])
def test_mttkrp_mode_reproducible_and_zero_extents(lib, dtype, mode):
    import torch
    shape = (20, 64, 256)
    cs, ds = factor_shapes(shape, mode, 32)
    B, C, D = (U.dev(U.gen(54, o, s, dtype)) for o, s in ((0, shape), (1, cs), (2, ds)))
    outs = []
    for _ in range(2):
        A = empty((shape[mode], 32), dtype)
        lib.distal_mttkrp_mode(mode, B, C, D, A)
        outs.append(U.host(A).tobytes())
    assert outs[0] == outs[1]
    tdt = getattr(torch, np.dtype(dtype).name)
    z = lambda *s: torch.zeros(s, dtype=tdt, device="cuda:0")
    # an empty summed mode gives zeros; an empty output mode is a no-op
    A = empty((3 if mode == 1 else 4, 5), dtype)
    lib.distal_mttkrp_mode(mode, z(0, 3, 4), z(0, 5), z(4 if mode == 1 else 3, 5), A)
    assert np.array_equal(U.host(A), np.zeros(tuple(A.shape)))
    if mode == 1:
        lib.distal_mttkrp_mode(1, z(2, 0, 4), z(2, 5), z(4, 5), z(0, 5))
    else:
        lib.distal_mttkrp_mode(2, z(2, 3, 0), z(2, 5), z(3, 5), z(0, 5))


# ------------------------------------------------------------------ nothing is written out of bounds

SENTINEL = 12345.0


def banded(shape, dtype, offset):
    """A contiguous tensor of `shape` inside a larger buffer of sentinels, `offset` elements in."""
    import torch
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * 512,), SENTINEL, dtype=getattr(torch, np.dtype(dtype).name), device="cuda:0")
    return buf, buf[offset:offset + n].view(*shape), (offset, n)


def bands_untouched(buf, span):
    off, n = span
    h = U.host(buf)
    return bool(np.all(h[:off] == SENTINEL) and np.all(h[off + n:] == SENTINEL))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("offset", [256, 259])          # 16-byte aligned and misaligned outputs
@pytest.mark.parametrize("K", [70, 128])                # element-load kernels / vector kernels, ragged variants
def test_outputs_and_workspaces_stay_inside_their_buffers(lib, oracle, dtype, offset, K):
    import torch
    I, J, L = 5, 37, 33                                      # ragged in every other mode
    B = U.gen(80, 0, (I, J, K), dtype)
    dB = U.dev(B)
    code = 1 if dtype == np.float64 else 0
    esz = np.dtype(dtype).itemsize
    # ttv, ttm and ttm along every mode
    c = U.gen(80, 1, (K,), dtype)
    buf, A, span = banded((I, J), dtype, offset)
    lib.distal_ttv(dB, U.dev(c), A)
    U.assert_close(U.host(A), oracle.ttv(B, c), dtype, K)
    assert bands_untouched(buf, span)
    for mode in (0, 1):
        cm = U.gen(80, 3, (B.shape[mode],), dtype)
        buf, A, span = banded([n for m, n in enumerate(B.shape) if m != mode], dtype, offset)
        lib.distal_ttv_mode(mode, dB, U.dev(cm), A)
        U.assert_close(U.host(A), oracle.ttv_mode(mode, B, cm), dtype, B.shape[mode])
        assert bands_untouched(buf, span)
    for mode in (0, 1, 2):
        Cm = U.gen(80, 2, (B.shape[mode], L), dtype)
        shape = list(B.shape)
        shape[mode] = L
        buf, A, span = banded(shape, dtype, offset)
        lib.distal_ttm_mode(mode, dB, U.dev(Cm), A)
        U.assert_close(U.host(A), oracle.ttm_mode(mode, B, Cm), dtype, B.shape[mode])
        assert bands_untouched(buf, span)
    # mttkrp along every mode, with a workspace of exactly the advertised size inside sentinels
    for mode in (0, 1, 2):
        a, b = [m for m in (0, 1, 2) if m != mode]
        Cf, Df = U.gen(81, 1, (B.shape[a], L), dtype), U.gen(81, 2, (B.shape[b], L), dtype)
        need = lib.mttkrp_mode_workspace_bytes(code, mode, I, J, K, L)
        assert need > 0 and need % esz == 0
        wbuf, ws, wspan = banded((need // esz,), dtype, 256)            # workspaces must be 256-byte aligned
        buf, A, span = banded((B.shape[mode], L), dtype, offset)
        lib.distal_mttkrp_mode(mode, dB, U.dev(Cf), U.dev(Df), A, workspace=ws)
        U.assert_close(U.host(A), oracle.mttkrp_mode(mode, B, Cf, Df), dtype, B.shape[a] * B.shape[b])
        assert bands_untouched(buf, span) and bands_untouched(wbuf, wspan)
    # innerprod: scalar output and its workspace
    need = lib.innerprod_workspace_bytes(code, I, J, K)
    wbuf, ws, wspan = banded((need // 8,), np.float64, 256)
    buf, a_out, span = banded((1,), dtype, offset)
    lib.distal_innerprod(dB, dB, a_out, workspace=ws)
    ref = oracle.innerprod(B, B)
    assert abs(float(U.host(a_out)[0]) - ref) <= 4 * np.finfo(dtype).eps * abs(ref)
    assert bands_untouched(buf, span) and bands_untouched(wbuf, wspan)
