"""GPU parity: every C-ABI entry point against the CPU oracle, element by element,
on the same seeded inputs.  Sizes span several tiles and ragged tails."""
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


# ------------------------------------------------------------------ gemm

GEMM_SHAPES = [(1, 1, 1), (256, 256, 256), (127, 129, 17), (130, 260, 33), (300, 200, 100),
               (128, 128, 16), (64, 384, 1000), (513, 31, 8),
               (384, 256, 48),          # whole 128 x 128 tiles: straight-line kernel
               (4096, 4096, 32),        # 256 big tiles (fp32 256 x 256 ...)
               (4096, 2048, 32)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm(lib, oracle, dtype, kind, M, N, K):
    seed = 0 if (M, N, K) == (256, 256, 256) else 100 + M
    A, B = U.gen(seed, 0, (M, K), dtype, kind), U.gen(seed, 1, (K, N), dtype, kind)
    C = empty((M, N), dtype)
    lib.distal_gemm(U.dev(A), U.dev(B), C)
    compare(U.host(C), oracle.gemm(A, B), dtype, kind, K, lambda: oracle.gemm(np.abs(A), np.abs(B)))


# every tile shape a dtype has kernels for, reached by name whatever the planner would choose
TILES = {np.float32: [(256, 256), (256, 128), (128, 256), (128, 128), (128, 64), (64, 128), (64, 64), (256, 64), (128, 32),
                      (64, 256), (32, 256)],
         np.float64: [(256, 128), (128, 128), (128, 64), (64, 128), (64, 64), (128, 32), (32, 256)]}
TILE_CASES = [(dt, t) for dt in DT for t in TILES[dt]]
# whole tiles and whole slabs (the straight-line form); ragged in M and N with trailing terms in K
# (edge-clamping form with a second pass); a ragged K made of whole slabs (edge form, one pass)
TILED_EXTENTS = [(512, 768, 128), (520, 712, 100), (300, 264, 96),
                 (256, 256, 256), (200, 136, 300),     # deep enough for the 32-deep slabs of binary32 64 x 64
                 (70, 72, 8)]                          # fewer than 16 terms: the bounds-checked kernel, whatever the tile


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("M,N,K", TILED_EXTENTS)
@pytest.mark.parametrize("dtype,tile", TILE_CASES)
def test_gemm_every_tile_by_name(lib, oracle, dtype, tile, M, N, K, ta):
    """distal_gemm_tiled with each tile, left operand stored either way, C a block inside a larger
    matrix of sentinels; then accumulated on top.  Every element is compared."""
    every_tile_case(lib, oracle, dtype, tile, M, N, K, ta)


# Rows of the right operand that end inside a 16-byte piece, on outputs narrow enough that the library
# keeps them inside the tiled kernels (their forms that fetch the last piece one vector early and
# shift it) instead of peeling the trailing columns off: ragged with whole slabs, with trailing
# terms, a last tile narrower than one piece (129, 257), an output narrower than every tile (7).
ODD_N_EXTENTS = [(302, 131, 96), (520, 71, 100), (260, 7, 48), (200, 129, 300), (136, 257, 64), (1100, 35, 528)]


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("M,N,K", ODD_N_EXTENTS)
@pytest.mark.parametrize("dtype,tile", TILE_CASES)
def test_gemm_every_tile_rows_ending_inside_a_piece(lib, oracle, dtype, tile, M, N, K, ta):
    for acc in (False, True):
        assert lib.gemm_peeled_columns(int(dtype == np.float64), ta, M, N, K, 1, acc) == 0      # what is tested runs in the tiled kernel
    every_tile_case(lib, oracle, dtype, tile, M, N, K, ta)


def every_tile_case(lib, oracle, dtype, tile, M, N, K, ta):
    kind = inputs.SMALLINT if (M + tile[0]) % 3 == 0 else inputs.UNIFORM
    vec = 16 // np.dtype(dtype).itemsize
    A, B = U.gen(700 + M, 0, (M, K), dtype, kind), U.gen(700 + M, 1, (K, N), dtype, kind)
    left = np.ascontiguousarray(A.T) if ta else A
    big = np.full((M + 3, N + 2 * vec), 77.0, dtype=dtype)
    dC = U.dev(big)
    view = dC[2:2 + M, vec:vec + N]
    lib.distal_gemm_tiled(tile, U.dev(left), U.dev(B), view, transposed_left=ta)
    out = U.host(dC)
    got = out[2:2 + M, vec:vec + N]
    mask = np.ones_like(big, dtype=bool)
    mask[2:2 + M, vec:vec + N] = False
    assert np.all(out[mask] == 77.0)
    ref = oracle.gemm(A, B)
    compare(got, ref, dtype, kind, K, lambda: oracle.gemm(np.abs(A), np.abs(B)))
    lib.distal_gemm_tiled(tile, U.dev(left), U.dev(B), view, accumulate=True, transposed_left=ta)
    out2 = U.host(dC)
    if kind == inputs.SMALLINT or dtype == np.float64:
        assert np.array_equal(out2[2:2 + M, vec:vec + N], got * 2)
    else:
        U.assert_close(out2[2:2 + M, vec:vec + N], got.astype(np.float64) * 2, dtype, K)
    assert np.all(out2[mask] == 77.0)


# The library decides how many wavefronts share a tile, for some binary64 tiles from the number
# of tiles in the grid (a tile alone on a compute unit is cut into more wavefronts).  Grids on
# both sides of each switch and the eight-wavefront binary32 tiles, whole and ragged, left
# operand stored either way: tile, M, N, what runs.
WAVEFRONT_SWITCHES = [
    (np.float32, (128, 128), 2048, 2048, "eight wavefronts of 2 x 4 blocks of the 16 x 16 x 4 instruction"),
    (np.float32, (128, 128), 2550, 2430, "the same, ragged"),
    (np.float32, (128, 64), 1024, 1022, "eight wavefronts of 2 x 2 blocks, ragged"),
    (np.float32, (64, 128), 1022, 1024, "eight wavefronts of 2 x 2 blocks, ragged"),
    (np.float32, (64, 64), 1400, 1470, "eight wavefronts of 1 x 2 blocks, ragged"),
    (np.float64, (128, 128), 2048, 2048, "256 tiles: sixteen wavefronts"),
    (np.float64, (128, 128), 2040, 2046, "256 tiles, ragged: sixteen wavefronts"),
    (np.float64, (128, 128), 2048, 2176, "272 tiles: eight wavefronts"),
    (np.float64, (64, 64), 1408, 1472, "506 tiles: eight wavefronts"),
    (np.float64, (64, 64), 1400, 1470, "506 tiles, ragged: eight wavefronts"),
    (np.float64, (64, 64), 1472, 1472, "529 tiles: four wavefronts"),
    (np.float64, (128, 64), 1024, 1022, "eight wavefronts at every grid size, ragged"),
    (np.float64, (64, 128), 1022, 1024, "eight wavefronts at every grid size, ragged"),
]


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("dtype,tile,M,N,what", WAVEFRONT_SWITCHES, ids=[f"{np.dtype(d).name}-{t[0]}x{t[1]}-{m}x{n}" for d, t, m, n, _ in WAVEFRONT_SWITCHES])
def test_gemm_tiled_wavefront_counts(lib, oracle, dtype, tile, M, N, what, ta):
    """Every element against the oracle, with K = 72 (four whole slabs and eight trailing terms),
    then accumulated on top: the result must not depend on how the tile is cut into wavefronts."""
    K = 72
    kind = inputs.SMALLINT
    A, B = U.gen(800 + M, 0, (M, K), dtype, kind), U.gen(800 + M, 1, (K, N), dtype, kind)
    left = np.ascontiguousarray(A.T) if ta else A
    C = empty((M, N), dtype)
    lib.distal_gemm_tiled(tile, U.dev(left), U.dev(B), C, transposed_left=ta)
    got = U.host(C)
    assert np.array_equal(got, oracle.gemm(A, B)), what                  # small integers: exact
    lib.distal_gemm_tiled(tile, U.dev(left), U.dev(B), C, accumulate=True, transposed_left=ta)
    assert np.array_equal(U.host(C), got * 2), what


# small outputs with a long contracted index: cut along k into (parts, the last one shorter or not)
SPLITK_SHAPES = [(512, 512, 8192), (100, 100, 3000), (300, 200, 5000), (300, 200, 5001), (64, 72, 70000), (130, 31, 4099)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M,N,K", SPLITK_SHAPES)
def test_gemm_ws_cut_along_k(lib, oracle, dtype, kind, M, N, K):
    """distal_gemm_ws on products it cuts along k: every element against the oracle; operands are
    views one column off alignment inside larger matrices, C a block between sentinels; then
    accumulated on top (the parts are summed first and added to the old C once)."""
    code = int(dtype == np.float64)
    need = lib.gemm_workspace_bytes(code, M, N, K)
    assert need > 0 and need % (M * N * np.dtype(dtype).itemsize) == 0
    import torch
    A, B = U.gen(900 + M, 0, (M, K), dtype, kind), U.gen(900 + M, 1, (K, N), dtype, kind)
    bigA, bigB = np.zeros((M, K + 5), dtype=dtype), np.zeros((K, N + 3), dtype=dtype)
    bigA[:, 1:1 + K], bigB[:, 1:1 + N] = A, B
    bigC = np.full((M + 2, N + 4), 77.0, dtype=dtype)
    dA, dB, dC = U.dev(bigA), U.dev(bigB), U.dev(bigC)
    view = dC[1:1 + M, 2:2 + N]
    ws = torch.full((need + 256,), 0xAB, dtype=torch.uint8, device="cuda:0")      # whatever it held before
    lib.distal_gemm_ws(dA[:, 1:1 + K], dB[:, 1:1 + N], view, workspace=ws[:need])
    out = U.host(dC)
    got = out[1:1 + M, 2:2 + N]
    ref = oracle.gemm(A, B)
    compare(got, ref, dtype, kind, K, lambda: oracle.gemm(np.abs(A), np.abs(B)))
    mask = np.ones_like(bigC, dtype=bool)
    mask[1:1 + M, 2:2 + N] = False
    assert np.all(out[mask] == 77.0)
    assert bool((ws[need:] == 0xAB).all())                                          # nothing past the stated size
    lib.distal_gemm_ws(dA[:, 1:1 + K], dB[:, 1:1 + N], view, accumulate=True)        # the binding's own scratch
    out2 = U.host(dC)
    if kind == inputs.SMALLINT or dtype == np.float64:
        assert np.array_equal(out2[1:1 + M, 2:2 + N], got * 2)
    else:
        U.assert_close(out2[1:1 + M, 2:2 + N], got.astype(np.float64) * 2, dtype, K)
    assert np.all(out2[mask] == 77.0)


def test_gemm_ws_uncut_is_gemm(lib):
    """Extents that are not cut: the same bits as distal_gemm, no workspace touched."""
    import torch
    A, B = U.dev(U.gen(31, 0, (700, 900), np.float32)), U.dev(U.gen(31, 1, (900, 500), np.float32))
    assert lib.gemm_workspace_bytes(0, 700, 500, 900) == 0
    C1, C2 = empty((700, 500), np.float32), empty((700, 500), np.float32)
    lib.distal_gemm(A, B, C1)
    lib.distal_gemm_ws(A, B, C2)
    assert torch.equal(C1, C2)


def test_gemm_tiled_rejects_unknown_tiles(lib):
    import torch
    A = torch.zeros(64, 64, dtype=torch.float64, device="cuda:0")
    C = torch.zeros(64, 64, dtype=torch.float64, device="cuda:0")
    for tile in ((256, 256), (256, 64), (48, 48), (0, 0)):      # binary32-only shapes and no shape at all
        with pytest.raises(lib.DistalError) as e:
            lib.distal_gemm_tiled(tile, A, A.clone(), C)
        assert e.value.status == 2


# every large tile at a size that gives each compute unit a tile or more, named by the caller
# (binary32: 256 x 256 with 32-deep slabs, 256 x 128, 128 x 256; binary64: 256 x 128 with sixteen
# wavefronts, 128 x 128 with eight), and one shape left to the planner per dtype
BIG_TILE_SHAPES = [(np.float32, 4096, 4096, 1024, (256, 256)), (np.float32, 4096, 4096, 512, (256, 128)),
                   (np.float32, 4096, 4096, 512, (128, 256)), (np.float32, 4096, 4096, 1024, None),
                   (np.float64, 4096, 4096, 4096, (256, 128)), (np.float64, 4096, 2048, 64, (128, 128)),
                   (np.float64, 4096, 2048, 64, None)]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype,M,N,K,tile", BIG_TILE_SHAPES)
def test_gemm_big_tile_configs(lib, oracle, kind, dtype, M, N, K, tile):
    """The oracle recomputes sampled rows of the product (all columns) from the same inputs."""
    run = (lambda a, b, c, **kw: lib.distal_gemm(a, b, c, **kw)) if tile is None else \
          (lambda a, b, c, **kw: lib.distal_gemm_tiled(tile, a, b, c, **kw))
    A, B = U.gen(200 + K, 0, (M, K), dtype, kind), U.gen(200 + K, 1, (K, N), dtype, kind)
    C = empty((M, N), dtype)
    run(U.dev(A), U.dev(B), C)
    got = U.host(C)
    assert np.all(np.isfinite(got))
    rows = np.sort(np.random.default_rng(K).choice(M, 24, replace=False))
    rows[0], rows[-1] = 0, M - 1
    compare(got[rows], oracle.gemm(np.ascontiguousarray(A[rows]), B), dtype, kind, K)
    # accumulate on top of the product: twice it (exactly, unless binary32 terms are added to the
    # old values one by one)
    run(U.dev(A), U.dev(B), C, accumulate=True)
    if kind == inputs.SMALLINT or dtype == np.float64:
        assert np.array_equal(U.host(C), got * 2)
    else:
        U.assert_close(U.host(C), got.astype(np.float64) * 2, dtype, K)


# ragged shapes that reach the same launch configurations in their edge-clamping form (M and N
# not whole tiles, K with trailing terms for the second pass).  split None: the tile is named by
# the caller; otherwise the planner runs the product and must choose this tile and this cut.
RAGGED_TILE_SHAPES = [(np.float32, 4000, 4000, 1028, (256, 256, 32), None), (np.float32, 4000, 4090, 520, (256, 128, 16), None),
                      (np.float32, 4000, 4090, 520, (128, 256, 16), 0), (np.float32, 3900, 4072, 1056, (128, 256, 16), 0),
                      (np.float64, 4000, 4090, 4100, (256, 128, 16), None), (np.float64, 4000, 2040, 72, (128, 128, 16), 0),
                      (np.float32, 3000, 2040, 100, (64, 128, 32), 0), (np.float32, 3900, 4072, 1056, (256, 256, 32), None),
                      # two launches: whole rounds of large tiles, the rest on small tiles - cut along the
                      # rows (binary32 128 x 256; binary64 128 x 128) and along the columns (binary64 128 x 128)
                      (np.float32, 4200, 4096, 1024, (128, 256, 16), 1), (np.float64, 8200, 8192, 272, (128, 128, 16), 1),
                      (np.float64, 8192, 8200, 272, (128, 128, 16), 2)]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype,M,N,K,tile,split", RAGGED_TILE_SHAPES)
def test_gemm_ragged_edge_tiles(lib, oracle, kind, dtype, M, N, K, tile, split):
    """C is a block inside a larger matrix filled with a sentinel: rows past M and columns past N
    of the edge tiles must not be stored.  The oracle recomputes sampled rows (first, last, some
    of the last tile row) over all columns."""
    vec = 16 // np.dtype(dtype).itemsize
    if split is None:
        run = lambda a, b, c, **kw: lib.distal_gemm_tiled(tile[:2], a, b, c, **kw)
    else:
        assert lib.gemm_plan(int(dtype == np.float64), False, M, N, K)[:2] == (tile, split)
        run = lambda a, b, c, **kw: lib.distal_gemm(a, b, c, **kw)
    A, B = U.gen(300 + K, 0, (M, K), dtype, kind), U.gen(300 + K, 1, (K, N), dtype, kind)
    big = np.full((M + 3, N + 2 * vec), 77.0, dtype=dtype)
    dC = U.dev(big)
    view = dC[2:2 + M, vec:vec + N]
    run(U.dev(A), U.dev(B), view)
    out = U.host(dC)
    got = out[2:2 + M, vec:vec + N]
    assert np.all(np.isfinite(got))
    mask = np.ones_like(big, dtype=bool)
    mask[2:2 + M, vec:vec + N] = False
    assert np.all(out[mask] == 77.0)
    rows = np.sort(np.random.default_rng(K).choice(M, 24, replace=False))
    rows[0], rows[-1], rows[-2], rows[-3] = 0, M - 1, M - 2, M - 70
    rows = np.unique(np.concatenate([rows, [min(M - 1, 4095), min(M - 1, 4096), min(M - 1, 2047), min(M - 1, 2048)]]))
    compare(got[rows], oracle.gemm(np.ascontiguousarray(A[rows]), B), dtype, kind, K)
    # accumulate on top of the product: twice it (exactly so in binary64, where the product is formed
    # first and then added; binary32 adds the terms to the old values one by one), and still nothing
    # outside
    run(U.dev(A), U.dev(B), view, accumulate=True)
    out2 = U.host(dC)
    if kind == inputs.SMALLINT or dtype == np.float64:
        assert np.array_equal(out2[2:2 + M, vec:vec + N], got * 2)
    else:
        U.assert_close(out2[2:2 + M, vec:vec + N], got.astype(np.float64) * 2, dtype, K)
    assert np.all(out2[mask] == 77.0)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("off", [0, 1, 2, 3])
def test_gemm_strided_views_accumulate(lib, oracle, dtype, kind, off):
    """Operands are sub-blocks of larger matrices (k-chunks of a tile), some misaligned."""
    M, N, K = 150, 141, 70
    big_a, big_b, big_c = (U.gen(7, 0, (M + 5, K + 9), dtype, kind), U.gen(7, 1, (K + 4, N + 7), dtype, kind),
                           U.gen(7, 2, (M + 3, N + 6), dtype, kind))
    dA, dB, dC = U.dev(big_a), U.dev(big_b), U.dev(big_c)
    vA, vB, vC = dA[2:2 + M, off:off + K], dB[1:1 + K, off:off + N], dC[3:3 + M, off:off + N]
    ref = oracle.gemm(big_a[2:2 + M, off:off + K], big_b[1:1 + K, off:off + N],
                      init=big_c[3:3 + M, off:off + N])
    lib.distal_gemm(vA, vB, vC, accumulate=True)
    out = U.host(dC)
    compare(out[3:3 + M, off:off + N], ref, dtype, kind, K + 1)
    # nothing outside the output block was written
    mask = np.ones_like(big_c, dtype=bool)
    mask[3:3 + M, off:off + N] = False
    assert np.array_equal(out[mask], big_c[mask])


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("accumulate", [False, True])
@pytest.mark.parametrize("M,N,K,offs", [(300, 259, 96, (1, 3, 2)), (257, 513, 528, (0, 1, 3)), (520, 130, 1040, (3, 0, 1)),
                                        (129, 3, 64, (1, 1, 1)), (64, 1027, 48, (2, 2, 0))])
def test_gemm_each_operand_misaligned_differently_and_odd_n(lib, oracle, dtype, kind, accumulate, M, N, K, offs):
    """Views whose bases sit at different element offsets from a 16-byte boundary, with row
    strides that are not multiples of the vector and N not a multiple of it: the straight-line
    kernels take all of it but the last N % vector columns, which a streaming kernel computes.
    Nothing outside the output block may be written."""
    oa, ob, oc = offs
    big_a, big_b = U.gen(17, 0, (M + 2, K + oa + 5), dtype, kind), U.gen(17, 1, (K + 1, N + ob + 3), dtype, kind)
    big_c = U.gen(17, 2, (M + 2, N + oc + 6), dtype, kind)
    dA, dB, dC = U.dev(big_a), U.dev(big_b), U.dev(big_c)
    sa, sb, sc = (slice(1, 1 + M), slice(oa, oa + K)), (slice(1, 1 + K), slice(ob, ob + N)), (slice(2, 2 + M), slice(oc, oc + N))
    ref = oracle.gemm(big_a[sa], big_b[sb], init=big_c[sc] if accumulate else None)
    lib.distal_gemm(dA[sa], dB[sb], dC[sc], accumulate=accumulate)
    out = U.host(dC)
    compare(out[sc], ref, dtype, kind, K + 1)
    mask = np.ones_like(big_c, dtype=bool)
    mask[sc] = False
    assert np.array_equal(out[mask], big_c[mask])


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M,N,K", [(300, 200, 101), (520, 264, 1029), (64, 64, 17)])
def test_gemm_k_not_a_multiple_of_the_vector(lib, oracle, dtype, kind, M, N, K):
    """A is the leading K columns of a wider, aligned matrix: its 16-byte pieces would straddle the
    end of K, so the trailing terms are a second pass that accumulates into C; with accumulate."""
    wide = U.gen(9, 0, (M, K + 7 - (K + 7) % 4 + 4), dtype, kind)
    B, C0 = U.gen(9, 1, (K, N), dtype, kind), U.gen(9, 2, (M, N), dtype, kind)
    dC = U.dev(C0)
    lib.distal_gemm(U.dev(wide)[:, :K], U.dev(B), dC, accumulate=True)
    compare(U.host(dC), oracle.gemm(np.ascontiguousarray(wide[:, :K]), B, init=C0), dtype, kind, K + 1)


@pytest.mark.parametrize("dtype", DT)
def test_gemm_identity_returns_input(lib, dtype):
    A = U.gen(8, 0, (200, 136), dtype)
    C = empty((200, 136), dtype)
    lib.distal_gemm(U.dev(A), U.dev(np.eye(136, dtype=dtype)), C)
    assert np.array_equal(U.host(C), A)
    C2 = empty((200, 136), dtype)
    lib.distal_gemm(U.dev(np.eye(200, dtype=dtype)), U.dev(A), C2)
    assert np.array_equal(U.host(C2), A)


@pytest.mark.parametrize("dtype", DT)
def test_gemm_schedules_bit_exact(lib, oracle, dtype):
    """SUMMA k-chunks with accumulate, Cannon's rotated chunk order and Johnson's
    independent partial products all reproduce the one-shot product (paper:
    matrix-multiplication case studies)."""
    import torch
    n, g = 384, 3
    t = n // g
    A, B = U.gen(9, 0, (n, n), dtype, inputs.SMALLINT), U.gen(9, 1, (n, n), dtype, inputs.SMALLINT)
    ref = oracle.gemm(A, B)
    dA, dB = U.dev(A), U.dev(B)
    # SUMMA: chunkSize 48, A += B_l x C_l
    C = torch.zeros((n, n), dtype=dA.dtype, device="cuda:0")
    for kc in range(0, n, 48):
        lib.distal_gemm(dA[:, kc:kc + 48], dB[kc:kc + 48, :], C, accumulate=True)
    U.assert_exact(U.host(C), ref)
    # Cannon on a 3x3 grid: tile (io,jo) takes k-tile (ko+io+jo) mod 3 at step ko
    C = torch.zeros((n, n), dtype=dA.dtype, device="cuda:0")
    for io in range(g):
        for jo in range(g):
            for ko in range(g):
                kos = (ko + io + jo) % g
                lib.distal_gemm(dA[io * t:(io + 1) * t, kos * t:(kos + 1) * t],
                                dB[kos * t:(kos + 1) * t, jo * t:(jo + 1) * t],
                                C[io * t:(io + 1) * t, jo * t:(jo + 1) * t], accumulate=True)
    U.assert_exact(U.host(C), ref)
    # Johnson: independent partial products, then a sum over k
    parts = []
    for k in range(g):
        P = empty((n, n), dtype)
        lib.distal_gemm(dA[:, k * t:(k + 1) * t], dB[k * t:(k + 1) * t, :], P)
        parts.append(U.host(P).astype(np.float64))
    U.assert_exact(sum(parts), ref)


# ------------------------------------------------------------------ ttm

TTM_SHAPES = [(3, 5, 7, 4), (16, 16, 64, 32), (9, 33, 129, 130), (2, 70, 256, 256), (1, 1, 1, 1), (5, 3, 40, 1)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("I,J,K,L", TTM_SHAPES)
def test_ttm(lib, oracle, dtype, kind, I, J, K, L):
    B, C = U.gen(3, 0, (I, J, K), dtype, kind), U.gen(3, 1, (K, L), dtype, kind)
    A = empty((I, J, L), dtype)
    lib.distal_ttm(U.dev(B), U.dev(C), A)
    compare(U.host(A), oracle.ttm(B, C), dtype, kind, K, lambda: oracle.ttm(np.abs(B), np.abs(C)))


@pytest.mark.parametrize("dtype", DT)
def test_ttm_equals_gemm_on_view_and_identity(lib, dtype):
    I, J, K, L = 6, 50, 96, 72
    B, C = U.gen(30, 0, (I, J, K), dtype), U.gen(30, 1, (K, L), dtype)
    dB, dC = U.dev(B), U.dev(C)
    A, G = empty((I, J, L), dtype), empty((I * J, L), dtype)
    lib.distal_ttm(dB, dC, A)
    lib.distal_gemm(dB.view(I * J, K), dC, G)
    assert np.array_equal(U.host(A).reshape(I * J, L), U.host(G))
    A2 = empty((I, J, K), dtype)
    lib.distal_ttm(dB, U.dev(np.eye(K, dtype=dtype)), A2)
    assert np.array_equal(U.host(A2), B)


# ------------------------------------------------------------------ ttv

TTV_SHAPES = [(4, 8, 1024), (3, 7, 1000), (5, 5, 7), (2, 9, 1), (1, 1, 64), (6, 11, 520), (2, 3, 8200),
              (33, 17, 128), (2, 2, 16388),
              (6, 11, 521), (2, 3, 8201), (40, 50, 1001), (9, 9, 67), (300, 7, 131),   # odd K: element-aligned 16-byte loads and a tail
              (40, 500, 64), (3, 1000, 32), (7, 77, 8),      # short rows: several rows per lane group
              (2, 3, 1 << 17), (1, 5, 70000),               # few long rows: one workgroup per row
              # >= 8192 rows of whole 4 KiB runs: whole rows per wavefront, a row range per workgroup
              # (one and several steps per row, ranges with a ragged end, both register sets last)
              (83, 101, 1024), (91, 97, 2048), (64, 129, 3072), (70, 120, 1536), (128, 65, 512), (8192, 1, 4096),
              (90, 93, 2560),   # binary32: rows of five 2 KiB runs (four rows per wavefront, five steps per row)
              (8200, 1, 8192), (4100, 2, 16384),   # 32 / 64 KiB rows: two rows per wavefront, many steps per row
              (1030, 1, 16384), (3, 400, 32768)]   # 1024 to 8191 long rows: one row per wavefront, four per workgroup


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("I,J,K", TTV_SHAPES)
def test_ttv(lib, oracle, dtype, kind, I, J, K):
    B, c = U.gen(2, 0, (I, J, K), dtype, kind), U.gen(2, 1, (K,), dtype, kind)
    A = empty((I, J), dtype)
    lib.distal_ttv(U.dev(B), U.dev(c), A)
    compare(U.host(A), oracle.ttv(B, c), dtype, kind, K, lambda: oracle.ttv(np.abs(B), np.abs(c)))


@pytest.mark.parametrize("dtype", DT)
def test_ttv_closed_forms(lib, dtype):
    I, J, K = 7, 13, 256
    B = U.gen(21, 0, (I, J, K), dtype, inputs.SMALLINT)
    A = empty((I, J), dtype)
    lib.distal_ttv(U.dev(B), U.dev(np.ones(K, dtype=dtype)), A)
    assert np.array_equal(U.host(A).astype(np.int64), B.astype(np.int64).sum(axis=2))
    Bu = U.gen(21, 0, (I, J, K), dtype)
    for m in (0, 77, 255):
        e = np.zeros(K, dtype=dtype)
        e[m] = 1
        lib.distal_ttv(U.dev(Bu), U.dev(e), A)
        assert np.array_equal(U.host(A), Bu[:, :, m])


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("I,J,K,ob,oc", [(3, 5, 64, 1, 1), (7, 9, 1001, 1, 3), (2, 3, 8200, 3, 0), (5, 4, 40, 1, 2), (64, 70, 256, 0, 1)])
def test_ttv_misaligned_operands(lib, oracle, dtype, I, J, K, ob, oc):
    """The tensor and the vector start ob and oc elements past a 16-byte boundary."""
    flat = U.gen(22, 0, (I * J * K + ob,), dtype)
    cc = U.gen(22, 1, (K + oc,), dtype)
    dB = U.dev(flat)[ob:].view(I, J, K)
    dc = U.dev(cc)[oc:]
    A = empty((I, J), dtype)
    lib.distal_ttv(dB, dc, A)
    U.assert_close(U.host(A), oracle.ttv(flat[ob:].reshape(I, J, K), cc[oc:]), dtype, K)


# ------------------------------------------------------------------ innerprod

IP_SHAPES = [(1, 1, 1), (1, 1, 3), (2, 3, 5), (4, 8, 1024), (3, 1 << 10, 1027), (7, 333, 1 << 10), (1, 1, (3 << 20) + 12345)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("I,J,K", IP_SHAPES)
def test_innerprod(lib, oracle, dtype, kind, I, J, K):
    B, C = U.gen(2, 0, (I, J, K), dtype, kind), U.gen(2, 2, (I, J, K), dtype, kind)
    a = empty((1,), dtype)
    lib.distal_innerprod(U.dev(B), U.dev(C), a)
    ref = oracle.innerprod(B, C)
    got = float(U.host(a)[0])
    if kind == inputs.SMALLINT:
        assert got == ref
    else:
        # binary64 accumulation on both sides: only the final rounding to dtype differs
        scale = float(np.sum(np.abs(B.astype(np.float64) * C.astype(np.float64))))
        eps = np.finfo(dtype).eps
        assert abs(got - ref) <= eps * abs(ref) + 1e-15 * scale, (got, ref)
        assert abs(got - ref) <= U.tol(dtype, I * J * K) * abs(ref) or abs(ref) < 1e-3 * scale


@pytest.mark.parametrize("dtype", DT)
def test_innerprod_closed_forms(lib, dtype):
    n = 200003
    B, C = U.gen(23, 0, (1, 1, n), dtype), U.gen(23, 2, (1, 1, n), dtype)
    dB, dC = U.dev(B), U.dev(C)
    a, b = empty((1,), dtype), empty((1,), dtype)
    lib.distal_innerprod(dB, dC, a)
    lib.distal_innerprod(dC, dB, b)
    assert U.host(a)[0] == U.host(b)[0]                       # symmetric, bit for bit
    lib.distal_innerprod(dB, dB, a)
    sq = float(np.sum(B.astype(np.float64) ** 2))
    assert U.host(a)[0] > 0 and abs(float(U.host(a)[0]) - sq) <= 2 * np.finfo(dtype).eps * sq
    Bi = U.gen(23, 0, (1, 1, n), dtype, inputs.SMALLINT)
    lib.distal_innerprod(U.dev(Bi), U.dev(np.ones_like(Bi)), a)
    assert float(U.host(a)[0]) == float(Bi.astype(np.int64).sum())


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("n,ob,oc", [(70001, 1, 1), (70001, 1, 2), (3, 1, 0), (1 << 21, 3, 1), (262147, 0, 1)])
def test_innerprod_misaligned(lib, oracle, dtype, n, ob, oc):
    """The operands start ob and oc elements past a 16-byte boundary; small integers: exact."""
    fb, fc = U.gen(24, 0, (n + ob,), dtype, inputs.SMALLINT), U.gen(24, 2, (n + oc,), dtype, inputs.SMALLINT)
    a = empty((1,), dtype)
    lib.distal_innerprod(U.dev(fb)[ob:].view(1, 1, n), U.dev(fc)[oc:].view(1, 1, n), a)
    assert float(U.host(a)[0]) == oracle.innerprod(fb[ob:].reshape(1, 1, n), fc[oc:].reshape(1, 1, n))
    lib.distal_innerprod_noalloc(U.dev(fb)[ob:].view(1, 1, n), U.dev(fc)[oc:].view(1, 1, n), a)
    assert float(U.host(a)[0]) == oracle.innerprod(fb[ob:].reshape(1, 1, n), fc[oc:].reshape(1, 1, n))


# ------------------------------------------------------------------ mttkrp

MTTKRP_SHAPES = [(1, 1, 1, 1), (3, 4, 5, 2), (4, 64, 64, 32), (5, 300, 40, 32), (3, 130, 129, 5),
                 (2, 257, 33, 40), (6, 32, 1024, 32), (2, 600, 16, 33)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("I,J,K,L", MTTKRP_SHAPES)
def test_mttkrp(lib, oracle, dtype, kind, I, J, K, L):
    r = 2 if kind == inputs.SMALLINT else 3     # keeps every partial sum exactly representable
    B = U.gen(4, 0, (I, J, K), dtype, kind, r)
    C, D = U.gen(4, 1, (J, L), dtype, kind, r), U.gen(4, 2, (K, L), dtype, kind, r)
    A = empty((I, L), dtype)
    lib.distal_mttkrp(U.dev(B), U.dev(C), U.dev(D), A)
    compare(U.host(A), oracle.mttkrp(B, C, D), dtype, kind, J * K,
            lambda: oracle.mttkrp(np.abs(B), np.abs(C), np.abs(D)))


@pytest.mark.parametrize("dtype", DT)
def test_mttkrp_rank1_and_selection(lib, dtype):
    I, J, K = 5, 70, 48
    B = U.gen(25, 0, (I, J, K), dtype, inputs.SMALLINT)
    A = empty((I, 1), dtype)
    lib.distal_mttkrp(U.dev(B), U.dev(np.ones((J, 1), dtype)), U.dev(np.ones((K, 1), dtype)), A)
    assert np.array_equal(U.host(A)[:, 0].astype(np.int64), B.astype(np.int64).sum(axis=(1, 2)))
    Bu = U.gen(25, 0, (I, J, K), dtype)
    ps, qs = [3, 0, 69], [1, 47, 20]
    C, D = np.zeros((J, 3), dtype), np.zeros((K, 3), dtype)
    for l, (p, q) in enumerate(zip(ps, qs)):
        C[p, l] = 1
        D[q, l] = 1
    A = empty((I, 3), dtype)
    lib.distal_mttkrp(U.dev(Bu), U.dev(C), U.dev(D), A)
    for l, (p, q) in enumerate(zip(ps, qs)):
        assert np.array_equal(U.host(A)[:, l], Bu[:, p, q])


# ------------------------------------------------------------------ degenerate extents, determinism

@pytest.mark.parametrize("dtype", DT)
def test_zero_extents(lib, dtype):
    import torch
    td = getattr(torch, np.dtype(dtype).name)
    z = lambda *s: torch.zeros(s, dtype=td, device="cuda:0")
    C = empty((3, 4), dtype)
    lib.distal_gemm(z(3, 0), z(0, 4), C)
    assert np.array_equal(U.host(C), np.zeros((3, 4)))
    keep = U.gen(26, 2, (3, 4), dtype)
    C = U.dev(keep)
    lib.distal_gemm(z(3, 0), z(0, 4), C, accumulate=True)
    assert np.array_equal(U.host(C), keep)
    lib.distal_gemm(z(0, 5), z(5, 4), z(0, 4))
    A = empty((2, 3), dtype)
    lib.distal_ttv(z(2, 3, 0), z(0), A)
    assert np.array_equal(U.host(A), np.zeros((2, 3)))
    a = empty((1,), dtype)
    lib.distal_innerprod(z(2, 0, 3), z(2, 0, 3), a)
    assert float(U.host(a)[0]) == 0.0
    A = empty((2, 3, 4), dtype)
    lib.distal_ttm(z(2, 3, 0), z(0, 4), A)
    assert np.array_equal(U.host(A), np.zeros((2, 3, 4)))
    A = empty((2, 4), dtype)
    lib.distal_mttkrp(z(2, 0, 3), z(0, 4), z(3, 4), A)
    assert np.array_equal(U.host(A), np.zeros((2, 4)))
    A = empty((2, 4), dtype)
    lib.distal_mttkrp(z(2, 3, 0), z(3, 4), z(0, 4), A)
    assert np.array_equal(U.host(A), np.zeros((2, 4)))


@pytest.mark.parametrize("dtype", DT)
def test_bitwise_reproducible(lib, dtype):
    B = U.dev(U.gen(27, 0, (8, 96, 200), dtype))
    C, D = U.dev(U.gen(27, 1, (96, 32), dtype)), U.dev(U.gen(27, 2, (200, 32), dtype))
    c = U.dev(U.gen(27, 1, (200,), dtype))
    outs = []
    for _ in range(2):
        A1, A2, A3, a = empty((8, 32), dtype), empty((8, 96), dtype), empty((8, 96, 32), dtype), empty((1,), dtype)
        lib.distal_mttkrp(B, C, D, A1)
        lib.distal_ttv(B, c, A2)
        lib.distal_ttm(B, D, A3)
        lib.distal_innerprod(B, B, a)
        outs.append([U.host(x).tobytes() for x in (A1, A2, A3, a)])
    assert outs[0] == outs[1]


def test_runs_on_a_side_stream(lib, oracle):
    import torch
    A, B = U.gen(28, 0, (200, 64), np.float32), U.gen(28, 1, (64, 136), np.float32)
    dA, dB = U.dev(A), U.dev(B)
    C = empty((200, 136), np.float32)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        lib.distal_gemm(dA, dB, C)
    s.synchronize()
    U.assert_close(U.host(C), oracle.gemm(A, B), np.float32, 64)


# ------------------------------------------------------------------ schedule driver

@pytest.mark.parametrize("dtype", DT)
def test_schedule_driver(lib, oracle, dtype):
    """The call sequences of schedules.py (SUMMA, Cannon, Johnson, PUMMA, Solomonik's 2.5D, COSMA)
    give the one-shot product, bit for bit on integer inputs."""
    import torch
    from paper_2203_08069_amd import schedules
    n = 768
    A, B = U.gen(50, 0, (n, n), dtype, inputs.SMALLINT), U.gen(50, 1, (n, n), dtype, inputs.SMALLINT)
    ref = oracle.gemm(A, B)
    dA, dB = U.dev(A), U.dev(B)
    z = lambda: torch.zeros((n, n), dtype=dA.dtype, device="cuda:0")
    U.assert_exact(U.host(schedules.summa(dA, dB, z(), 2, 3, 128)), ref)
    U.assert_exact(U.host(schedules.summa(dA, dB, z(), 1, 1, 100)), ref)       # ragged last chunk
    U.assert_exact(U.host(schedules.cannon(dA, dB, z(), 3)), ref)
    parts = schedules.johnson(dA, dB, z(), 2, [empty((n, n), dtype) for _ in range(2)])
    U.assert_exact(sum(U.host(p).astype(np.float64) for p in parts), ref)
    U.assert_exact(U.host(schedules.pumma(dA, dB, z(), 3, 2)), ref)
    parts = schedules.solomonik(dA, dB, z(), 4, 2, [z() for _ in range(2)])          # 4 x 4 x 2, two steps per layer
    U.assert_exact(sum(U.host(p).astype(np.float64) for p in parts), ref)
    parts = schedules.cosma(dA, dB, z(), 2, 4, 3, 2, [z() for _ in range(3)])        # 2 x 4 x 3 grid, two sequential steps
    U.assert_exact(sum(U.host(p).astype(np.float64) for p in parts), ref)


# ------------------------------------------------------------------ graph capture

def test_calls_can_be_captured_in_a_graph(lib, oracle):
    """Nothing in the library allocates, synchronises or records a memset, so a caller may capture
    a launch-bound sequence (here the k-steps of a SUMMA schedule plus one call of every other
    entry point) in a HIP graph.  Every replay is compared with the eager result, bit for bit,
    with eager work and synchronisations between the replays."""
    import torch
    from paper_2203_08069_amd import schedules
    dt = np.float32
    n = 384
    A, Bm = U.dev(U.gen(60, 0, (n, n), dt)), U.dev(U.gen(60, 1, (n, n), dt))
    T = U.dev(U.gen(61, 0, (12, 64, 128), dt))
    Cf, Df, cv = U.dev(U.gen(61, 1, (64, 32), dt)), U.dev(U.gen(61, 2, (128, 32), dt)), U.dev(U.gen(61, 1, (128,), dt))
    Cg = torch.zeros((n, n), dtype=torch.float32, device="cuda:0")
    o_ttv, o_ttm = empty((12, 64), dt), empty((12, 64, 32), dt)
    o_mk, o_mk2, o_ip = empty((12, 32), dt), empty((128, 32), dt), empty((1,), dt)
    Ci = U.dev(U.gen(61, 3, (12, 32), dt))

    def work():
        Cg.zero_()                                        # a fill kernel, not a memset node
        schedules.summa(A, Bm, Cg, 1, 1, 64)              # six accumulate k-steps
        lib.distal_ttv(T, cv, o_ttv)
        lib.distal_ttm(T, Df, o_ttm)
        lib.distal_mttkrp(T, Cf, Df, o_mk)
        lib.distal_mttkrp_mode(2, T, Ci, Cf, o_mk2)
        lib.distal_innerprod(T, T, o_ip)

    outs = (Cg, o_ttv, o_ttm, o_mk, o_mk2, o_ip)
    work()                                                # eager: also sizes the cached workspaces
    torch.cuda.synchronize()
    eager = [U.host(o).copy() for o in outs]
    U.assert_close(eager[0], oracle.gemm(U.host(A), U.host(Bm)), dt, n)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for replay in range(3):
        for o in outs:
            o.fill_(float("nan"))                         # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert np.array_equal(U.host(o), e), f"replay {replay} differs from the eager result"
