"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot redo a 2^30-element contraction in seconds, so each case checks
outputs the oracle CAN compute one by one - sampled rows, fibres, slices or index
ranges, regenerated on the host from the same pure input function - plus a
property that holds for the whole output."""
import numpy as np
import pytest

from paper_2203_08069_amd import inputs

import _util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2203_08069_amd import binding
    binding.load_library()
    return binding


def devgen(seed, ordinal, shape, dtype):
    """The seeded tensor, filled in place on the device by the torch-integer form of the generator
    (test_device_inputs_are_the_generators_bytes pins it to the numpy form on the GPU; every case
    below recomputes its expected values from inputs regenerated on the host by the numpy form)."""
    from paper_2203_08069_amd.device_inputs import generate_on_device
    return generate_on_device(seed, ordinal, shape, dtype, device="cuda:0")


def host_rows(seed, ordinal, row_len, rows, dtype):
    """Rows of a 2-D (or flattened) tensor regenerated on the host: element n = row*row_len + col."""
    return np.stack([inputs.values(seed, ordinal, int(r) * row_len, row_len, dtype) for r in rows])


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_gemm_8192(lib, oracle, dtype):
    """configs[1]: M = N = K = 8192, uniform[-1,1) from seed 1, C zero-initialised."""
    import torch
    n = 8192
    A, B = devgen(1, 0, (n, n), dtype), devgen(1, 1, (n, n), dtype)
    C = torch.zeros((n, n), dtype=A.dtype, device="cuda:0")
    lib.distal_gemm(A, B, C)
    rng = np.random.default_rng(7)
    # one whole row of C inside every band of 128 rows, at a random offset in the band: every row
    # of tiles of every tiling (256 x 128, 256 x 256) and every column tile is covered
    rows = np.arange(0, n, 128) + rng.integers(0, 128, n // 128)
    hA = host_rows(1, 0, n, rows, dtype)                                   # 64 x K
    hB = inputs.tensor(1, 1, (n, n), dtype, threads=8)
    ref = oracle.gemm(hA, hB)                                              # 64 full rows of C
    got = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    U.assert_close(got, ref, dtype, n)
    absref = oracle.gemm(np.abs(hA), np.abs(hB))
    U.assert_componentwise(got, ref, absref, dtype, n)
    # whole output: Freivalds' check C x = A (B x) with x = +-1, evaluated in binary64 on the host
    x = rng.integers(0, 2, n).astype(np.float64) * 2 - 1
    hC = C.cpu().numpy().astype(np.float64)
    bx = hB.astype(np.float64) @ x
    del hB
    hAfull = inputs.tensor(1, 0, (n, n), dtype, threads=8).astype(np.float64)
    want = hAfull @ bx
    gotv = hC @ x
    denom = np.max(np.abs(want))
    assert np.max(np.abs(gotv - want)) / denom <= (1e-11 if dtype == np.float64 else 1e-4)
    # accumulate on top: C += A B doubles every entry - exactly in binary64, where the product is
    # formed first and added to C in the epilogue (power-of-two scaling); in binary32 the terms are
    # added to the old C one by one, so each entry is twice the product to within the tolerance
    lib.distal_gemm(A, B, C, accumulate=True)
    if dtype == np.float64:
        assert np.array_equal(C[:64].cpu().numpy(), (2 * hC[:64]).astype(dtype))
    else:
        U.assert_close(C[:64].cpu().numpy(), 2 * hC[:64], dtype, n)


@pytest.fixture(scope="module")
def cfg3_B():
    return devgen(2, 0, (1024, 1024, 1024), np.float32)


def test_ttv_1024(lib, oracle, cfg3_B):
    """configs[2]: A(i,j) = sum_k B(i,j,k) c(k), B 1024^3 fp32, seed 2."""
    import torch
    I = J = K = 1024
    c = devgen(2, 1, (K,), np.float32)
    A = torch.full((I, J), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_ttv(cfg3_B, c, A)
    assert bool(torch.isfinite(A).all())
    A1 = torch.empty_like(A)
    lib.distal_ttv(cfg3_B, torch.ones(K, dtype=torch.float32, device="cuda:0"), A1)
    hc = inputs.values(2, 1, 0, K, np.float32)
    # every one of the 2^20 outputs, the tensor regenerated on the host 64 slices at a time
    step = 64
    hB = np.empty((step, J, K), np.float32)
    for i0 in range(0, I, step):
        inputs.fill(hB.reshape(-1), 2, 0, i0 * J * K, threads=8)
        U.assert_close(A[i0:i0 + step].cpu().numpy(), oracle.ttv(hB, hc), np.float32, K)
        # all-ones vector: every output is the plain k-sum
        U.assert_close(A1[i0:i0 + step].cpu().numpy(), hB.sum(axis=2, dtype=np.float64), np.float32, K)


def test_innerprod_1024(lib, oracle, cfg3_B):
    """configs[2]: a = sum B .* C over 2^30 elements; binary64 accumulation on both sides."""
    import torch
    n = 1 << 30
    C = devgen(2, 2, (1024, 1024, 1024), np.float32)
    a = torch.empty(1, dtype=torch.float32, device="cuda:0")
    lib.distal_innerprod(cfg3_B, C, a)
    full = float(a.item())
    # the sum splits over contiguous index ranges: GPU pieces add up to the GPU total ...
    pieces, piece_len = [], n // 16
    fb, fc = cfg3_B.view(-1), C.view(-1)
    for p in range(16):
        sl = slice(p * piece_len, (p + 1) * piece_len)
        lib.distal_innerprod(fb[sl].view(1, 1, -1), fc[sl].view(1, 1, -1), a)
        pieces.append(float(a.item()))
    assert abs(sum(pieces) - full) <= 16 * np.finfo(np.float32).eps * sum(abs(p) for p in pieces)
    # ... and every piece is recomputed by the oracle from regenerated inputs
    hb = np.empty((1, 1, piece_len), np.float32)
    hc = np.empty((1, 1, piece_len), np.float32)
    total = 0.0
    for p in range(16):
        inputs.fill(hb.reshape(-1), 2, 0, p * piece_len, threads=8)
        inputs.fill(hc.reshape(-1), 2, 2, p * piece_len, threads=8)
        ref = oracle.innerprod(hb, hc)
        total += ref
        assert abs(pieces[p] - ref) <= 2 * np.finfo(np.float32).eps * abs(ref) + 1e-3
    assert abs(full - total) <= 2 * np.finfo(np.float32).eps * abs(total) + 1e-2
    # symmetry, bit for bit, at full size
    lib.distal_innerprod(C, cfg3_B, a)
    assert float(a.item()) == full


def test_ttm_1024(lib, oracle):
    """configs[3]: A(i,j,l) = sum_k B(i,j,k) C(k,l), B 1024^3, C 1024 x 256, fp32, seed 3."""
    import torch
    I = J = K = 1024
    L = 256
    B, C = devgen(3, 0, (I, J, K), np.float32), devgen(3, 1, (K, L), np.float32)
    A = torch.full((I, J, L), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_ttm(B, C, A)
    rng = np.random.default_rng(9)
    # one whole fibre A(i,j,:) inside every band of 256 rows of the (I*J) x L view: every output tile
    fibres = np.arange(0, I * J, 256) + rng.integers(0, 256, I * J // 256)
    hB = host_rows(3, 0, K, fibres, np.float32).reshape(1, -1, K)
    hC = inputs.tensor(3, 1, (K, L), np.float32)
    ref = oracle.ttm(hB, hC)[0]
    got = A.view(I * J, L)[torch.from_numpy(fibres).cuda()].cpu().numpy()
    U.assert_close(got, ref, np.float32, K)
    assert bool(torch.isfinite(A).all())
    # linear in C: the contraction with 2C is exactly twice the result (the same shape both times:
    # another shape may run on another tile, whose instruction sums the terms in another order)
    A1, A2 = torch.empty_like(A[:8]), torch.empty_like(A[:8])
    lib.distal_ttm(B[:8], C, A1)
    lib.distal_ttm(B[:8], C * 2, A2)
    assert torch.equal(A2, A1 * 2)
    U.assert_close(A1.cpu().numpy(), A[:8].cpu().numpy().astype(np.float64), np.float32, K)


# TTM over the last mode with a rank-sized factor on a long tensor: the kernel that keeps the factor
# in registers (one to four 256-byte slices of it per wavefront).  I, J, K, L and what is reached.
RANK_SIZED_TTM = [
    (np.float32, 256, 256, 512, 32, "one slice per wavefront, whole"),
    (np.float32, 256, 256, 1024, 32, "two slices, whole"),
    (np.float32, 256, 256, 1536, 32, "three slices, whole"),
    (np.float32, 256, 256, 2048, 32, "four slices, whole"),
    (np.float32, 255, 259, 2048, 32, "four slices, the last 29 rows as a tiled product"),
    (np.float32, 257, 256, 1024, 31, "two whole slices, the last 16 rows as a tiled product"),
    (np.float32, 255, 259, 1000, 32, "two slices, a short last slice, a short last block of rows"),
    (np.float32, 256, 257, 960, 17, "two slices, the last wavefront's second slice past K, 17 columns"),
    (np.float32, 300, 300, 452, 1, "one slice, short last slice, one column"),
    (np.float32, 256, 256, 1024, 8, "two slices, 8 columns"),
    (np.float64, 256, 256, 256, 32, "one slice, whole"),
    (np.float64, 256, 256, 512, 32, "two slices, whole"),
    (np.float64, 256, 256, 768, 30, "three slices, 30 columns"),
    (np.float64, 256, 256, 1024, 32, "four slices, whole"),
    (np.float64, 256, 256, 1024, 5, "four slices, 5 columns"),
    (np.float64, 255, 259, 768, 32, "three slices, the last 29 rows as a tiled product"),
    (np.float64, 255, 259, 500, 32, "two slices, ragged"),
    (np.float64, 256, 257, 480, 31, "two slices, the last wavefront's second slice past K"),
    (np.float64, 257, 256, 226, 32, "one slice, short last slice"),
]


@pytest.mark.parametrize("dtype,I,J,K,L,what", RANK_SIZED_TTM,
                         ids=[f"{np.dtype(d).name}-{i}x{j}x{k}-L{l}" for d, i, j, k, l, _ in RANK_SIZED_TTM])
def test_ttm_rank_sized_factor_on_a_long_tensor(lib, oracle, dtype, I, J, K, L, what):
    import torch
    from paper_2203_08069_amd import binding
    assert binding.ttm_slices_per_wave(int(dtype == np.float64), I * J, K, L) in (1, 2, 3, 4)      # the kernel under test runs
    B, C = devgen(31, 0, (I, J, K), dtype), devgen(31, 1, (K, L), dtype)
    tdt = B.dtype
    # sentinels around the output: nothing outside it is written
    flat = torch.full((I * J * L + 64,), 77.0, dtype=tdt, device="cuda:0")
    A = flat[32:32 + I * J * L].view(I, J, L)
    lib.distal_ttm(B, C, A)
    assert bool((flat[:32] == 77.0).all()) and bool((flat[32 + I * J * L:] == 77.0).all())
    assert bool(torch.isfinite(A).all())
    # two fibres of every block of 32 rows of the (I*J) x L view, and the last rows
    rng = np.random.default_rng(32)
    R = I * J
    starts = np.arange(0, R - 31, 32)
    fibres = np.unique(np.concatenate([starts + rng.integers(0, 32, starts.size), starts + rng.integers(0, 32, starts.size),
                                       np.arange(max(R - 40, 0), R)]))
    hB = host_rows(31, 0, K, fibres, dtype).reshape(1, -1, K)
    hC = inputs.tensor(31, 1, (K, L), dtype)
    got = A.view(R, L)[torch.from_numpy(fibres).cuda()].cpu().numpy()
    U.assert_close(got, oracle.ttm(hB, hC)[0], dtype, K)
    # the whole output against the tiled contraction on the same view (another summation order)
    A2 = torch.empty((R, L), dtype=tdt, device="cuda:0")
    lib.distal_gemm(B.view(R, K), C, A2)
    U.assert_close(A.view(R, L).cpu().numpy(), A2.cpu().numpy().astype(np.float64), dtype, K)
    # the same bits on a second call, and exact linearity in the factor
    A3 = torch.empty_like(A)
    lib.distal_ttm(B, C, A3)
    assert torch.equal(A3, A)
    lib.distal_ttm(B, C * 2, A3)
    assert torch.equal(A3, A * 2)


def test_mttkrp_1024(lib, oracle):
    """configs[4]: A(i,l) = sum_jk B(i,j,k) C(j,l) D(k,l), B 1024^3, rank 32, fp32, seed 4."""
    import torch
    I = J = K = 1024
    L = 32
    B = devgen(4, 0, (I, J, K), np.float32)
    C, D = devgen(4, 1, (J, L), np.float32), devgen(4, 2, (K, L), np.float32)
    A = torch.full((I, L), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_mttkrp(B, C, D, A)
    hC, hD = inputs.tensor(4, 1, (J, L), np.float32), inputs.tensor(4, 2, (K, L), np.float32)
    assert bool(torch.isfinite(A).all())
    # every one of the 1024 output rows, the tensor regenerated on the host 64 slices at a time
    step = 64
    hB = np.empty((step, J, K), np.float32)
    got = A.cpu().numpy()
    for i0 in range(0, I, step):
        inputs.fill(hB.reshape(-1), 4, 0, i0 * J * K, threads=8)
        U.assert_close(got[i0:i0 + step], oracle.mttkrp(hB, hC, hD), np.float32, J * K)
    # second call gives the same bits (fixed summation order, no atomics)
    A2 = torch.empty_like(A)
    lib.distal_mttkrp(B, C, D, A2)
    assert torch.equal(A, A2)


def test_device_inputs_are_the_generators_bytes():
    """The device copy that the full-size cases read slices back from is the generator's output."""
    import torch
    from paper_2203_08069_amd.device_inputs import device_tensor
    for dtype in (np.float32, np.float64):
        t = devgen(3, 0, (64, 1024, 1024), dtype)                         # filled in place by torch integer ops
        u = device_tensor(3, 0, (8, 1024, 1024), dtype, device="cuda:0")  # generated by numpy, copied
        assert torch.equal(t[:8], u)
        for start in (0, 12345 * 1024, 64 * 1024 * 1024 - 4096):
            want = inputs.values(3, 0, start, 4096, dtype)
            assert np.array_equal(t.view(-1)[start:start + 4096].cpu().numpy(), want)
    for kind, r in ((inputs.SMALLINT, 3), (inputs.SMALLINT, 2)):
        from paper_2203_08069_amd.device_inputs import generate_on_device
        t = generate_on_device(6, 1, (3, 1000, 1000), np.float32, kind, r, device="cuda:0")
        assert np.array_equal(t.cpu().numpy(), inputs.tensor(6, 1, (3, 1000, 1000), np.float32, kind, r, threads=8))


@pytest.mark.parametrize("mode", [0, 1])
def test_ttm_mode_1024(lib, oracle, mode):
    """TTM along modes 0 and 1 of the configs[3] tensor, in the launch configuration bench.py times
    (256 x 256 tiles, transposed left operand; mode 1 as a batch of 1024 products)."""
    import torch
    I = J = K = 1024
    R = 256
    B, C = devgen(3, 0, (I, J, K), np.float32), devgen(3, 1, (K, R), np.float32)
    shape = [I, J, K]
    shape[mode] = R
    A = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_ttm_mode(mode, B, C, A)
    assert bool(torch.isfinite(A).all())
    hC = inputs.tensor(3, 1, (K, R), np.float32)
    # outputs that depend on one slice of B only, recomputed by the oracle from that slice
    for x in (0, 511, 1023):
        if mode == 0:       # A(:, j, k0:k0+16) <- B(:, j, k0:k0+16)
            k0 = (x * 7) % (K - 16)
            hB = np.ascontiguousarray(B[:, x:x + 1, k0:k0 + 16].cpu().numpy())
            got = A[:, x:x + 1, k0:k0 + 16].cpu().numpy()
        else:               # A(i, :, k0:k0+16) <- B(i, :, k0:k0+16)
            k0 = (x * 5) % (K - 16)
            hB = np.ascontiguousarray(B[x:x + 1, :, k0:k0 + 16].cpu().numpy())
            got = A[x:x + 1, :, k0:k0 + 16].cpu().numpy()
        U.assert_close(got, oracle.ttm_mode(mode, hB, hC), np.float32, 1024)
    # linear in C, exactly, for a power of two
    A2 = torch.empty_like(A)
    lib.distal_ttm_mode(mode, B, C * 2, A2)
    assert torch.equal(A2, A * 2)


@pytest.mark.parametrize("mode", [1, 2])
def test_mttkrp_mode_1024(lib, oracle, mode):
    """MTTKRP along modes 1 and 2 of the configs[4] tensor, rank 32, as bench.py launches it."""
    import torch
    I = J = K = 1024
    L = 32
    B = devgen(4, 0, (I, J, K), np.float32)
    C, D = devgen(4, 1, (J, L), np.float32), devgen(4, 2, (K, L), np.float32)   # I = J = K: they fit every mode
    A = torch.full((1024, L), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_mttkrp_mode(mode, B, C, D, A)
    assert bool(torch.isfinite(A).all())
    hC, hD = inputs.tensor(4, 1, (J, L), np.float32), inputs.tensor(4, 2, (K, L), np.float32)
    # output row x depends on the slice of B with that mode fixed at x
    for x in (0, 357, 1023):
        hB = np.ascontiguousarray((B[:, x:x + 1, :] if mode == 1 else B[:, :, x:x + 1]).cpu().numpy())
        ref = oracle.mttkrp_mode(mode, hB, hC, hD)[0]
        U.assert_close(A[x].cpu().numpy(), ref, np.float32, 1 << 20)
    A2 = torch.empty_like(A)
    lib.distal_mttkrp_mode(mode, B, C, D, A2)
    assert torch.equal(A, A2)


def test_ttv_more_row_groups_than_the_grid_cap(lib, oracle):
    """2^26 + 5 rows of four values: more 16-row groups than the launch caps its grid at, so the
    kernel's grid-stride loop runs; sampled rows and the ragged tail against the oracle."""
    import torch
    rows, K = (1 << 26) + 5, 4
    B = devgen(5, 0, (1, rows, K), np.float32)
    c = devgen(5, 1, (K,), np.float32)
    A = torch.full((1, rows), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_ttv(B, c, A)
    assert bool(torch.isfinite(A).all())
    hc = inputs.values(5, 1, 0, K, np.float32)
    for start in (0, (1 << 22) * 16 - 60, (1 << 25) + 12345, rows - 64):
        hB = inputs.values(5, 0, start * K, 64 * K, np.float32).reshape(1, 64, K)
        U.assert_close(A[0, start:start + 64].cpu().numpy(), oracle.ttv(hB, hc)[0], np.float32, K)


# ---------------------------------------------------------------------------------------------
# binary64 (the paper's own element type) at the full sizes: the instantiations these shapes
# select - the row-streaming TTV kernel, 256 x 128 contraction tiles, the two-row-block MTTKRP
# layout - are reached only here.  Sampled outputs are recomputed by the oracle from inputs
# regenerated on the host; whole-output properties cover the rest.
# ---------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def cfg3_B64():
    return devgen(2, 0, (1024, 1024, 1024), np.float64)


def test_ttv_1024_f64(lib, oracle, cfg3_B64):
    import torch
    I = J = K = 1024
    c = devgen(2, 1, (K,), np.float64)
    A = torch.full((I, J), float("nan"), dtype=torch.float64, device="cuda:0")
    lib.distal_ttv(cfg3_B64, c, A)
    assert bool(torch.isfinite(A).all())
    hc = inputs.values(2, 1, 0, K, np.float64)
    rng = np.random.default_rng(18)
    # four whole i-slices (4096 rows each) spread over the tensor: a row range of every workgroup kind
    for i in (0, int(rng.integers(1, 511)), int(rng.integers(512, 1023)), 1023):
        hB = inputs.values(2, 0, i * J * K, J * K, np.float64).reshape(1, J, K)
        U.assert_close(A[i:i + 1].cpu().numpy(), oracle.ttv(hB, hc), np.float64, K)
    # one sampled row in every run of 256 rows of the (I*J) x K view
    rows = np.arange(0, I * J, 256) + rng.integers(0, 256, I * J // 256)
    hB = host_rows(2, 0, K, rows, np.float64).reshape(1, -1, K)
    got = A.view(-1)[torch.from_numpy(rows).cuda()].cpu().numpy()
    U.assert_close(got, oracle.ttv(hB, hc)[0], np.float64, K)


def test_innerprod_1024_f64(lib, oracle, cfg3_B64):
    import torch
    n = 1 << 30
    C = devgen(2, 2, (1024, 1024, 1024), np.float64)
    a = torch.empty(1, dtype=torch.float64, device="cuda:0")
    lib.distal_innerprod(cfg3_B64, C, a)
    full = float(a.item())
    pieces, piece_len = [], n // 16
    fb, fc = cfg3_B64.view(-1), C.view(-1)
    for p in range(16):
        sl = slice(p * piece_len, (p + 1) * piece_len)
        lib.distal_innerprod(fb[sl].view(1, 1, -1), fc[sl].view(1, 1, -1), a)
        pieces.append(float(a.item()))
    scale = sum(abs(p) for p in pieces)
    assert abs(sum(pieces) - full) <= 1e-12 * scale
    hb = np.empty((1, 1, piece_len), np.float64)
    hc = np.empty((1, 1, piece_len), np.float64)
    for p in (0, 5, 10, 15):
        inputs.fill(hb.reshape(-1), 2, 0, p * piece_len, threads=8)
        inputs.fill(hc.reshape(-1), 2, 2, p * piece_len, threads=8)
        ref = oracle.innerprod(hb, hc)
        # 2^26 terms of magnitude <= 1 summed in binary64 in another order than the oracle's
        assert abs(pieces[p] - ref) <= 1e-12 * max(abs(ref), np.sqrt(piece_len) / 3)
    lib.distal_innerprod(C, cfg3_B64, a)
    assert float(a.item()) == full


def test_ttm_1024_f64(lib, oracle):
    import torch
    I = J = K = 1024
    L = 256
    B, C = devgen(3, 0, (I, J, K), np.float64), devgen(3, 1, (K, L), np.float64)
    A = torch.full((I, J, L), float("nan"), dtype=torch.float64, device="cuda:0")
    lib.distal_ttm(B, C, A)
    assert bool(torch.isfinite(A).all())
    rng = np.random.default_rng(19)
    fibres = np.arange(0, I * J, 256) + rng.integers(0, 256, I * J // 256)     # every band of 256 rows: every tile
    hB = host_rows(3, 0, K, fibres, np.float64).reshape(1, -1, K)
    hC = inputs.tensor(3, 1, (K, L), np.float64)
    got = A.view(I * J, L)[torch.from_numpy(fibres).cuda()].cpu().numpy()
    U.assert_close(got, oracle.ttm(hB, hC)[0], np.float64, K)
    A2 = torch.empty_like(A[:8])
    lib.distal_ttm(B[:8], C * 2, A2)
    assert torch.equal(A2, A[:8] * 2)


def test_mttkrp_1024_f64(lib, oracle):
    import torch
    I = J = K = 1024
    L = 32
    B = devgen(4, 0, (I, J, K), np.float64)
    C, D = devgen(4, 1, (J, L), np.float64), devgen(4, 2, (K, L), np.float64)
    A = torch.full((I, L), float("nan"), dtype=torch.float64, device="cuda:0")
    lib.distal_mttkrp(B, C, D, A)
    assert bool(torch.isfinite(A).all())
    hC, hD = inputs.tensor(4, 1, (J, L), np.float64), inputs.tensor(4, 2, (K, L), np.float64)
    rng = np.random.default_rng(20)
    got = A.cpu().numpy()
    # two rows of every block of 32 output rows (every row block of every workgroup)
    for i in np.sort(np.concatenate([np.arange(0, I, 32) + rng.integers(0, 16, I // 32),
                                     np.arange(0, I, 32) + rng.integers(16, 32, I // 32)])):
        hB = inputs.values(4, 0, int(i) * J * K, J * K, np.float64).reshape(1, J, K)
        U.assert_close(got[i:i + 1], oracle.mttkrp(hB, hC, hD), np.float64, J * K)
    A2 = torch.empty_like(A)
    lib.distal_mttkrp(B, C, D, A2)
    assert torch.equal(A, A2)
