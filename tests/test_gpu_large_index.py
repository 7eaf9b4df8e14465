"""GPU parity on operands of more than 2^32 elements (4100 x 1024 x 1024 binary32, 16 GiB):
element offsets that fit neither a signed nor an unsigned 32-bit integer.

One seeded tensor serves every case, reshaped as the call needs it.  The oracle recomputes
outputs that depend on the start of the tensor, on the elements either side of offset 2^31 and
of offset 2^32, and on its very end, from inputs regenerated on the host by index."""
import numpy as np
import pytest

from paper_2203_08069_amd import inputs

import _util as U

pytestmark = pytest.mark.gpu

I, J, K = 4100, 1024, 1024                    # I*J*K = 2^32 + 2^22
SEED = 9
# i-slices at the start, either side of element offset 2^31, either side of 2^32, and the last
SLICES = (0, 2047, 2048, 4095, 4096, 4099)


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2203_08069_amd import binding
    binding.load_library()
    return binding


def devgen(ordinal, shape, dtype=np.float32, kind=inputs.UNIFORM):
    from paper_2203_08069_amd.device_inputs import generate_on_device
    return generate_on_device(SEED, ordinal, shape, dtype, kind=kind, device="cuda:0")


def host(ordinal, start, count, kind=inputs.UNIFORM):
    return inputs.values(SEED, ordinal, int(start), int(count), np.float32, kind)


@pytest.fixture(scope="module")
def big():
    B = devgen(0, (I, J, K))
    assert B.numel() > 1 << 32
    return B


def test_generated_bytes_past_2_to_32(big):
    """The device-side generator and the host-side one agree on the elements around offset 2^32
    and at the end (everything below relies on regenerating inputs on the host by index)."""
    flat = big.view(-1)
    for start in ((1 << 31) - 512, (1 << 32) - 512, I * J * K - 1024):
        assert np.array_equal(flat[start:start + 1024].cpu().numpy(), host(0, start, 1024))


def test_ttv_past_2_to_32(lib, oracle, big):
    import torch
    c = devgen(1, (K,))
    A = torch.full((I, J), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_ttv(big, c, A)
    assert bool(torch.isfinite(A).all())
    hc = host(1, 0, K)
    for i in SLICES:
        hB = host(0, i * J * K, J * K).reshape(1, J, K)
        U.assert_close(A[i:i + 1].cpu().numpy(), oracle.ttv(hB, hc), np.float32, K)


@pytest.mark.parametrize("mode", [0, 1])
def test_ttv_mode_past_2_to_32(lib, oracle, big, mode):
    """Contraction over i (every output sums elements from both sides of offset 2^32) and over j."""
    import torch
    n = (I, J)[mode]
    c = devgen(2 + mode, (n,))
    hc = host(2 + mode, 0, n)
    if mode == 0:
        A = torch.full((J, K), float("nan"), dtype=torch.float32, device="cuda:0")
        lib.distal_ttv_mode(0, big, c, A)
        assert bool(torch.isfinite(A).all())
        for j in (0, 517, 1023):               # A(j, :) = sum_i c(i) B(i, j, :)
            hB = np.stack([host(0, (i * J + j) * K, K) for i in range(I)]).reshape(I, 1, K)
            U.assert_close(A[j:j + 1].cpu().numpy(), oracle.ttv_mode(0, hB, hc), np.float32, I)
    else:
        A = torch.full((I, K), float("nan"), dtype=torch.float32, device="cuda:0")
        lib.distal_ttv_mode(1, big, c, A)
        assert bool(torch.isfinite(A).all())
        for i in SLICES:                       # A(i, :) = sum_j c(j) B(i, j, :)
            hB = host(0, i * J * K, J * K).reshape(1, J, K)
            U.assert_close(A[i:i + 1].cpu().numpy(), oracle.ttv_mode(1, hB, hc), np.float32, J)


def test_innerprod_past_2_to_32(lib, oracle):
    """Small-integer operands: every partial sum is an integer below 2^53 and the total below 2^24,
    so the one call over 2^32 + 2^22 elements must equal, exactly, the sum of calls over 17 pieces
    (the pieces are what test_gpu_fullsize checks against the oracle at 2^30 elements; the last
    piece, which lies wholly past offset 2^32, is checked against the oracle here)."""
    import torch
    B, C = devgen(4, (I, J, K), kind=inputs.SMALLINT), devgen(5, (I, J, K), kind=inputs.SMALLINT)
    a = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_innerprod(B, C, a)
    total = float(a.item())
    assert abs(total) < 1 << 24 and total == int(total)
    pieces = []
    for lo in range(0, I, 256):
        hi = min(I, lo + 256)
        lib.distal_innerprod(B[lo:hi], C[lo:hi], a)
        pieces.append(float(a.item()))
    assert sum(pieces) == total
    n_last = (I - 4096) * J * K
    hB = host(4, 4096 * J * K, n_last, inputs.SMALLINT).reshape(I - 4096, J, K)
    hC = host(5, 4096 * J * K, n_last, inputs.SMALLINT).reshape(I - 4096, J, K)
    assert pieces[-1] == float(oracle.innerprod(hB, hC))
    # and with the allocation-free entry point
    lib.distal_innerprod_noalloc(B, C, a)
    assert float(a.item()) == total


def test_ttm_past_2_to_32(lib, oracle, big):
    import torch
    L = 64
    C = devgen(6, (K, L))
    A = torch.full((I, J, L), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_ttm(big, C, A)
    assert bool(torch.isfinite(A).all())
    hC = host(6, 0, K * L).reshape(K, L)
    for i in SLICES:                           # 48 fibres of each slice: its first and last rows and some between
        js = np.unique(np.concatenate([[0, 1, J - 2, J - 1], np.random.default_rng(i).integers(0, J, 44)]))
        hB = np.stack([host(0, (i * J + j) * K, K) for j in js]).reshape(1, len(js), K)
        got = A[i][torch.from_numpy(js).cuda()].cpu().numpy().reshape(1, len(js), L)
        U.assert_close(got, oracle.ttm(hB, hC), np.float32, K)


def test_mttkrp_past_2_to_32(lib, oracle, big):
    import torch
    L = 32
    C, D = devgen(7, (J, L)), devgen(8, (K, L))
    A = torch.full((I, L), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_mttkrp(big, C, D, A)
    assert bool(torch.isfinite(A).all())
    hC, hD = host(7, 0, J * L).reshape(J, L), host(8, 0, K * L).reshape(K, L)
    for i in SLICES:
        hB = host(0, i * J * K, J * K).reshape(1, J, K)
        U.assert_close(A[i:i + 1].cpu().numpy(), oracle.mttkrp(hB, hC, hD), np.float32, J * K)


def test_gemm_left_operand_past_2_to_32(lib, oracle, big):
    """The tensor as a 65600 x 65536 left operand (its last 64 rows start past offset 2^32)."""
    import torch
    M, Kd, N = I * J * K // 65536, 65536, 64
    A = big.view(M, Kd)
    Bm = devgen(10, (Kd, N))
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_gemm(A, Bm, C)
    assert bool(torch.isfinite(C).all())
    hB = host(10, 0, Kd * N).reshape(Kd, N)
    rows = np.array([0, 1, 32767, 32768, 65535, 65536, 65537, M - 2, M - 1])
    hA = np.stack([host(0, r * Kd, Kd) for r in rows])
    U.assert_close(C[torch.from_numpy(rows).cuda()].cpu().numpy(), oracle.gemm(hA, hB), np.float32, Kd)


def test_gemm_output_past_2_to_32(lib, oracle):
    """A 65600 x 65536 output (2^32 + 2^22 elements) of a 16-deep product, overwritten and then
    accumulated on: rows from both ends and either side of offsets 2^31 and 2^32, all columns."""
    import torch
    M, N, Kd = 65600, 65536, 16
    A, Bm = devgen(11, (M, Kd)), devgen(12, (Kd, N))
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_gemm(A, Bm, C)
    hA, hB = host(11, 0, M * Kd).reshape(M, Kd), host(12, 0, Kd * N).reshape(Kd, N)
    rows = np.array([0, 32767, 32768, 65535, 65536, M - 1])
    sel = torch.from_numpy(rows).cuda()
    ref = oracle.gemm(np.ascontiguousarray(hA[rows]), hB)
    U.assert_close(C[sel].cpu().numpy(), ref, np.float32, Kd)
    # whole-output property, in pieces: no NaN sentinel is left anywhere
    for lo in range(0, M, 8200):
        assert bool(torch.isfinite(C[lo:lo + 8200]).all())
    lib.distal_gemm(A, Bm, C, accumulate=True)
    U.assert_close(C[sel].cpu().numpy(), 2.0 * ref.astype(np.float64), np.float32, Kd)


@pytest.mark.parametrize("mode", [0, 1])
def test_ttm_mode_past_2_to_32(lib, oracle, big, mode):
    """Tensor times matrix over i (one transposed-left product whose right operand is the whole
    tensor) and over j (a batch of 4100 products)."""
    import torch
    R = 16
    n = (I, J)[mode]
    C = devgen(13 + mode, (n, R))
    hC = host(13 + mode, 0, n * R).reshape(n, R)
    if mode == 0:
        A = torch.full((R, J, K), float("nan"), dtype=torch.float32, device="cuda:0")
        lib.distal_ttm_mode(0, big, C, A)
        assert bool(torch.isfinite(A).all())
        for j in (0, 517, 1023):
            hB = np.stack([host(0, (i * J + j) * K, K) for i in range(I)]).reshape(I, 1, K)
            U.assert_close(A[:, j:j + 1, :].cpu().numpy(), oracle.ttm_mode(0, hB, hC), np.float32, I)
    else:
        A = torch.full((I, R, K), float("nan"), dtype=torch.float32, device="cuda:0")
        lib.distal_ttm_mode(1, big, C, A)
        assert bool(torch.isfinite(A).all())
        for i in SLICES:
            hB = host(0, i * J * K, J * K).reshape(1, J, K)
            U.assert_close(A[i:i + 1].cpu().numpy(), oracle.ttm_mode(1, hB, hC), np.float32, J)


@pytest.mark.parametrize("mode", [1, 2])
def test_mttkrp_mode_past_2_to_32(lib, oracle, big, mode):
    """MTTKRP with i among the summed indices: every output row sums elements from the whole
    tensor.  The slice of B an output row depends on is copied back from the device tensor (whose
    bytes the first test of this file and the generator test of the full-size suite pin)."""
    import torch
    L = 32
    shapes = {1: ((I, L), (K, L), J), 2: ((I, L), (J, L), K)}[mode]
    C, D = devgen(15, shapes[0]), devgen(16, shapes[1])
    A = torch.full((shapes[2], L), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_mttkrp_mode(mode, big, C, D, A)
    assert bool(torch.isfinite(A).all())
    hC = host(15, 0, I * L).reshape(I, L)
    hD = host(16, 0, shapes[1][0] * L).reshape(shapes[1][0], L)
    for x in (0, 517, 1023):
        hB = np.ascontiguousarray((big[:, x:x + 1, :] if mode == 1 else big[:, :, x:x + 1]).cpu().numpy())
        ref = oracle.mttkrp_mode(mode, hB, hC, hD)[0]
        U.assert_close(A[x].cpu().numpy(), ref, np.float32, I * (K if mode == 1 else J))


# (tile, rows of the view, what the case exercises).  The tensor viewed as `rows` rows gives a
# leading dimension of (2^32 + 2^22) / rows elements.
HUGE_LD = [
    ((256, 128), 1024, "rows of a 256-row tile 4.28e9 bytes apart: unsigned 32-bit offsets, just inside their range"),
    ((256, 128), 512, "8.5e9 bytes apart: beyond 32 bits, the pointer-addressed kernel takes over"),
    ((128, 128), 512, "4.27e9 bytes apart within a 128-row tile: inside the range again"),
    ((64, 64), 128, "8.5e9 bytes apart within a 64-row tile: beyond"),
]


@pytest.mark.parametrize("tile,rows,why", HUGE_LD, ids=[f"{t[0]}x{t[1]}-rows{r}" for t, r, _ in HUGE_LD])
def test_gemm_left_operand_rows_gigabytes_apart(lib, oracle, big, tile, rows, why):
    """Left operand: the first 256 columns of the tensor viewed as a few very long rows, so that the
    rows of one tile lie up to and beyond 4 GiB apart (the straight-line kernels address a tile
    with 32-bit byte offsets and must hand over where those do not reach)."""
    import torch
    ld = I * J * K // rows
    Kd, N = 256, 128
    A = big.view(rows, ld)[:, :Kd]
    Bm = devgen(20, (Kd, N))
    C = torch.full((rows, N), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_gemm_tiled(tile, A, Bm, C)
    assert bool(torch.isfinite(C).all())
    hB = host(20, 0, Kd * N).reshape(Kd, N)
    hA = np.stack([host(0, r * ld, Kd) for r in range(rows)])
    U.assert_close(C.cpu().numpy(), oracle.gemm(hA, hB), np.float32, Kd)
    C2 = torch.full((rows, N), float("nan"), dtype=torch.float32, device="cuda:0")
    lib.distal_gemm(A, Bm, C2)                                  # and whatever the plan picks
    U.assert_close(C2.cpu().numpy(), oracle.gemm(hA, hB), np.float32, Kd)


@pytest.mark.parametrize("transposed_left", [False, True])
def test_gemm_slab_rows_gigabytes_apart(lib, oracle, big, transposed_left):
    """The contracted index walks rows 537 MB apart (32 rows of the tensor): for the right operand,
    and for a left operand stored K x M, the 16 rows of one slab then span 8 GB."""
    import torch
    Kd, ld = 32, I * J * K // 32
    wide = big.view(Kd, ld)
    M, N = 256, 192
    if transposed_left:
        A, Bm = wide[:, 4096:4096 + M], devgen(21, (Kd, N))
        hA = np.stack([host(0, k * ld + 4096, M) for k in range(Kd)]).T
        hB = host(21, 0, Kd * N).reshape(Kd, N)
    else:
        A, Bm = devgen(22, (M, Kd)), wide[:, 8192:8192 + N]
        hA = host(22, 0, M * Kd).reshape(M, Kd)
        hB = np.stack([host(0, k * ld + 8192, N) for k in range(Kd)])
    ref = oracle.gemm(np.ascontiguousarray(hA), hB)
    for tile in ((128, 128), (64, 64), (128, 64)):
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        lib.distal_gemm_tiled(tile, A, Bm, C, transposed_left=transposed_left)
        U.assert_close(C.cpu().numpy(), ref, np.float32, Kd)
    if not transposed_left:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        lib.distal_gemm(A, Bm, C)
        U.assert_close(C.cpu().numpy(), ref, np.float32, Kd)
