"""The library's calls under HIP graph capture: a whole SUMMA schedule of accumulating tile steps
on views, and the higher-order calls with caller-held workspaces, are captured once and replayed
several times with eager work between the replays; every replay must reproduce the eager result
bit for bit (the same kernels run in the same order).  The calls allocate nothing, clear memory
with a fill kernel and synchronise nothing, which is what makes them capturable; the one-time
per-kernel set-up of a call's first launch is done by the eager run that precedes the capture."""
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


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_captured_summa_schedule_replays_exactly(lib, oracle, dtype):
    import torch
    from paper_2203_08069_amd import schedules
    n, g, chunk = 512, 2, 64
    hA, hB = U.gen(71, 0, (n, n), dtype, inputs.SMALLINT), U.gen(71, 1, (n, n), dtype, inputs.SMALLINT)
    A, B = U.dev(hA), U.dev(hB)
    C = torch.zeros((n, n), dtype=A.dtype, device="cuda:0")
    schedules.summa(A, B, C, g, g, chunk)                   # eager: also the first launch of every kernel
    torch.cuda.synchronize()
    want = C.clone()
    assert np.array_equal(U.host(want), oracle.gemm(hA, hB))        # small integers: exact
    graph = torch.cuda.CUDAGraph()
    C.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        C.zero_()                                           # a fill kernel, not a memset node
        schedules.summa(A, B, C, g, g, chunk)
    for rep in range(4):
        C.fill_(float(rep + 7))                             # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, want), f"replay {rep}"


def test_captured_tensor_calls_replay_exactly(lib, oracle):
    import torch
    I, J, K, L = 40, 96, 256, 32
    dt = np.float32
    hB, hc = U.gen(72, 0, (I, J, K), dt), U.gen(72, 1, (K,), dt)
    hC, hD, hM = U.gen(72, 2, (J, L), dt), U.gen(72, 3, (K, L), dt), U.gen(72, 4, (K, L), dt)
    B, c, C, D, M = (U.dev(x) for x in (hB, hc, hC, hD, hM))
    out_ttv = torch.empty((I, J), dtype=torch.float32, device="cuda:0")
    out_ttm = torch.empty((I, J, L), dtype=torch.float32, device="cuda:0")
    out_mk = torch.empty((I, L), dtype=torch.float32, device="cuda:0")
    out_ip = torch.empty(1, dtype=torch.float32, device="cuda:0")
    ws = torch.empty(max(lib.mttkrp_workspace_bytes(0, I, J, K, L), 256), dtype=torch.uint8, device="cuda:0")

    def run():
        lib.distal_ttv(B, c, out_ttv)
        lib.distal_ttm(B, M, out_ttm)
        lib.distal_mttkrp(B, C, D, out_mk, workspace=ws)
        lib.distal_innerprod_noalloc(B, B, out_ip)

    run()
    torch.cuda.synchronize()
    want = [t.clone() for t in (out_ttv, out_ttm, out_mk, out_ip)]
    U.assert_close(U.host(want[0]), oracle.ttv(hB, hc), dt, K)
    U.assert_close(U.host(want[2]), oracle.mttkrp(hB, hC, hD), dt, J * K)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        for t in (out_ttv, out_ttm, out_mk, out_ip):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((out_ttv, out_ttm, out_mk, out_ip), want):
            assert torch.equal(got, ref), f"replay {rep}"


def test_captured_rank_sized_ttm_replays_exactly(lib):
    """The TTM kernel that keeps a rank-sized factor in registers (a long tensor, at most 32 columns) under
    capture: replays with eager work between give the eager call's bits."""
    import torch
    I, J, K, L = 256, 256, 512, 32
    assert lib.ttm_slices_per_wave(0, I * J, K, L) == 1
    gen = torch.Generator(device="cuda:0").manual_seed(73)
    B = torch.rand((I, J, K), dtype=torch.float32, device="cuda:0", generator=gen) - 0.5
    M = torch.rand((K, L), dtype=torch.float32, device="cuda:0", generator=gen) - 0.5
    out = torch.empty((I, J, L), dtype=torch.float32, device="cuda:0")
    lib.distal_ttm(B, M, out)
    torch.cuda.synchronize()
    want = out.clone()
    ref = B.view(I * J, K)[:4096].double() @ M.double()
    assert float((want.view(I * J, L)[:4096].double() - ref).abs().max()) < 1e-4
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lib.distal_ttm(B, M, out)
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep}"
