"""The paper's matrix-multiplication schedules, run on ONE GPU as sequences of leaf calls.

A distributed schedule in the paper (matrix-multiplication case studies: SUMMA, Cannon,
Johnson) makes every processor issue one leaf update per k-step on the tiles or chunks it
holds at that step.  With a single GPU there is nothing to communicate: the functions below
walk the processor grid in a loop and issue exactly the leaf calls each processor would, on
views of the full matrices, so that (a) the call sequences are exercised end to end and
(b) the leaf can be timed at the tile shapes a g x g grid produces.  All arithmetic happens
inside ``distal_gemm``; this module only slices.
"""
from __future__ import annotations

from . import binding


def _check(A, B, C):
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not match C(M,N) = A(M,K) B(K,N)")
    return M, N, K


def summa(A, B, C, gx: int, gy: int, chunk: int):
    """SUMMA on a gx x gy grid: every processor steps k in chunks of `chunk` and adds
    A(its rows, chunk) x B(chunk, its columns) to its tile of C.  C must hold the initial
    value (zeros for a plain product)."""
    M, N, K = _check(A, B, C)
    if M % gx or N % gy or chunk <= 0:
        raise ValueError("grid must divide the matrix and chunk must be positive")
    tm, tn = M // gx, N // gy
    for io in range(gx):
        for jo in range(gy):
            ct = C[io * tm:(io + 1) * tm, jo * tn:(jo + 1) * tn]
            for kc in range(0, K, chunk):
                binding.distal_gemm(A[io * tm:(io + 1) * tm, kc:kc + chunk],
                                    B[kc:kc + chunk, jo * tn:(jo + 1) * tn], ct, accumulate=True)
    return C


def cannon(A, B, C, g: int):
    """Cannon's algorithm on a g x g grid: at step ko processor (io, jo) multiplies the
    k-tile kos = (ko + io + jo) mod g (the rotated iteration of the paper's schedule)."""
    M, N, K = _check(A, B, C)
    if M % g or N % g or K % g:
        raise ValueError("grid must divide all three extents")
    tm, tn, tk = M // g, N // g, K // g
    for io in range(g):
        for jo in range(g):
            ct = C[io * tm:(io + 1) * tm, jo * tn:(jo + 1) * tn]
            for ko in range(g):
                kos = (ko + io + jo) % g
                binding.distal_gemm(A[io * tm:(io + 1) * tm, kos * tk:(kos + 1) * tk],
                                    B[kos * tk:(kos + 1) * tk, jo * tn:(jo + 1) * tn], ct, accumulate=True)
    return C


def johnson(A, B, C, g: int, partials):
    """Johnson's algorithm on a g x g x g cube: processor (i, j, k) forms the independent
    partial product A(i-tile, k-tile) x B(k-tile, j-tile) into ``partials[k]`` (an M x N
    buffer per k-layer); the layers are then summed into C by g accumulate calls against an
    identity-free path: partial k = 0 is copied, the rest are added by the caller's reduce.
    Returns the list of partial buffers; the reduction over k is the caller's (a collective
    in the distributed setting)."""
    M, N, K = _check(A, B, C)
    if M % g or N % g or K % g or len(partials) != g:
        raise ValueError("grid must divide all three extents and there must be g partial buffers")
    tm, tn, tk = M // g, N // g, K // g
    for k in range(g):
        for i in range(g):
            for j in range(g):
                binding.distal_gemm(A[i * tm:(i + 1) * tm, k * tk:(k + 1) * tk],
                                    B[k * tk:(k + 1) * tk, j * tn:(j + 1) * tn],
                                    partials[k][i * tm:(i + 1) * tm, j * tn:(j + 1) * tn], accumulate=False)
    return partials
