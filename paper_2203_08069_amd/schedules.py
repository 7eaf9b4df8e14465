"""The paper's matrix-multiplication schedules, run on ONE GPU as sequences of leaf calls.

A distributed schedule in the paper (matrix-multiplication case studies and the algorithm
table: Cannon, PUMMA, SUMMA, Johnson, Solomonik's 2.5D, COSMA) makes every processor issue one
leaf update per k-step on the tiles or chunks it
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


def pumma(A, B, C, gx: int, gy: int):
    """PUMMA on a gx x gy grid (the paper's algorithm table): k is divided into gx tiles and
    the k-loop of processor (io, jo) is rotated by io only - one operand is broadcast, the
    other moves systolically - so at step ko it multiplies the k-tile (ko + io) mod gx."""
    M, N, K = _check(A, B, C)
    if M % gx or N % gy or K % gx:
        raise ValueError("grid must divide the matrix and gx must divide K")
    tm, tn, tk = M // gx, N // gy, K // gx
    for io in range(gx):
        for jo in range(gy):
            ct = C[io * tm:(io + 1) * tm, jo * tn:(jo + 1) * tn]
            for ko in range(gx):
                kos = (ko + io) % gx
                binding.distal_gemm(A[io * tm:(io + 1) * tm, kos * tk:(kos + 1) * tk],
                                    B[kos * tk:(kos + 1) * tk, jo * tn:(jo + 1) * tn], ct, accumulate=True)
    return C


def solomonik(A, B, C, g: int, c: int, partials):
    """Solomonik's 2.5D algorithm on a g x g x c grid (g = sqrt(p / c)): k is distributed over
    the c layers; inside a layer the k-range is divided into `steps` = max(1, g // c) chunks that
    processor (io, jo) visits in the rotated order (kio + io + jo) mod steps, as in Cannon's
    algorithm.  Layer ko accumulates into ``partials[ko]`` (zero-initialised M x N buffers);
    the reduction over the layers is the caller's."""
    M, N, K = _check(A, B, C)
    steps = max(1, g // c)
    if M % g or N % g or K % (c * steps) or len(partials) != c:
        raise ValueError("grid must divide the matrix, c * steps must divide K, one partial buffer per layer")
    tm, tn, tk = M // g, N // g, K // (c * steps)
    for ko in range(c):
        for io in range(g):
            for jo in range(g):
                pt = partials[ko][io * tm:(io + 1) * tm, jo * tn:(jo + 1) * tn]
                for kio in range(steps):
                    kios = (kio + io + jo) % steps
                    k0 = (ko * steps + kios) * tk
                    binding.distal_gemm(A[io * tm:(io + 1) * tm, k0:k0 + tk],
                                        B[k0:k0 + tk, jo * tn:(jo + 1) * tn], pt, accumulate=True)
    return partials


def cosma(A, B, C, gx: int, gy: int, gz: int, num_steps: int, partials):
    """The distribution layer of COSMA as the paper states it: a gx x gy x gz grid chosen by
    COSMA's scheduler, k distributed over gz, and each processor's k-range walked in
    `num_steps` sequential chunks.  Layer ko accumulates into ``partials[ko]``
    (zero-initialised); the reduction over ko is the caller's."""
    M, N, K = _check(A, B, C)
    if M % gx or N % gy or K % (gz * num_steps) or len(partials) != gz:
        raise ValueError("grid must divide the matrix, gz * num_steps must divide K, one partial buffer per layer")
    tm, tn, tk = M // gx, N // gy, K // (gz * num_steps)
    for ko in range(gz):
        for io in range(gx):
            for jo in range(gy):
                pt = partials[ko][io * tm:(io + 1) * tm, jo * tn:(jo + 1) * tn]
                for kio in range(num_steps):
                    k0 = (ko * num_steps + kio) * tk
                    binding.distal_gemm(A[io * tm:(io + 1) * tm, k0:k0 + tk],
                                        B[k0:k0 + tk, jo * tn:(jo + 1) * tn], pt, accumulate=True)
    return partials
