"""Definition of the sparse product, in fp64.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The TW/TVW GEMM is exactly a dense GEMM with the pruned weight: pruning zeroes
elements of B (Algorithm 3 "Prune ..."), and the kernel of Section V only skips
the partial sums of pruned elements, so

    C = A . (B (.) mask),      A: M x K,  B: K x N,  mask in {0,1}^(K x N).

Inputs are the fp16 values the GPU sees, widened exactly to fp64; finite inputs
are assumed (0 * inf would be NaN here, while a kernel that skips the term
gives 0).
"""
from __future__ import annotations

import math

import numpy as np


def masked_weight(B16: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """B (.) mask in fp64.  mask is 0/1, same shape as B."""
    if B16.shape != mask.shape:
        raise ValueError("B and mask must have the same shape")
    return B16.astype(np.float64) * (mask != 0).astype(np.float64)


def gemm_oracle(A16: np.ndarray, B16: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """C_ref = A . (B (.) mask), fp64, M x N (Section III-A: C = A x B)."""
    return A16.astype(np.float64) @ masked_weight(B16, mask)


def abs_bound(A16: np.ndarray, B16: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """S = |A| . |B (.) mask| : the scale of the per-element error bound."""
    return np.abs(A16.astype(np.float64)) @ np.abs(masked_weight(B16, mask))


def gemm_bruteforce(A16: np.ndarray, B16: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Per-element dot products with exactly rounded sums (math.fsum), only
    over the kept elements.  Slow; for tiny inputs.  Independent of
    gemm_oracle: no matmul, no multiplication by the mask."""
    M, K = A16.shape
    K2, N = B16.shape
    assert K == K2
    a = [[float(A16[i, k]) for k in range(K)] for i in range(M)]
    b = [[float(B16[k, n]) for n in range(N)] for k in range(K)]
    C = np.zeros((M, N), dtype=np.float64)
    for n in range(N):
        kept = [k for k in range(K) if mask[k, n]]
        for i in range(M):
            C[i, n] = math.fsum(a[i][k] * b[k][n] for k in kept)
    return C


# ---------------------------------------------------------------------------
# 8-bit integer variant.  The paper treats quantisation as orthogonal to its
# sparsity (Section II-B; Section VI-B "Int8 Quantization" runs the tensor cores
# in Int8): the product is the same definition over integers, and it is exact.
# ---------------------------------------------------------------------------
def gemm_i8_oracle(A8: np.ndarray, B8: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """C = A . (B (.) mask) for int8 A (M x K) and B (K x N), exact, int64."""
    if A8.dtype != np.int8 or B8.dtype != np.int8 or B8.shape != mask.shape:
        raise ValueError("int8 A and B, mask of B's shape")
    return A8.astype(np.int64) @ (B8.astype(np.int64) * (mask != 0))


def gemm_i8_bruteforce(A8: np.ndarray, B8: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """The same with Python integers, element by element, over the kept elements only."""
    M, K = A8.shape
    N = B8.shape[1]
    a, b = A8.tolist(), B8.tolist()
    C = np.zeros((M, N), dtype=np.int64)
    for n in range(N):
        kept = [k for k in range(K) if mask[k, n]]
        for i in range(M):
            C[i, n] = sum(a[i][k] * b[k][n] for k in kept)
    return C


def requantize_i8(acc: np.ndarray, scale: float) -> np.ndarray:
    """int32 sums -> int8: the sum converted to fp32 (round to nearest even), times the fp32
    scale (one fp32 rounding), rounded to the nearest integer (halves to even), clamped to
    [-128, 127].  Every step has one IEEE-defined result, so this is bit-exact to follow."""
    x = acc.astype(np.int32).astype(np.float32) * np.float32(scale)
    return np.clip(np.rint(x), -128, 127).astype(np.int8)
