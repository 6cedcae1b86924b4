"""Convolution as the GEMM the paper runs (Section VI-A: the convolutional layers are
converted to GEMM by img2col; the weight matrix has one column per output channel and the
filter elements of one input channel next to each other in a column), in fp64.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Row m of the img2col matrix A is the flattened input window of output position m, so
C = A . (B (.) mask) with k = (c * R + r) * S + s.  The input is stored "wide": per channel
one contiguous run of B image blocks of L lines of P elements, padding included, whatever
the caller put there:

    X[c][b*L*P + yy*P + xx],   c < C,  b < B,  yy < L,  xx < P,   L >= H+R-1,  P >= W+S-1.

Output position m = b*L*P + y*P + x is VALID iff y < H and x < W; its window is
X[c][m + r*P + s] (r < R, s < S): the same shift for every position, which is what lets a
kernel read the window rows straight out of X instead of a materialised A.  Invalid
positions (the padding lanes of the wide grid) are 0 by definition here.
"""
from __future__ import annotations

import math

import numpy as np

from . import gemm as _gemm


def valid_positions(*, B: int, H: int, W: int, P: int, L: int) -> np.ndarray:
    m = np.arange(B * L * P)
    return ((m // P) % L < H) & (m % P < W)


def im2col_wide(X: np.ndarray, *, R: int, S: int, B: int, H: int, W: int, P: int, L: int,
                rows=None) -> np.ndarray:
    """The img2col matrix over the wide grid: (B*L*P) x (C*R*S), rows of invalid positions 0.
    `rows` (positions m of the wide grid) asks for those rows of the matrix only, in that order:
    the same definition, for checks at sizes where the whole matrix is too large to multiply."""
    C, ldx = X.shape
    if L < H + R - 1 or P < W + S - 1 or ldx < B * L * P:
        raise ValueError("image block too small for the filter, or X too short")
    valid = valid_positions(B=B, H=H, W=W, P=P, L=L)
    pos = np.arange(B * L * P) if rows is None else np.asarray(rows, dtype=np.int64)
    sel = np.flatnonzero(valid[pos])           # rows of the result that are output pixels
    mv = pos[sel]
    A = np.zeros((pos.size, C * R * S), X.dtype)
    for c in range(C):
        for r in range(R):
            for s in range(S):
                A[sel, (c * R + r) * S + s] = X[c, mv + r * P + s]
    return A


def conv_wide_oracle(X16, B16, mask, **geom) -> np.ndarray:
    """C_ref over the wide grid, (B*L*P) x N, fp64: the GEMM definition on the img2col matrix."""
    return _gemm.gemm_oracle(im2col_wide(X16, **geom), B16, mask)


def conv_wide_abs_bound(X16, B16, mask, **geom) -> np.ndarray:
    return _gemm.abs_bound(im2col_wide(X16, **geom), B16, mask)


def conv_bruteforce(X16, B16, mask, *, R, S, B, H, W, P, L) -> np.ndarray:
    """Seven plain loops with exactly rounded sums over the kept weight elements; no img2col
    matrix, no matmul.  Tiny inputs only."""
    C = X16.shape[0]
    N = B16.shape[1]
    out = np.zeros((B * L * P, N), np.float64)
    x = X16.astype(np.float64)
    w = B16.astype(np.float64)
    for b in range(B):
        for y in range(H):
            for xx in range(W):
                m = b * L * P + y * P + xx
                for n in range(N):
                    out[m, n] = math.fsum(
                        x[c, b * L * P + (y + r) * P + (xx + s)] * w[(c * R + r) * S + s, n]
                        for c in range(C) for r in range(R) for s in range(S)
                        if mask[(c * R + r) * S + s, n])
    return out
