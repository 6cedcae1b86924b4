"""Pins for oracle/gemm.py: the definition C = A . (B (.) mask)."""
import numpy as np
import pytest

from oracle import gemm as og
from tests.helpers import random_tw_mask
import workloads as wl


def _rand16(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


@pytest.mark.parametrize("M,K,N,seed", [(5, 7, 6, 0), (3, 16, 9, 1), (8, 5, 4, 2)])
def test_matches_bruteforce_random_mask(M, K, N, seed):
    rng = np.random.default_rng(seed)
    A, B = _rand16(rng, (M, K)), _rand16(rng, (K, N))
    mask = (rng.random((K, N)) < 0.5).astype(np.uint8)
    ref = og.gemm_bruteforce(A, B, mask)
    got = og.gemm_oracle(A, B, mask)
    # fsum is exactly rounded; a K-term fp64 dot product differs by a few ulp
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13 * max(1.0, np.abs(ref).max()))


def test_matches_bruteforce_on_config1_slice():
    c = wl.make_case(1)
    rows = np.arange(0, c.M, 37)
    cols = np.arange(0, c.N, 29)
    ref = og.gemm_bruteforce(c.A[rows], c.B[:, cols], c.mask[:, cols])
    got = og.gemm_oracle(c.A, c.B, c.mask)[np.ix_(rows, cols)]
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11)


def test_small_integers_are_exact():
    rng = np.random.default_rng(3)
    Ai = rng.integers(-8, 9, (11, 13))
    Bi = rng.integers(-8, 9, (13, 10))
    mask = (rng.random((13, 10)) < 0.6).astype(np.uint8)
    want = Ai @ (Bi * mask)                        # int64, exact
    got = og.gemm_oracle(Ai.astype(np.float16), Bi.astype(np.float16), mask)
    assert np.array_equal(got, want.astype(np.float64))


def test_zero_sparsity_is_dense():
    rng = np.random.default_rng(4)
    A, B = _rand16(rng, (9, 12)), _rand16(rng, (12, 7))
    ones = np.ones((12, 7), np.uint8)
    dense = og.gemm_bruteforce(A, B, ones)
    np.testing.assert_allclose(og.gemm_oracle(A, B, ones), dense, rtol=0, atol=1e-13)


def test_identity_A_returns_masked_B_exactly():
    rng = np.random.default_rng(5)
    K, N = 24, 20
    B = _rand16(rng, (K, N))
    mask = random_tw_mask(rng, K, N, 8)
    C = og.gemm_oracle(np.eye(K, dtype=np.float16), B, mask)
    assert np.array_equal(C, B.astype(np.float64) * mask)


def test_all_ones_counts_kept_elements():
    rng = np.random.default_rng(6)
    K, N = 40, 33
    mask = random_tw_mask(rng, K, N, 8)
    C = og.gemm_oracle(np.ones((3, K), np.float16), np.ones((K, N), np.float16), mask)
    assert np.array_equal(C, np.broadcast_to(mask.sum(axis=0).astype(np.float64), (3, N)))


def test_pruned_columns_are_exactly_zero_and_pruned_rows_do_not_matter():
    rng = np.random.default_rng(7)
    M, K, N, G = 6, 32, 40, 8
    A, B = _rand16(rng, (M, K)), _rand16(rng, (K, N))
    mask = random_tw_mask(rng, K, N, G, col_keep=0.7, row_keep=0.4)
    C = og.gemm_oracle(A, B, mask)
    dead = ~mask.any(axis=0)
    assert dead.any()
    assert not C[:, dead].any()
    assert not og.abs_bound(A, B, mask)[:, dead].any()
    # rows pruned in the first tile: changing those A columns leaves that tile alone
    cols = np.flatnonzero(mask.any(axis=0))[:G]
    pruned_rows = np.flatnonzero(~mask[:, cols].any(axis=1))
    assert pruned_rows.size
    A2 = A.copy()
    A2[:, pruned_rows] = _rand16(rng, (M, pruned_rows.size), 50.0)
    C2 = og.gemm_oracle(A2, B, mask)
    assert np.array_equal(C[:, cols], C2[:, cols])


def test_linearity_over_disjoint_masks():
    # Section III-A (TEW): A.(B1+B2) = A.B1 + A.B2
    rng = np.random.default_rng(8)
    A, B = _rand16(rng, (7, 15)), _rand16(rng, (15, 11))
    m1 = (rng.random((15, 11)) < 0.4).astype(np.uint8)
    m2 = ((rng.random((15, 11)) < 0.5) & (m1 == 0)).astype(np.uint8)
    lhs = og.gemm_oracle(A, B, m1) + og.gemm_oracle(A, B, m2)
    rhs = og.gemm_oracle(A, B, m1 | m2)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-12)


def test_abs_bound_dominates_and_matches_bruteforce():
    rng = np.random.default_rng(9)
    A, B = _rand16(rng, (4, 9)), _rand16(rng, (9, 5))
    mask = (rng.random((9, 5)) < 0.5).astype(np.uint8)
    S = og.abs_bound(A, B, mask)
    Sb = og.gemm_bruteforce(np.abs(A), np.abs(B), mask)
    np.testing.assert_allclose(S, Sb, rtol=0, atol=1e-13)
    assert (np.abs(og.gemm_oracle(A, B, mask)) <= S + 1e-15).all()


def test_planted_mistakes_are_caught():
    """A transposed operand or a dropped mask must fail the brute-force pin."""
    rng = np.random.default_rng(10)
    A, B = _rand16(rng, (6, 6)), _rand16(rng, (6, 6))
    mask = (rng.random((6, 6)) < 0.5).astype(np.uint8)
    ref = og.gemm_bruteforce(A, B, mask)
    wrong_T = A.astype(np.float64) @ (B.astype(np.float64) * mask).T
    wrong_mask_T = A.astype(np.float64) @ (B.astype(np.float64) * mask.T)
    wrong_nomask = A.astype(np.float64) @ B.astype(np.float64)
    for w in (wrong_T, wrong_mask_T, wrong_nomask):
        assert np.abs(w - ref).max() > 1e-3


# ---- int8 variant -------------------------------------------------------------------------------
def test_i8_oracle_equals_bruteforce_and_dense():
    rng = np.random.default_rng(0)
    A = rng.integers(-128, 128, (5, 9), dtype=np.int8)
    B = rng.integers(-128, 128, (9, 7), dtype=np.int8)
    mask = (rng.random((9, 7)) < 0.6).astype(np.uint8)
    C = og.gemm_i8_oracle(A, B, mask)
    assert C.dtype == np.int64 and np.array_equal(C, og.gemm_i8_bruteforce(A, B, mask))
    ones = np.ones_like(mask)
    assert np.array_equal(og.gemm_i8_oracle(A, B, ones), A.astype(np.int64) @ B.astype(np.int64))
    # extreme values do not wrap: (-128) * (-128) * 9
    A[:] = -128; B[:] = -128
    assert (og.gemm_i8_oracle(A, B, ones) == 9 * 16384).all()
    # pruned columns are zero, pruned rows do not matter, disjoint masks add up
    m1 = mask.copy(); m1[:, 2] = 0
    assert not og.gemm_i8_oracle(A, B, m1)[:, 2].any()
    m2 = (1 - mask).astype(np.uint8)
    assert np.array_equal(og.gemm_i8_oracle(A, B, mask) + og.gemm_i8_oracle(A, B, m2), og.gemm_i8_oracle(A, B, ones))


def test_i8_planted_mistakes_fail():
    rng = np.random.default_rng(1)
    A = rng.integers(-128, 128, (6, 6), dtype=np.int8)
    B = rng.integers(-128, 128, (6, 6), dtype=np.int8)
    mask = (rng.random((6, 6)) < 0.5).astype(np.uint8)
    C = og.gemm_i8_oracle(A, B, mask)
    assert not np.array_equal(C, og.gemm_i8_oracle(A.T.copy(), B, mask))
    assert not np.array_equal(C, og.gemm_i8_oracle(A, B, mask.T.copy()))
    assert not np.array_equal(C, A.astype(np.int64) @ B.astype(np.int64))
    assert not np.array_equal(C, (A.view(np.uint8).astype(np.int64)) @ (B.astype(np.int64) * mask))   # sign dropped


def test_requantize_rule():
    acc = np.array([0, 1, 2, 3, -1, -3, 5, 7, 1000, -1000, 2 ** 24 + 1, 254, 255, -256, -257], np.int64)
    q = og.requantize_i8(acc, 0.5)
    #            0  .5->0  1  1.5->2  -.5->-0  -1.5->-2  2.5->2  3.5->4  clamp  clamp  clamp  127  127.5->128->127  -128  -128.5->-128
    assert q.tolist() == [0, 0, 1, 2, 0, -2, 2, 4, 127, -128, 127, 127, 127, -128, -128]
    # int32 -> fp32 is itself rounded (to even): 2^24 + 1 becomes 2^24
    assert og.requantize_i8(np.array([2 ** 24 + 1]), 2.0 ** -18).tolist() == [64]
    assert og.requantize_i8(np.array([3]), np.float32(1 / 3)).tolist() == [1]


def _rne_to_fp32(x):
    """Nearest binary32 value of a positive rational in the normal range, ties to even, in exact
    arithmetic (Fractions): the IEEE 754 definition written out, no floating point used."""
    from fractions import Fraction
    assert x > 0
    e = 0
    while x >= 2:
        x /= 2
        e += 1
    while x < 1:
        x *= 2
        e -= 1
    assert -126 <= e <= 127
    scaled = x * 2 ** 23                   # 24 significant bits: 2^23 <= scaled < 2^24
    n, r = divmod(scaled.numerator, scaled.denominator)
    if 2 * r > scaled.denominator or (2 * r == scaled.denominator and n % 2 == 1):
        n += 1
    return Fraction(n, 2 ** 23) * Fraction(2) ** e


def test_requantize_against_exact_rational_arithmetic():
    """Every step of the rule redone with Fractions on random sums and scales: int -> binary32
    (nearest even), one binary32 product (nearest even), round half to even, clamp."""
    from fractions import Fraction
    rng = np.random.default_rng(17)
    sums = np.concatenate([rng.integers(-2 ** 26, 2 ** 26, 300), rng.integers(-3000, 3000, 300),
                           [2 ** 24 + 1, 2 ** 24 + 3, -(2 ** 25 + 2), 1, -1]]).astype(np.int64)
    scales = np.concatenate([rng.uniform(1e-6, 1e-1, 600), [0.5, 0.25, 1.5, 2.5, 1e-3]]).astype(np.float32)
    got = og.requantize_i8(sums, 1.0)                       # shapes differ: call element by element below
    for s, sc in zip(sums.tolist(), scales.tolist()):
        want = 0
        if s != 0:
            a = _rne_to_fp32(Fraction(abs(s)))               # |sum| as binary32
            p = _rne_to_fp32(a * Fraction(sc))               # the product as binary32 (sc is a binary32 value)
            n, r = divmod(p.numerator, p.denominator)        # round half to even
            if 2 * r > p.denominator or (2 * r == p.denominator and n % 2 == 1):
                n += 1
            want = min(n, 128 if s < 0 else 127) * (-1 if s < 0 else 1)
        assert int(og.requantize_i8(np.array([s]), np.float32(sc))[0]) == want, (s, sc)
    assert got.shape == sums.shape


def test_element_bar_below_the_normal_range_of_fp16():
    """One product below 2^-14: the correctly rounded fp16 value is up to half a subnormal spacing
    (2^-25) from the exact one, more than 4e-3 of it; the bar accepts that value, not the grid
    points beyond its two nearest ones, and still wants exact zeros where nothing is kept."""
    from tests.helpers import assert_C_close
    a, b = np.float16(-0.0004715919494628906), np.float16(-0.0147247314453125)
    A, B = np.array([[a]], np.float16), np.array([[b, b]], np.float16)
    mask = np.array([[1, 0]], np.uint8)
    ref, S = og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask)
    exact = float(a) * float(b)
    stored = float(np.float16(exact))
    assert abs(stored - exact) > 4e-3 * abs(exact) and abs(stored) < 2.0 ** -14
    assert_C_close(np.array([[stored, 0.0]]), ref, S)
    away = np.sign(stored - exact) * 2.0 ** -24            # one spacing further from the exact value
    for wrong in ([[stored + away, 0.0]], [[stored - 2 * away, 0.0]], [[stored, 2.0 ** -24]]):
        with pytest.raises(AssertionError):
            assert_C_close(np.array(wrong), ref, S)
