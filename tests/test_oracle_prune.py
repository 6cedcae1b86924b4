"""Pins for oracle/prune.py and cross-check of the shared input generator."""
import math

import numpy as np
import pytest

from oracle import prune as op
import workloads as wl


def _w(seed, K, N):
    return wl.rng_fp16(seed, (K, N), 1.0)


def test_closed_forms():
    # Algorithm 3: s = 1 - sqrt(1 - s_t);  TVW: s = 1 - 2 (1 - s_t)
    assert op.tw_split_sparsity(0.75) == pytest.approx(0.5)
    assert op.tw_split_sparsity(0.0) == 0.0
    assert (1 - op.tw_split_sparsity(0.9)) ** 2 == pytest.approx(0.1)
    assert op.tvw_tw_sparsity(0.875) == pytest.approx(0.75)
    assert op.tvw_tw_sparsity(0.5) == 0.0          # TVW minimum: plain 2:4
    assert op.n_tiles(768, 128) == 6 and op.n_tiles(692, 128) == 6 and op.n_tiles(129, 128) == 2


def test_tw_paper_hits_target_within_one_unit():
    K, N, G = 64, 96, 16
    w = _w(1, K, N)
    m = op.tw_paper(w, 0.75, G)
    # 50% of columns, then 50% of (tile,row) units
    assert m.any(axis=0).sum() == N // 2
    assert m.sum() == (N // 2) * K // 2
    assert 1 - m.mean() == pytest.approx(0.75)


def test_g1_without_column_step_is_elementwise():
    # Introduction: tile size one makes TW equivalent to EW
    w = _w(2, 12, 10)
    s = 0.6
    m_tw = op.tw(w, 1, s_cols=0.0, s_rows=s)
    m_ew = op.ew(w, s)
    assert np.array_equal(m_tw, m_ew)
    # and EW is "keep the largest magnitudes": a one-liner
    thr = np.sort((w.astype(np.float64) ** 2).ravel())[int(math.floor(s * w.size))]
    assert np.array_equal(m_ew, ((w.astype(np.float64) ** 2) >= thr).astype(np.uint8))


def test_single_tile_is_global_row_and_column_pruning():
    # Introduction: tile size = matrix size gives plain row/column pruning
    K, N = 20, 16
    w = _w(3, K, N)
    m = op.tw(w, N, s_cols=0.25, s_rows=0.5)
    sq = w.astype(np.float64) ** 2
    cols = np.sort(np.argsort(sq.sum(0), kind="stable")[N // 4:])
    rows = np.sort(np.argsort(sq[:, cols].sum(1), kind="stable")[K // 2:])
    want = np.zeros((K, N), np.uint8)
    want[np.ix_(rows, cols)] = 1
    assert np.array_equal(m, want)


def test_tiles_are_cut_on_kept_columns():
    # Section III-A TW-C: after column pruning every tile is G wide again
    K, N, G = 16, 40, 8
    w = _w(4, K, N)
    m = op.tw(w, G, n_cols_pruned=10, rows_kept_per_tile=5)
    cols = np.flatnonzero(m.any(0))
    assert cols.size == 30
    for i in range(0, 30, G):
        tc = cols[i:i + G]
        sub = m[:, tc]
        assert (sub.sum(0) == 5).all()
        assert (sub == sub[:, :1]).all()           # same rows across the tile


def test_plain_2_4_when_tw_part_is_zero():
    # TVW at 50%: TW part 0, every aligned group of 4 along K keeps exactly 2
    K, N = 32, 24
    w = _w(5, K, N)
    m, tm = op.tvw_paper(w, 0.5, 8)
    assert tm.all()
    assert (m.reshape(K // 4, 4, N).sum(1) == 2).all()
    # and they are the two largest magnitudes of each group
    mag = np.abs(w.astype(np.float64)).reshape(K // 4, 4, N)
    kept_min = np.where(m.reshape(K // 4, 4, N) == 1, mag, np.inf).min(1)
    dropped_max = np.where(m.reshape(K // 4, 4, N) == 0, mag, -np.inf).max(1)
    assert (kept_min >= dropped_max).all()


def test_2_4_tie_keeps_lower_position():
    w = np.array([[1, 1, 1, 1]], np.float16).T.repeat(3, axis=1)    # 4 x 3, all equal
    m = op.vw24_condensed(w, np.ones((4, 3), np.uint8), 8)
    assert np.array_equal(m[:, 0], [1, 1, 0, 0])


def test_tvw_groups_follow_condensed_rows():
    K, N, G = 48, 32, 8
    w = _w(6, K, N)
    m, tm = op.tvw_paper(w, 0.875, G)
    assert 1 - tm.mean() == pytest.approx(0.75, abs=0.02)
    cols = np.flatnonzero(tm.any(0))
    for i in range(0, cols.size, G):
        tc = cols[i:i + G]
        rows = np.flatnonzero(tm[:, tc].any(1))
        for g in range(0, rows.size - rows.size % 4, 4):
            assert (m[np.ix_(rows[g:g + 4], tc)].sum(0) == 2).all()
    assert not (m & ~tm).any()


def test_rows_per_tile_rule():
    # BERT-base 768x768, 10% columns pruned, 75% total: rho = .25*768/692
    assert op.rows_per_tile(768, 768, 692, 0.25) == 213
    assert op.rows_per_tile(768, 768, 692, 0.25, 4) == 212
    assert op.rows_per_tile(256, 256, 256, 0.5) == 128
    assert op.rows_per_tile(100, 10, 10, 1.0, 4) == 100


# ---- the shared generator (workloads) against the oracle's own construction ----
@pytest.mark.parametrize("K,N,G,sp,cf", [(64, 80, 16, 0.75, 0.1), (40, 50, 8, 0.5, 0.0), (96, 70, 32, 0.9, 0.2)])
def test_workloads_per_tile_equals_oracle(K, N, G, sp, cf):
    w = _w(10 + K, K, N)
    got = wl.tw_mask(w, G, density=1 - sp, col_frac=cf, recipe="per_tile")
    ncp = int(math.floor(cf * N))
    want = op.tw(w, G, n_cols_pruned=ncp,
                 rows_kept_per_tile=op.rows_per_tile(K, N, N - ncp, 1 - sp))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("K,N,G,sp", [(64, 80, 16, 0.75), (48, 64, 8, 0.5)])
def test_workloads_paper_recipe_equals_oracle(K, N, G, sp):
    w = _w(20 + K, K, N)
    got = wl.tw_mask(w, G, density=1 - sp, col_frac=None, recipe="paper")
    assert np.array_equal(got, op.tw_paper(w, sp, G))


def test_workloads_tvw_equals_oracle():
    K, N, G, sp, cf = 64, 80, 16, 0.875, 0.1
    w = _w(30, K, N)
    m, tm = wl.tvw_mask(w, G, sparsity=sp, col_frac=cf)
    ncp = int(math.floor(cf * N))
    tm_o = op.tw(w, G, n_cols_pruned=ncp,
                 rows_kept_per_tile=op.rows_per_tile(K, N, N - ncp, 2 * (1 - sp), 4))
    assert np.array_equal(tm, tm_o)
    assert np.array_equal(m, op.vw24_condensed(w, tm_o, G))


def test_config1_recipe():
    c = wl.make_case(1)
    assert (c.M, c.K, c.N, c.G) == (128, 256, 256, 64)
    assert c.mask.any(0).all()                                # no column pruning
    for t in range(4):
        sub = c.mask[:, 64 * t:64 * t + 64]
        assert (sub.sum(0) == 128).all() and (sub == sub[:, :1]).all()
    want = op.tw(c.B, 64, n_cols_pruned=0, rows_kept_per_tile=128)
    assert np.array_equal(c.mask, want)


def test_config2_structure():
    c = wl.make_case(2, 0, with_A=False)
    cols = np.flatnonzero(c.mask.any(0))
    assert cols.size == 768 - 76
    assert 1 - c.mask.mean() == pytest.approx(0.75, abs=2e-3)
    kt = [int(c.mask[:, cols[i:i + 128]].any(1).sum()) for i in range(0, cols.size, 128)]
    assert kt == [213] * 6


def test_global_recipe_gives_uneven_tiles():
    c = wl.make_case(2, 0, recipe="global", with_A=False)
    cols = np.flatnonzero(c.mask.any(0))
    kt = [int(c.mask[:, cols[i:i + 128]].any(1).sum()) for i in range(0, cols.size, 128)]
    assert len(set(kt)) > 1
    assert 1 - c.mask.mean() == pytest.approx(0.75, abs=1e-2)


# ---- TEW (Algorithm 3, TEW; Section III-A "TEW") -------------------------------------
def test_tew_with_delta_zero_is_tw():
    w = wl.rng_fp16(3, (24, 20))
    m, tm = op.tew(w, 4, 0.5, 0.0)
    assert np.array_equal(m, tm) and np.array_equal(m, op.tw_paper(w, 0.5, 4))


def test_tew_worked_by_hand():
    """K = N = 4, G = 2, integer weights.  TW at s_t + delta = 0.4375 + 0.3125 = 0.75:
    s = 1 - sqrt(0.25) = 0.5 -> the two columns with the smallest sums of squares go
    (columns 2 and 3: 1+1+1+4 = 7 and 1+1+4+9 = 15 against 101 and 62), one tile of two
    columns is left, and its two weakest rows go (rows 1, 3: 1+4 = 5 and 1+16 = 17 against
    100+16 and 0+25).  delta * 16 = 5 elements come back: the five largest squares among the
    pruned ones, 16 (3,1), 9 (3,3), 4 (1,1), 4 (2,3) and 4 (3,2): all three 4s fit."""
    w = np.array([[10, 4, 1, 1],
                  [1, 2, 1, 1],
                  [0, 5, 1, 2],
                  [1, 4, 2, 3]], np.float16)
    m, tm = op.tew(w, 2, 0.4375, 0.3125)
    want_tm = np.zeros((4, 4), np.uint8)
    want_tm[np.ix_([0, 2], [0, 1])] = 1
    assert np.array_equal(tm, want_tm)
    want = want_tm.copy()
    for k, n in [(3, 1), (3, 3), (1, 1), (2, 3), (3, 2)]:
        want[k, n] = 1
    assert np.array_equal(m, want)


@pytest.mark.parametrize("seed,K,N,G,s_t,delta", [(0, 40, 36, 8, 0.6, 0.05), (1, 33, 50, 16, 0.75, 0.015),
                                                   (2, 16, 16, 4, 0.5, 0.25), (3, 30, 30, 8, 0.9, 0.1)])
def test_tew_invariants(seed, K, N, G, s_t, delta):
    w = wl.rng_fp16(seed, (K, N))
    m, tm = op.tew(w, G, s_t, delta)
    assert np.array_equal(tm, op.tw_paper(w, s_t + delta, G))        # the TW part is TW at s_t + delta
    assert not (tm & ~m).any()                                        # nothing the TW step kept is lost
    n_back = int(m.sum() - tm.sum())
    assert n_back == min(int(math.floor(delta * K * N)), int((tm == 0).sum()))
    sq = w.astype(np.float64) ** 2
    back, gone = (m == 1) & (tm == 0), m == 0
    if back.any() and gone.any():
        assert sq[back].min() >= sq[gone].max()                       # the highest scores came back
    # equal scores at the cut: the lower flat index is restored first
    cut = sq[back].min() if back.any() else None
    if cut is not None:
        tied_gone = np.flatnonzero((gone & (sq == cut)).reshape(-1))
        tied_back = np.flatnonzero((back & (sq == cut)).reshape(-1))
        if tied_gone.size and tied_back.size:
            assert tied_back.max() < tied_gone.min()


def test_tew_tie_at_the_cut_keeps_lower_index():
    w = np.ones((4, 4), np.float16)
    w[0, :] = 3
    m, tm = op.tew(w, 4, 0.5, 0.125, tw_fn=lambda w_, s, G: np.repeat((np.arange(4) == 0)[:, None], 4, 1).astype(np.uint8))
    assert np.array_equal(np.flatnonzero(m.reshape(-1))[:6], [0, 1, 2, 3, 4, 5])   # row 0 + flat 4, 5
    assert m.sum() == 6


@pytest.mark.parametrize("K,N,G,sp,delta,cf", [(64, 96, 32, 0.75, 0.015, 0.1), (40, 70, 16, 0.5, 0.05, 0.0)])
def test_workloads_tew_equals_oracle(K, N, G, sp, delta, cf):
    """The generator's vectorised TEW against the oracle's, same TW step."""
    w = wl.rng_fp16(5, (K, N))
    m, tm = wl.tew_mask(w, G, sparsity=sp, delta=delta, col_frac=cf)
    m2, tm2 = op.tew(w, G, sp, delta,
                     tw_fn=lambda w_, s, G_: wl.tw_mask(w_, G_, density=1.0 - s, col_frac=cf))
    assert np.array_equal(tm, tm2) and np.array_equal(m, m2)


# ---- exact integer scores (used where a GPU pruner has to take the same decisions) ------------
def test_exact_square_scores_are_the_squares():
    vals = np.array([0.0, -0.0, 6e-8, -6.1e-5, 1.0, -1.5, 0.333, 65504.0, -65504.0, 2.0 ** -24, 1023 * 2.0 ** -24],
                    np.float16)
    got = op.exact_square_scores(vals)
    for v, s in zip(vals.tolist(), got):
        assert s == int(round(float(v) * 2 ** 24)) ** 2          # float(v) * 2^24 is an exact integer
        assert s * 2.0 ** -48 == float(v) ** 2 or s >= 2 ** 53    # and agrees with the fp64 square where that is exact


@pytest.mark.parametrize("seed,K,N,G,cp,rk", [(0, 40, 36, 8, 4, 10), (1, 33, 50, 16, 0, 7), (2, 64, 70, 32, 9, 16)])
def test_exact_scores_give_the_float_mask_on_generic_data(seed, K, N, G, cp, rk):
    w = wl.rng_fp16(seed, (K, N))
    assert np.array_equal(op.tw(w, G, n_cols_pruned=cp, rows_kept_per_tile=rk, exact=True),
                          op.tw(w, G, n_cols_pruned=cp, rows_kept_per_tile=rk))


def test_exact_scores_resolve_what_fp64_cannot():
    """Column 0 holds one 64 and many tiny values whose squares fall below half an ulp of 4096 in
    fp64 one by one; column 1 holds 64 alone.  Exactly, column 0 scores higher; a sequential fp64
    sum cannot see it.  With exact scores column 1 is the one pruned."""
    K = 40
    w = np.zeros((K, 2), np.float16)
    w[0, :] = 64.0
    w[1:, 0] = 2.0 ** -24
    s = op.exact_square_scores(w)
    assert sum(s[0::2]) > sum(s[1::2])
    acc = 0.0
    for k in range(K):
        acc += float(w[k, 0]) ** 2
    assert acc == 4096.0                                          # the fp64 running sum lost them
    m = op.tw(w, 1, n_cols_pruned=1, rows_kept_per_tile=K, exact=True)
    assert m[:, 0].all() and not m[:, 1].any()
