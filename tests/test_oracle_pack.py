"""Pins for oracle/pack.py: the canonical logical packed form."""
import numpy as np
import pytest

from oracle import pack as opk
from tests.helpers import random_tw_mask, random_tvw_mask
import workloads as wl


def _read_golden(path):
    rows = []
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            rows.append(line.split())
    return rows


def test_worked_example_of_section_v(golden_dir):
    tiles = []
    for tok in _read_golden(f"{golden_dir}/cto_worked_example.txt"):
        i_r, i_o = tok.index("rows"), tok.index("offsets")
        rows = [int(x) for x in tok[i_r + 1:i_o]]
        offs = [int(x) for x in tok[i_o + 1:] if x != "derived"]
        tiles.append((rows, offs))
    G, K = 2, 5
    mask = np.zeros((K, G * len(tiles)), np.uint8)
    for t, (rows, _) in enumerate(tiles):
        mask[rows, t * G:(t + 1) * G] = 1
    B = wl.rng_fp16(0, mask.shape)
    p = opk.ref_pack(B, mask, G, opk.PATTERN_TW)
    assert p["n_tiles"] == len(tiles)
    for t, (rows, offs) in enumerate(tiles):
        assert p["row_idx"][t].tolist() == rows
        assert p["cto_k"][t].tolist() == offs
        # position + offset = index
        assert (np.arange(len(rows)) + p["cto_k"][t]).tolist() == rows


def test_column_regrouping_example_of_section_iii(golden_dir):
    spec = [(int(t[3]), int(t[5])) for t in _read_golden(f"{golden_dir}/twc_regroup_example.txt")]
    G, K = 8, 20
    widths = [G + c for c, _ in spec]
    N = sum(widths)
    mask = np.zeros((K, N), np.uint8)
    n0 = 0
    rng = np.random.default_rng(0)
    for (c, r), wdt in zip(spec, widths):
        cols = np.sort(rng.permutation(wdt)[c:]) + n0       # prune c of this block's columns
        rows = np.sort(rng.permutation(K)[r:])              # prune r rows
        mask[np.ix_(rows, cols)] = 1
        n0 += wdt
    B = wl.rng_fp16(1, mask.shape)
    p = opk.ref_pack(B, mask, G, opk.PATTERN_TW)
    assert p["n_tiles"] == 4 and p["n_kept"] == 4 * G
    assert [v.shape[1] for v in p["values"]] == [G] * 4                       # all G wide
    assert [len(r) for r in p["row_idx"]] == [K - r for _, r in spec]         # K-2, K-4, K-8, K-1


@pytest.mark.parametrize("seed,K,N,G", [(0, 16, 24, 8), (1, 37, 53, 16), (2, 64, 130, 32), (3, 9, 7, 4)])
def test_tw_round_trip(seed, K, N, G):
    rng = np.random.default_rng(seed)
    mask = random_tw_mask(rng, K, N, G)
    B = wl.rng_fp16(seed, (K, N))
    p = opk.ref_pack(B, mask, G, opk.PATTERN_TW)
    Bm, m2 = opk.ref_unpack(p)
    assert np.array_equal(m2, mask)
    assert np.array_equal(Bm, np.where(mask != 0, B.view(np.uint16), 0))
    assert p["col_idx"].tolist() == np.flatnonzero(mask.any(0)).tolist()
    assert (np.arange(p["n_kept"]) + p["cto_n"]).tolist() == p["col_idx"].tolist()
    # condensed values are B[rows][:, cols]
    for t in range(p["n_tiles"]):
        cols = p["col_idx"][t * G:(t + 1) * G]
        assert np.array_equal(p["values"][t], B.view(np.uint16)[np.ix_(p["row_idx"][t], cols)])


@pytest.mark.parametrize("seed,K,N,G,full", [(0, 16, 24, 8, True), (1, 37, 53, 16, True),
                                              (2, 30, 20, 8, False), (3, 9, 7, 4, False)])
def test_tvw_round_trip(seed, K, N, G, full):
    rng = np.random.default_rng(seed)
    mask, tm = random_tvw_mask(rng, K, N, G, full=full)
    B = wl.rng_fp16(seed, (K, N))
    p = opk.ref_pack(B, mask, G, opk.PATTERN_TVW, tile_mask=tm)
    Bm, m2 = opk.ref_unpack(p)
    assert np.array_equal(m2, mask)
    assert np.array_equal(Bm, np.where(mask != 0, B.view(np.uint16), 0))
    for t in range(p["n_tiles"]):
        me = p["meta"][t]
        p0, p1 = me & 3, (me >> 2) & 3
        assert (p0 < p1).all() and (me < 16).all()
        # fill values are +0
        v, va = p["values"][t], p["valid"][t]
        assert not v[:, 0, :][(va & 1) == 0].any()
        assert not v[:, 1, :][(va & 2) == 0].any()


def test_tvw_meta_hand_example():
    # one tile, one group of kept rows (1,2,5,7) of K=8, three columns
    K, G = 8, 4
    tm = np.zeros((K, 3), np.uint8); tm[[1, 2, 5, 7]] = 1
    mask = np.zeros_like(tm)
    mask[[2, 7], 0] = 1          # positions 1,3  -> nibble 1 | 3<<2 = 13, both valid
    mask[[5], 1] = 1             # position 2 only -> fill with 0 -> (0,2) = 0 | 2<<2 = 8, valid = 0b10
    #                              column 2: nothing -> (0,1) = 4, valid 0
    B = (np.arange(K * 3, dtype=np.float16).reshape(K, 3) + 1)
    p = opk.ref_pack(B, mask, G, opk.PATTERN_TVW, tile_mask=tm)
    assert p["row_idx"][0].tolist() == [1, 2, 5, 7]
    assert p["meta"][0].tolist() == [[13, 8, 4]]
    assert p["valid"][0].tolist() == [[3, 2, 0]]
    v = p["values"][0].view(np.float16)
    assert v[0, :, 0].tolist() == [float(B[2, 0]), float(B[7, 0])]
    assert v[0, :, 1].tolist() == [0.0, float(B[5, 1])]
    assert v[0, :, 2].tolist() == [0.0, 0.0]


def test_short_last_group():
    # K_t = 5: second group has one real row (position 0); fill goes to position 1
    tm = np.zeros((6, 2), np.uint8); tm[[0, 1, 2, 3, 5]] = 1
    mask = np.zeros_like(tm); mask[[0, 3, 5]] = 1
    B = wl.rng_fp16(5, (6, 2))
    p = opk.ref_pack(B, mask, 2, opk.PATTERN_TVW, tile_mask=tm)
    assert p["meta"][0].tolist() == [[0 | 3 << 2] * 2, [0 | 1 << 2] * 2]
    assert p["valid"][0].tolist() == [[3, 3], [1, 1]]
    Bm, m2 = opk.ref_unpack(p)
    assert np.array_equal(m2, mask)


def test_non_conformant_masks_are_rejected():
    mask = np.ones((8, 8), np.uint8)
    mask[3, 2] = 0                                          # a hole in a kept row
    B = wl.rng_fp16(0, (8, 8))
    with pytest.raises(opk.MaskError):
        opk.ref_pack(B, mask, 4, opk.PATTERN_TW)
    m3 = np.zeros((8, 4), np.uint8); m3[[0, 1, 2]] = 1      # 3 of 4 in one group
    with pytest.raises(opk.MaskError):
        opk.ref_pack(wl.rng_fp16(0, (8, 4)), m3, 4, opk.PATTERN_TVW)
    tm = np.zeros((8, 4), np.uint8); tm[:4] = 1
    m4 = np.zeros((8, 4), np.uint8); m4[5, 0] = 1           # outside the tile mask
    with pytest.raises(opk.MaskError):
        opk.ref_pack(wl.rng_fp16(0, (8, 4)), m4, 4, opk.PATTERN_TVW, tile_mask=tm)


def test_degenerate_masks():
    B = wl.rng_fp16(0, (6, 10))
    p = opk.ref_pack(B, np.zeros((6, 10), np.uint8), 4, opk.PATTERN_TW)
    assert p["n_kept"] == 0 and p["n_tiles"] == 0
    p = opk.ref_pack(B, np.ones((6, 10), np.uint8), 4, opk.PATTERN_TW)
    assert p["n_tiles"] == 3 and [v.shape for v in p["values"]] == [(6, 4), (6, 4), (6, 2)]
    assert all((c == 0).all() for c in p["cto_k"]) and (p["cto_n"] == 0).all()


def test_configured_masks_are_conformant():
    c = wl.make_case(2, 0, with_A=False)
    p = opk.ref_pack(c.B, c.mask, c.G, opk.PATTERN_TW)
    assert p["n_tiles"] == 6 and [len(r) for r in p["row_idx"]] == [213] * 6
    c = wl.make_case(3, 0, with_A=False)
    p = opk.ref_pack(c.B, c.mask, c.G, opk.PATTERN_TVW, tile_mask=c.tile_mask)
    assert [len(r) for r in p["row_idx"]] == [212] * 6       # 2*(1-.875)*768/692*768 = 213.1 -> multiple of 4
    assert all((v & 3).min() == 3 for v in p["valid"])        # every group full


# ---- TEW: TW form + restored elements in compressed sparse column form -----------------
def _random_tew(rng, K, N, G, extra=0.08):
    tm = random_tw_mask(rng, K, N, G)
    m = tm | ((rng.random((K, N)) < extra) & (tm == 0)).astype(np.uint8)
    return m, tm


def test_tew_hand_example():
    """4 x 5, G = 2: columns 0, 1, 3 kept by the TW step (tile 0 = {0, 1} rows {0, 2};
    tile 1 = {3} rows {1}); restored elements (3,0), (1,1), (0,2), (3,2), (0,3)."""
    tm = np.zeros((4, 5), np.uint8)
    tm[np.ix_([0, 2], [0, 1])] = 1
    tm[1, 3] = 1
    m = tm.copy()
    for k, n in [(3, 0), (1, 1), (0, 2), (3, 2), (0, 3)]:
        m[k, n] = 1
    B = (np.arange(20, dtype=np.float32).reshape(4, 5) + 1).astype(np.float16)
    p = opk.ref_pack(B, m, 2, opk.PATTERN_TEW, tile_mask=tm)
    assert p["col_idx"].tolist() == [0, 1, 3] and p["n_tiles"] == 2
    assert [r.tolist() for r in p["row_idx"]] == [[0, 2], [1]]
    assert p["ew_col_ptr"].tolist() == [0, 1, 2, 4, 5, 5]
    assert p["ew_row"].tolist() == [3, 1, 0, 3, 0]
    assert p["ew_val"].view(np.float16).tolist() == [16.0, 7.0, 3.0, 18.0, 4.0]
    assert p["values"][0].view(np.float16).tolist() == [[1.0, 2.0], [11.0, 12.0]]


@pytest.mark.parametrize("seed", range(6))
def test_tew_round_trip_and_csc_invariants(seed):
    rng = np.random.default_rng(200 + seed)
    K, N, G = int(rng.integers(1, 60)), int(rng.integers(1, 150)), int(rng.choice([32, 64, 128]))
    m, tm = _random_tew(rng, K, N, G)
    B = wl.rng_fp16(seed, (K, N))
    p = opk.ref_pack(B, m, G, opk.PATTERN_TEW, tile_mask=tm)
    tw_part = opk.ref_pack(B, tm, G, opk.PATTERN_TW)
    for key in ("col_idx", "cto_n"):
        assert np.array_equal(p[key], tw_part[key])
    for a, b in zip(p["values"], tw_part["values"]):
        assert np.array_equal(a, b)
    ptr = p["ew_col_ptr"]
    assert ptr[0] == 0 and ptr[-1] == int((m & ~tm & 1).sum()) == len(p["ew_row"]) == len(p["ew_val"])
    assert (np.diff(ptr) >= 0).all()
    for n in range(N):
        r = p["ew_row"][ptr[n]:ptr[n + 1]]
        assert (np.diff(r) > 0).all()                                    # ascending, no duplicates
        assert np.array_equal(r, np.flatnonzero((m[:, n] != 0) & (tm[:, n] == 0)))
    Bm, m2 = opk.ref_unpack(p)
    assert np.array_equal(m2, m)
    assert np.array_equal(Bm, np.where(m != 0, B.view(np.uint16), 0))


def test_tew_without_restored_elements_is_the_tw_form():
    rng = np.random.default_rng(9)
    tm = random_tw_mask(rng, 30, 70, 32)
    B = wl.rng_fp16(9, tm.shape)
    p = opk.ref_pack(B, tm, 32, opk.PATTERN_TEW, tile_mask=tm)
    assert p["ew_col_ptr"].tolist() == [0] * 71 and len(p["ew_row"]) == 0


def test_tew_rejects_bad_masks():
    rng = np.random.default_rng(10)
    m, tm = _random_tew(rng, 20, 40, 32)
    B = wl.rng_fp16(10, m.shape)
    with pytest.raises(ValueError):
        opk.ref_pack(B, m, 32, opk.PATTERN_TEW)                          # no tile mask
    bad = m.copy()
    k, n = np.argwhere(tm != 0)[0]
    bad[k, n] = 0                                                        # a TW element missing from the mask
    with pytest.raises(opk.MaskError):
        opk.ref_pack(B, bad, 32, opk.PATTERN_TEW, tile_mask=tm)
    with pytest.raises(opk.MaskError):
        opk.ref_pack(B, m, 32, opk.PATTERN_TEW, tile_mask=m)             # tile mask that is not tile-wise
