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
