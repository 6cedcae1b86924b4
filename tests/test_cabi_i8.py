"""Host side of the int8 entry points (no GPU): the packer agrees with the oracle's
canonical form on the structure and with the definition V[j][w] = B[row][col] on the
values; argument errors come back as statuses."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import pack as opk
from tests.helpers import random_tw_mask, random_tvw_mask
import workloads as wl


@pytest.mark.parametrize("seed", range(6))
def test_i8_export_structure_and_values(seed):
    rng = np.random.default_rng(100 + seed)
    K, N = int(rng.integers(1, 150)), int(rng.integers(1, 300))
    G = int(rng.choice([32, 64, 128]))
    mask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.1, 1.0))
    B = wl.rng_i8(seed, (K, N))
    B[0, 0], B[-1, -1] = -128, 127
    p = tw.tw_pack_i8_host(B, mask, G)
    e = p.export()
    r = opk.ref_pack(np.zeros((K, N), np.float16), mask, G, opk.PATTERN_TW)   # structure: mask only
    assert e["dtype"] == tw.DTYPE_I8 and e["pattern"] == tw.PATTERN_TW
    assert e["n_kept"] == r["n_kept"] and e["n_tiles"] == r["n_tiles"]
    assert np.array_equal(e["col_idx"], r["col_idx"]) and np.array_equal(e["cto_n"], r["cto_n"])
    for t in range(r["n_tiles"]):
        assert np.array_equal(e["row_idx"][t], r["row_idx"][t])
        assert np.array_equal(e["cto_k"][t], r["cto_k"][t])
        cols = e["col_idx"][e["tile_col_off"][t]:e["tile_col_off"][t + 1]]
        assert e["values"][t].dtype == np.int8
        assert np.array_equal(e["values"][t], B[np.ix_(e["row_idx"][t], cols)])
    Bm, m2 = p.unpack()
    assert Bm.dtype == np.int8 and np.array_equal(m2, mask)
    assert np.array_equal(Bm, np.where(mask != 0, B, 0))
    p.free()


@pytest.mark.parametrize("seed,full", [(0, True), (1, False), (2, True)])
def test_i8_tvw_export_equals_oracle_pack(seed, full):
    """The packer moves 16-bit patterns without looking at them: the TVW form of an int8 weight is
    the oracle's TVW form of the same integers held in fp16 (exact), value for value."""
    rng = np.random.default_rng(200 + seed)
    K, N = int(rng.integers(4, 150)), int(rng.integers(1, 300))
    G = int(rng.choice([64, 128]))
    mask, tmask = random_tvw_mask(rng, K, N, G, full=full)
    B = wl.rng_i8(seed, (K, N))
    p = tw.tw_pack_i8_host(B, mask, G, tw.PATTERN_TVW, tile_mask=tmask)
    e = p.export()
    r = opk.ref_pack(B.astype(np.float16), mask, G, opk.PATTERN_TVW, tile_mask=tmask)
    assert e["dtype"] == tw.DTYPE_I8 and e["pattern"] == tw.PATTERN_TVW
    assert np.array_equal(e["col_idx"], r["col_idx"])
    for t in range(r["n_tiles"]):
        assert np.array_equal(e["row_idx"][t], r["row_idx"][t])
        assert np.array_equal(e["meta"][t], r["meta"][t]) and np.array_equal(e["valid"][t], r["valid"][t])
        assert np.array_equal(e["values"][t].astype(np.float16).view(np.uint16), r["values"][t])
    Bm, m2 = p.unpack()
    assert np.array_equal(m2, mask) and np.array_equal(Bm, np.where(mask != 0, B, 0))
    p.free()


def test_i8_rejects_a_non_tw_mask():
    mask = np.ones((8, 64), np.uint8)
    mask[3, 5] = 0
    with pytest.raises(tw.TwError) as ei:
        tw.tw_pack_i8_host(np.ones((8, 64), np.int8), mask, 64)
    assert ei.value.status == 2
    with pytest.raises(tw.TwError) as ei:
        tw.tw_pack_i8_host(np.ones((8, 64), np.int8), np.ones((8, 64), np.uint8), 64, tw.PATTERN_TEW,
                           tile_mask=np.ones((8, 64), np.uint8))
    assert ei.value.status == 3


def test_i8_concat_and_dtype_mismatch():
    rng = np.random.default_rng(3)
    K, G = 70, 64
    parts, Bs, masks = [], [], []
    for i, N in enumerate((100, 64, 37)):
        m = random_tw_mask(rng, K, N, G)
        B = wl.rng_i8(10 + i, (K, N))
        parts.append(tw.tw_pack_i8_host(B, m, G)); Bs.append(B); masks.append(m)
    cat = tw.tw_concat(parts, upload=False)
    Bm, m2 = cat.unpack()
    assert np.array_equal(m2, np.concatenate(masks, 1))
    assert np.array_equal(Bm, np.where(m2 != 0, np.concatenate(Bs, 1), 0))
    f16 = tw.tw_pack_host(np.ones((K, 64), np.float16), np.ones((K, 64), np.uint8), G, tw.PATTERN_TW)
    with pytest.raises(tw.TwError) as ei:
        tw.tw_concat([parts[0], f16], upload=False)
    assert ei.value.status == 1


def test_i8_gemm_argument_errors_need_no_device():
    K, N, G, M = 64, 64, 64, 32
    fake = 0x10000                      # aligned, never dereferenced: every call fails before
    p8 = tw.tw_pack_i8_host(np.ones((K, N), np.int8), np.ones((K, N), np.uint8), G)
    p16 = tw.tw_pack_host(np.ones((K, N), np.float16), np.ones((K, N), np.uint8), G, tw.PATTERN_TW)

    def status(fn, *a):
        with pytest.raises(tw.TwError) as ei:
            fn(*a)
        return ei.value.status

    assert status(tw.tw_gemm, fake, M, 32, tw.LAYOUT_KM, p8, fake, 32) == 1          # int8 handle
    assert status(tw.tw_gemm_i8, fake, M, 32, p16, fake, 32) == 1                    # fp16 handle
    assert status(tw.tw_gemm_i8, fake, M, 24, p8, fake, 32) == 1                     # lda % 16
    assert status(tw.tw_gemm_i8, fake, M, 32, p8, fake, 16) == 1                     # ldc < M
    assert status(tw.tw_gemm_i8, fake + 8, M, 32, p8, fake, 32) == 1                 # alignment
    assert status(tw.tw_gemm_i8, fake, M, 32, p8, fake, 32, 2) == 1                  # c_dtype
    assert status(tw.tw_gemm_i8, fake, M, 32, p8, fake, 32) == 6                     # not uploaded
    assert status(tw.tw_dense_gemm_i8, fake, fake, fake, M, 65, N, 32, 64, 32) == 3  # K % 64
    assert status(tw.tw_dense_gemm_i8, fake, fake, fake, M, 64, N, 32, 48, 32) == 1  # ldb < N
    p8.free(); p16.free()
