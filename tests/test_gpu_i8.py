"""Int8 TW path against the integer oracle, through the C ABI (-m gpu): every sum is
exact, so every comparison is bit for bit."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from tests.helpers import random_tw_mask, random_tvw_mask
from tests import gpu_util as gu
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    tw.tw_set_option("tile_m", 0)
    tw.tw_set_option("ksplit", 0)
    yield
    tw.tw_set_option("tile_m", 0)
    tw.tw_set_option("ksplit", 0)


def _case(seed, M, K, N, G, col_keep=0.8, row_keep=0.5):
    rng = np.random.default_rng(seed)
    mask = random_tw_mask(rng, K, N, G, col_keep=col_keep, row_keep=row_keep)
    return wl.rng_i8(seed, (M, K)), wl.rng_i8(seed + 1, (K, N)), mask


@pytest.mark.parametrize("G,tile_m", [(64, 128), (64, 256), (128, 64), (128, 128), (128, 256)])
def test_i8_ragged_shapes_int32(G, tile_m):
    M, K, N = 333, 210, 300                       # all ragged, several tiles in M and N
    A, B, mask = _case(G + tile_m, M, K, N, G)
    print(f"i8 ragged G={G} tile_m={tile_m} M={M} K={K} N={N}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack_i8(B, mask, G)
    C, raw = gu.run_tw_i8(tw, p, A, N)
    p.free()
    assert np.array_equal(C, og.gemm_i8_oracle(A, B, mask))
    assert (raw[:, M:] == -77).all()              # padding of C untouched
    assert (raw[~mask.any(0), :M] == 0).all()     # pruned columns are written as 0


@pytest.mark.parametrize("G,tile_m", [(128, 64), (128, 128), (64, 256)])
def test_i8_requantised_output(G, tile_m):
    M, K, N = 190, 300, 200
    A, B, mask = _case(7 + G, M, K, N, G)
    scale = 1.0 / 151.0
    print(f"i8 requantised G={G} tile_m={tile_m}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack_i8(B, mask, G)
    C, raw = gu.run_tw_i8(tw, p, A, N, c_dtype=1, scale=scale)
    p.free()
    want = og.requantize_i8(og.gemm_i8_oracle(A, B, mask), scale)
    assert (want == 127).any() and (want == -128).any() and (np.abs(want) < 100).any()   # clamps and interior both hit
    assert np.array_equal(C, want.astype(np.int64))
    assert (raw[:, M:] == -77).all()


def test_i8_halves_round_to_even():
    """scale = 0.5 on sums of known parity: x.5 must go to the even neighbour."""
    K, N, G, M = 64, 64, 64, 40
    A = np.zeros((M, K), np.int8)
    A[:, 0] = np.arange(M) - 20                    # sum = (i - 20) * 1
    B = np.zeros((K, N), np.int8)
    B[0, :] = 1
    mask = np.ones((K, N), np.uint8)
    p = tw.tw_pack_i8(B, mask, G)
    C, _ = gu.run_tw_i8(tw, p, A, N, c_dtype=1, scale=0.5)
    p.free()
    want = og.requantize_i8(og.gemm_i8_oracle(A, B, mask), 0.5)
    assert np.array_equal(C, want.astype(np.int64))
    assert C[21, 0] == 0 and C[23, 0] == 2 and C[17, 0] == -2     # 0.5 -> 0, 1.5 -> 2, -1.5 -> -2


def test_i8_extreme_values_do_not_overflow():
    K, N, G, M = 4096, 128, 128, 130
    A = np.full((M, K), -128, np.int8)
    B = np.full((K, N), -128, np.int8)
    B[:, 1] = 127
    mask = np.ones((K, N), np.uint8)
    p = tw.tw_pack_i8(B, mask, G)
    C, _ = gu.run_tw_i8(tw, p, A, N)
    p.free()
    assert (C[:, 0] == 4096 * 16384).all() and (C[:, 1] == -4096 * 128 * 127).all()
    assert np.array_equal(C, og.gemm_i8_oracle(A, B, mask))


def test_i8_identity_A_returns_the_masked_weight():
    """A = I: C = B (.) mask; pins row and column index lists and the byte layout end to end."""
    rng = np.random.default_rng(11)
    K, N, G = 200, 330, 64
    mask = random_tw_mask(rng, K, N, G)
    B = wl.rng_i8(11, (K, N))
    p = tw.tw_pack_i8(B, mask, G)
    C, _ = gu.run_tw_i8(tw, p, np.eye(K, dtype=np.int8), N)
    p.free()
    assert np.array_equal(C, np.where(mask != 0, B, 0).astype(np.int64))


def test_i8_degenerate_masks():
    M, K, N, G = 70, 100, 150, 64
    A, B = wl.rng_i8(1, (M, K)), wl.rng_i8(2, (K, N))
    for name, mask in (("nothing kept", np.zeros((K, N), np.uint8)), ("everything kept", np.ones((K, N), np.uint8))):
        print(f"i8 degenerate: {name}", flush=True)
        p = tw.tw_pack_i8(B, mask, G)
        C, _ = gu.run_tw_i8(tw, p, A, N)
        p.free()
        assert np.array_equal(C, og.gemm_i8_oracle(A, B, mask))
    mask = np.zeros((K, N), np.uint8)              # one tile whose columns keep a single row
    mask[37, 5:40] = 1
    p = tw.tw_pack_i8(B, mask, G)
    C, _ = gu.run_tw_i8(tw, p, A, N)
    p.free()
    assert np.array_equal(C, og.gemm_i8_oracle(A, B, mask))


@pytest.mark.parametrize("c_dtype", [0, 1])
def test_i8_dense_baseline(c_dtype):
    M, K, N = 300, 192, 200
    A, B = wl.rng_i8(5, (M, K)), wl.rng_i8(6, (K, N))
    scale = 1.0 / 977.0
    for tile_m in (64, 128, 256):
        print(f"i8 dense c_dtype={c_dtype} tile_m={tile_m}", flush=True)
        tw.tw_set_option("tile_m", tile_m)
        C, raw = gu.run_dense_i8(tw, A, B, c_dtype=c_dtype, scale=scale)
        want = og.gemm_i8_oracle(A, B, np.ones((K, N), np.uint8))
        if c_dtype:
            want = og.requantize_i8(want, scale).astype(np.int64)
        assert np.array_equal(C, want)
        assert (raw[:, M:] == -77).all()


def test_i8_concat_runs_as_one_launch():
    rng = np.random.default_rng(21)
    M, K, G = 150, 130, 128
    A = wl.rng_i8(20, (M, K))
    parts, Bs, masks = [], [], []
    for i, N in enumerate((200, 128, 70)):
        masks.append(random_tw_mask(rng, K, N, G)); Bs.append(wl.rng_i8(30 + i, (K, N)))
        parts.append(tw.tw_pack_i8_host(Bs[-1], masks[-1], G))
    cat = tw.tw_concat(parts)
    C, _ = gu.run_tw_i8(tw, cat, A, 398)
    cat.free()
    assert np.array_equal(C, og.gemm_i8_oracle(A, np.concatenate(Bs, 1), np.concatenate(masks, 1)))


def test_i8_full_size_bert_shape_on_sampled_rows():
    """768 x 3072 at M = 4096 in the launch configuration the benchmark times (automatic tile
    choice), checked on sampled rows of C the oracle computes one by one."""
    M, K, N, G = 4096, 768, 3072, 128
    A, B = wl.rng_i8(40, (M, K)), wl.rng_i8(41, (K, N), sigma=30.0)
    rng = np.random.default_rng(42)
    mask = random_tw_mask(rng, K, N, G, col_keep=0.5, row_keep=0.5)
    print("i8 full size 768x3072 M=4096", flush=True)
    p = tw.tw_pack_i8(B, mask, G)
    C, _ = gu.run_tw_i8(tw, p, A, N)
    p.free()
    rows = np.concatenate([[0, 127, 128, 255, 256, M - 1], rng.integers(0, M, 58)])
    assert np.array_equal(C[rows], og.gemm_i8_oracle(A[rows], B, mask))


# ---- TVW on the sparse int8 matrix instruction -------------------------------------------

@pytest.mark.parametrize("G,tile_m", [(128, 64), (128, 128), (64, 128)])
@pytest.mark.parametrize("full", [True, False])
def test_i8_tvw_ragged_shapes(G, tile_m, full):
    M, K, N = 333, 420, 300                       # K_t of about 210: two stages with a ragged tail
    rng = np.random.default_rng(G + tile_m + full)
    mask, tmask = random_tvw_mask(rng, K, N, G, col_keep=0.85, row_keep=0.5, full=full)
    A, B = wl.rng_i8(50, (M, K)), wl.rng_i8(51, (K, N))
    print(f"i8 tvw G={G} tile_m={tile_m} full={full}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack_i8(B, mask, G, tw.PATTERN_TVW, tile_mask=tmask)
    C, raw = gu.run_tw_i8(tw, p, A, N)
    p.free()
    assert np.array_equal(C, og.gemm_i8_oracle(A, B, mask))
    assert (raw[:, M:] == -77).all()
    assert (raw[~tmask.any(0), :M] == 0).all()


def test_i8_tvw_every_position_pair_and_identity_A():
    """A = I and a mask that walks all six position pairs through every group and column:
    C must be B (.) mask exactly (pins the position words and the byte order of the sparse operand)."""
    K, N, G = 256, 128, 128
    pairs = [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3)]
    mask = np.zeros((K, N), np.uint8)
    for g4 in range(K // 4):
        for n in range(N):
            a, b = pairs[(g4 * 5 + n) % 6]
            mask[4 * g4 + a, n] = mask[4 * g4 + b, n] = 1
    B = wl.rng_i8(60, (K, N))
    B[B == 0] = 3
    p = tw.tw_pack_i8(B, mask, G, tw.PATTERN_TVW, tile_mask=np.ones((K, N), np.uint8))
    C, _ = gu.run_tw_i8(tw, p, np.eye(K, dtype=np.int8), N)
    p.free()
    assert np.array_equal(C, np.where(mask != 0, B, 0).astype(np.int64))


def test_i8_tvw_requantised_and_full_size_samples():
    M, K, N, G = 4096, 768, 3072, 128
    A, B = wl.rng_i8(70, (M, K)), wl.rng_i8(71, (K, N), sigma=30.0)
    rng = np.random.default_rng(72)
    mask, tmask = random_tvw_mask(rng, K, N, G, col_keep=0.9, row_keep=0.3)
    scale = 1.0 / 97.0
    print("i8 tvw full size 768x3072 M=4096, int8 output", flush=True)
    p = tw.tw_pack_i8(B, mask, G, tw.PATTERN_TVW, tile_mask=tmask)
    C, _ = gu.run_tw_i8(tw, p, A, N, c_dtype=1, scale=scale)
    p.free()
    rows = np.concatenate([[0, 63, 64, 127, 128, M - 1], rng.integers(0, M, 58)])
    want = og.requantize_i8(og.gemm_i8_oracle(A[rows], B, mask), scale)
    assert (np.abs(want) < 100).any() and (np.abs(want) == 127).any()
    assert np.array_equal(C[rows], want.astype(np.int64))


def test_i8_requantisation_of_sums_beyond_24_bits():
    """Sums of 2^24 + 1 and 2^24 + 3 are not binary32 values: the conversion must round them to even
    (2^24 and 2^24 + 4) before the one fp32 product, which a scale of 2.5 * 2^-24 turns into 2.5
    (-> 2, half to even) and 2.5000006 (-> 3)."""
    K, N, G, M = 1043, 64, 64, 20
    a = np.zeros(K, np.int8)
    cols = np.zeros((K, 3), np.int8)
    a[:1040] = 127; cols[:1040, :] = 127                   # 1040 * 16129 = 16774160
    a[1040] = 24; cols[1040, :] = 127                      # + 3048
    a[1041] = 9; cols[1041, :] = 1                         # + 9          = 2^24 + 1
    a[1042] = 2; cols[1042, 2] = 1                         # third column: + 2 = 2^24 + 3
    cols[:, 1] = -cols[:, 1]                               # second column: -(2^24 + 1)
    A = np.tile(a, (M, 1))
    B = np.zeros((K, N), np.int8)
    B[:, :3] = cols
    mask = np.ones((K, N), np.uint8)
    scale = float(np.float32(2.5 * 2.0 ** -24))
    sums = og.gemm_i8_oracle(A, B, mask)
    assert sums[0, :3].tolist() == [2 ** 24 + 1, -(2 ** 24 + 1), 2 ** 24 + 3]
    p = tw.tw_pack_i8(B, mask, G)
    C32, _ = gu.run_tw_i8(tw, p, A, N)
    C8, _ = gu.run_tw_i8(tw, p, A, N, c_dtype=1, scale=scale)
    p.free()
    assert np.array_equal(C32, sums)
    assert np.array_equal(C8, og.requantize_i8(sums, scale).astype(np.int64))
    assert C8[0, :3].tolist() == [2, -2, 3]


def test_i8_refuses_what_the_32_bit_addressing_cannot_reach():
    """K * lda >= 2^32 bytes of A: refused with a status before anything is launched (the pointers
    are never dereferenced)."""
    K, N, G = 70000, 64, 64
    B = np.zeros((K, N), np.int8)
    B[::1000, :] = 1
    mask = np.zeros((K, N), np.uint8)
    mask[::1000, :] = 1
    p = tw.tw_pack_i8(B, mask, G)
    fake = 0x7f0000000000
    with pytest.raises(tw.TwError) as ei:
        tw.tw_gemm_i8(fake, 65536, 65536, p, fake, 65536)
    assert ei.value.status == 3
    # the same weight with a short M is fine and exact
    M = 48
    A = wl.rng_i8(80, (M, K))
    C, _ = gu.run_tw_i8(tw, p, A, N)
    p.free()
    assert np.array_equal(C, og.gemm_i8_oracle(A, B, mask))


@pytest.mark.parametrize("G,tile_m", [(128, 64), (128, 128), (64, 128)])
@pytest.mark.parametrize("stages64", [1, 4, 7])
@pytest.mark.parametrize("c_dtype", [0, 1])
def test_i8_k_split_inside_the_workgroup(G, tile_m, stages64, c_dtype):
    """Two K groups per workgroup: an odd number of 64-row stages leaves group 1 idle on the tail."""
    M, N = 200, 300
    K = 64 * stages64 + 90                        # kept rows per tile: 64*stages64 - 20 .. (ragged)
    rng = np.random.default_rng(G + tile_m + stages64 + c_dtype)
    mask = np.zeros((K, N), np.uint8)
    cols = np.flatnonzero(rng.random(N) < 0.9)
    for i in range(0, cols.size, G):
        rows = rng.permutation(K)[:64 * stages64 - int(rng.integers(0, 40))]
        mask[np.ix_(np.sort(rows), cols[i:i + G])] = 1
    A, B = wl.rng_i8(90, (M, K)), wl.rng_i8(91, (K, N))
    scale = 1.0 / 900.0
    print(f"i8 ksplit G={G} tile_m={tile_m} stages64={stages64} c_dtype={c_dtype}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    tw.tw_set_option("ksplit", 2)
    p = tw.tw_pack_i8(B, mask, G)
    C, raw = gu.run_tw_i8(tw, p, A, N, c_dtype=c_dtype, scale=scale)
    p.free()
    want = og.gemm_i8_oracle(A, B, mask)
    if c_dtype:
        want = og.requantize_i8(want, scale).astype(np.int64)
    assert np.array_equal(C, want)
    assert (raw[:, M:] == -77).all()


def test_i8_k_split_is_chosen_for_long_k_few_tiles():
    """3072 x 768 at M = 4096 (the shape the automatic choice splits), sampled rows."""
    M, K, N, G = 4096, 3072, 768, 128
    A, B = wl.rng_i8(92, (M, K)), wl.rng_i8(93, (K, N), sigma=30.0)
    mask = wl.tw_mask(B.astype(np.float16), G, density=0.25, col_frac=0.10)
    p = tw.tw_pack_i8(B, mask, G)
    C, _ = gu.run_tw_i8(tw, p, A, N, c_dtype=1, scale=1.0 / 2000.0)
    p.free()
    rng = np.random.default_rng(94)
    rows = np.concatenate([[0, 63, 64, M - 1], rng.integers(0, M, 60)])
    want = og.requantize_i8(og.gemm_i8_oracle(A[rows], B, mask), 1.0 / 2000.0)
    assert (np.abs(want) > 10).any()
    assert np.array_equal(C[rows], want.astype(np.int64))
