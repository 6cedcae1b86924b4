"""Parity of the HIP path against the CPU oracle, through the C ABI (-m gpu)."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from tests.helpers import assert_C_close, random_tw_mask
from tests import gpu_util as gu
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    for k, v in (("tile_m", 0), ("xcd_map", 1), ("kernel", 0), ("depth", 3), ("waves", 4), ("ksplit", 0)):
        tw.tw_set_option(k, v)
    yield
    for k, v in (("tile_m", 0), ("xcd_map", 1), ("kernel", 0), ("depth", 3), ("waves", 4), ("ksplit", 0)):
        tw.tw_set_option(k, v)


def _check_case(c, tile_m=0, **kw):
    print(f"case {c.name} M={c.M} K={c.K} N={c.N} G={c.G} seed={c.seed} tile_m={tile_m}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack(c.B, c.mask, c.G, tw.PATTERN_TW)
    C, raw = gu.run_tw(tw, p, c.A, c.N, **kw)
    p.free()
    assert_C_close(C, og.gemm_oracle(c.A, c.B, c.mask), og.abs_bound(c.A, c.B, c.mask))
    return raw


def test_config1_tiny_tw():
    _check_case(wl.make_case(1))


@pytest.mark.parametrize("tile_m", [64, 128, 256])
@pytest.mark.parametrize("G", [32, 64, 128])
def test_tile_shapes(G, tile_m):
    if G == 32 and tile_m == 64:
        pytest.skip("no 64x32 instance")
    rng = np.random.default_rng(G + tile_m)
    M, K, N = 328, 150, 300                     # M, K, N all ragged
    mask = random_tw_mask(rng, K, N, G, col_keep=0.85, row_keep=0.5)
    c = wl.Case("ragged", M, K, N, G, "tw", 0.0, G + tile_m, wl.make_A(1, M, K), wl.make_B(1, K, N, 1.0), mask, mask)
    _check_case(c, tile_m)


def test_identity_A_is_bit_exact():
    """A = I: every C element has at most one term, so C must equal fp16(B (.) mask)
    bit for bit; pins row_idx, col_idx and the tile layout end to end."""
    rng = np.random.default_rng(5)
    K, N, G = 200, 330, 64
    mask = random_tw_mask(rng, K, N, G)
    B = wl.make_B(5, K, N, 1.0)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    C, raw = gu.run_tw(tw, p, np.eye(K, dtype=np.float16), N)
    p.free()
    want = np.where(mask != 0, B, np.float16(0)).astype(np.float16)
    assert np.array_equal(raw[:, :K].T.view(np.uint16), want.view(np.uint16))


def test_all_ones_counts_kept_rows():
    rng = np.random.default_rng(6)
    K, N, G, M = 500, 260, 128, 72
    mask = random_tw_mask(rng, K, N, G)
    p = tw.tw_pack(np.ones((K, N), np.float16), mask, G, tw.PATTERN_TW)
    C, _ = gu.run_tw(tw, p, np.ones((M, K), np.float16), N)
    p.free()
    assert np.array_equal(C, np.broadcast_to(mask.sum(0).astype(np.float64), (M, N)))


def test_pruned_columns_are_plus_zero_and_padding_untouched():
    c = wl.make_case(1, M=100)
    rng = np.random.default_rng(7)
    mask = random_tw_mask(rng, c.K, c.N, c.G, col_keep=0.6, row_keep=0.5)
    c.mask = mask
    raw = _check_case(c, lda=112, ldc=120, fill=7.0)
    dead = ~mask.any(0)
    assert dead.any()
    assert not raw[dead, :100].view(np.uint16).any()          # +0, not -0
    assert (raw[:, 100:] == 7.0).all()                        # ldc padding untouched


@pytest.mark.parametrize("M", [1, 7, 8, 63, 65, 129, 1568])
def test_M_tails(M):
    c = wl.make_case(1, M=M)
    _check_case(c)


def test_empty_mask_and_empty_tile():
    c = wl.make_case(1, M=40)
    c.mask = np.zeros_like(c.mask)
    raw = _check_case(c)
    assert not raw[:, :40].view(np.uint16).any()
    # one tile with no kept rows cannot exist (its columns would be pruned); a tile
    # with a single kept row is the smallest
    c.mask = np.zeros_like(c.mask)
    c.mask[17, 64:128] = 1
    _check_case(c)


def test_zero_sparsity_equals_dense_baseline():
    c = wl.make_case(1, sparsity=0.0, M=200)
    raw_tw = _check_case(c)
    C, raw_d = gu.run_dense(tw, c.A, c.B)
    assert_C_close(C, og.gemm_oracle(c.A, c.B, c.mask), og.abs_bound(c.A, c.B, c.mask))
    assert np.array_equal(raw_tw.view(np.uint16)[:, :200], raw_d.view(np.uint16)[:, :200])


@pytest.mark.parametrize("M,K,N", [(128, 256, 256), (333, 100, 77), (64, 33, 520), (1000, 770, 136)])
def test_dense_baseline(M, K, N):
    A, B = wl.make_A(M + K, M, K), wl.make_B(N, K, N, 0.05)
    ones = np.ones((K, N), np.uint8)
    for tm in (0, 64, 128, 256):
        tw.tw_set_option("tile_m", tm)
        C, raw = gu.run_dense(tw, A, B, ldb=(N + 7) // 8 * 8 + 8)
        assert_C_close(C, og.gemm_oracle(A, B, ones), og.abs_bound(A, B, ones))


@pytest.mark.parametrize("M", [1024, 1000])      # M-tiles a multiple of 8 (tile-major order applies) and not
def test_workgroup_orders_give_the_same_result(M):
    c = wl.make_case(2, 0, M=M)
    raw1 = _check_case(c)
    for mode in (0, 2):
        tw.tw_set_option("xcd_map", mode)
        raw2 = _check_case(c)
        assert np.array_equal(raw1.view(np.uint16), raw2.view(np.uint16))
        if M == 1024:
            assert np.array_equal(_check_case(c, tile_m=64).view(np.uint16), raw1.view(np.uint16))


@pytest.mark.parametrize("recipe", ["per_tile", "global", "paper"])
def test_bert_base_recipes_reduced_M(recipe):
    c = wl.make_case(2, 0, M=512, recipe=recipe)
    _check_case(c)


@pytest.mark.parametrize("shape_index", [0, 1, 2])
def test_config2_full_size_sampled(shape_index):
    """Full BERT-base shapes in the launch configuration the benchmark times;
    the oracle is evaluated on sampled rows of C (all columns)."""
    c = wl.make_case(2, shape_index)
    print(f"case {c.name}", flush=True)
    p = tw.tw_pack(c.B, c.mask, c.G, tw.PATTERN_TW)
    C, raw = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    rows = np.r_[0:8, 120:136, 2040:2056, c.M - 8:c.M, np.arange(3, c.M, 257)]
    assert_C_close(C[rows], og.gemm_oracle(c.A[rows], c.B, c.mask), og.abs_bound(c.A[rows], c.B, c.mask))
    dead = ~c.mask.any(0)
    assert not raw[dead].view(np.uint16).any()
    assert np.isfinite(C).all()
