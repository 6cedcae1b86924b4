"""Parity of the TVW (tile-wise + 2:4) HIP path against the CPU oracle (-m gpu)."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from tests.helpers import assert_C_close, random_tvw_mask
from tests import gpu_util as gu
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    tw.tw_set_option("tile_m", 0)
    yield
    tw.tw_set_option("tile_m", 0)


def _run(A, B, mask, tile_mask, G, **kw):
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TVW, tile_mask=tile_mask)
    C, raw = gu.run_tw(tw, p, A, B.shape[1], **kw)
    p.free()
    return C, raw


def test_every_position_pair_bit_exact():
    """A = I_K and one group of four kept rows per pair (p0, p1): each C element
    has at most one term, so C must be fp16(B (.) mask) bit for bit.  All six
    position pairs occur in every lane group and column block; this pins the
    2-bit position encoding and the operand layout of the sparse instruction."""
    K, N, G = 256, 128, 128
    pairs = [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3)]
    mask = np.zeros((K, N), np.uint8)
    for g in range(K // 4):
        for n in range(N):
            p0, p1 = pairs[(g + n) % 6]
            mask[4 * g + p0, n] = 1
            mask[4 * g + p1, n] = 1
    B = wl.make_B(11, K, N, 1.0)
    print("case tvw position pairs", flush=True)
    C, raw = _run(np.eye(K, dtype=np.float16), B, mask, np.ones_like(mask), G)
    want = np.where(mask != 0, B, np.float16(0)).astype(np.float16)
    assert np.array_equal(raw[:, :K].T.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("G", [64, 128])
def test_identity_A_random_structure_bit_exact(G):
    rng = np.random.default_rng(21 + G)
    K, N = 300, 330
    mask, tm = random_tvw_mask(rng, K, N, G, full=False)
    B = wl.make_B(21, K, N, 1.0)
    print("case tvw identity random", flush=True)
    C, raw = _run(np.eye(K, dtype=np.float16), B, mask, tm, G)
    want = np.where(mask != 0, B, np.float16(0)).astype(np.float16)
    assert np.array_equal(raw[:, :K].T.view(np.uint16), want.view(np.uint16))


def test_all_ones_counts_kept_elements():
    rng = np.random.default_rng(22)
    K, N, G, M = 520, 260, 128, 72
    mask, tm = random_tvw_mask(rng, K, N, G)
    print("case tvw all ones", flush=True)
    C, _ = _run(np.ones((M, K), np.float16), np.ones((K, N), np.float16), mask, tm, G)
    assert np.array_equal(C, np.broadcast_to(mask.sum(0).astype(np.float64), (M, N)))


@pytest.mark.parametrize("tile_m", [256, 64])
@pytest.mark.parametrize("M", [8, 300, 520])
def test_other_tile_heights(M, tile_m):
    """The 256 x 128 (8 waves) and 64 x 128 instances: identity A pins the layout bit for
    bit, random A goes against the oracle; M below, across and beyond one tile."""
    rng = np.random.default_rng(40 + M)
    K, N, G = 330, 300, 128
    mask, tm = random_tvw_mask(rng, K, N, G, full=(M != 300))
    B = wl.make_B(40, K, N, 1.0)
    tw.tw_set_option("tile_m", tile_m)
    print(f"case tvw {tile_m}-row tiles M={M}", flush=True)
    A = wl.make_A(M, M, K)
    C, raw = _run(A, B, mask, tm, G, fill=3.0, ldc=(M + 7) // 8 * 8 + 8)
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    assert not raw[~mask.any(0), :M].view(np.uint16).any()
    assert (raw[:, M:] == 3.0).all()
    C, raw = _run(np.eye(K, dtype=np.float16), B, mask, tm, G)
    want = np.where(mask != 0, B, np.float16(0)).astype(np.float16)
    assert np.array_equal(raw[:, :K].T.view(np.uint16), want.view(np.uint16))
    tw.tw_set_option("tile_m", 128)
    _, raw128 = _run(A, B, mask, tm, G)
    tw.tw_set_option("tile_m", tile_m)
    _, raw256 = _run(A, B, mask, tm, G)
    assert np.array_equal(raw128[:, :M].view(np.uint16), raw256[:, :M].view(np.uint16))


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("M", [1, 8, 129, 333])
def test_random_masks_and_M_tails(M, G):
    rng = np.random.default_rng(30 + M + G)
    K, N = 410, 300
    mask, tm = random_tvw_mask(rng, K, N, G, full=(M % 2 == 1))
    A, B = wl.make_A(M, M, K), wl.make_B(M, K, N, 1.0)
    print(f"case tvw random M={M}", flush=True)
    C, raw = _run(A, B, mask, tm, G, fill=3.0, ldc=(M + 7) // 8 * 8 + 8)
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    dead = ~mask.any(0)
    assert not raw[dead, :M].view(np.uint16).any()
    assert (raw[:, M:] == 3.0).all()


def test_plain_2_4_is_tvw_with_nothing_pruned_tile_wise():
    # TVW at 50 %: every aligned group of four K rows keeps two (plain 2:4)
    c = wl.make_case(3, 0, sparsity=0.5, col_frac=0.0, M=256)
    assert c.tile_mask.all()
    print(f"case {c.name}", flush=True)
    C, _ = _run(c.A, c.B, c.mask, c.tile_mask, c.G)
    assert_C_close(C, og.gemm_oracle(c.A, c.B, c.mask), og.abs_bound(c.A, c.B, c.mask))


@pytest.mark.parametrize("recipe", ["per_tile", "global"])
def test_bert_base_tvw_reduced_M(recipe):
    c = wl.make_case(3, 0, M=512, recipe=recipe)
    print(f"case {c.name}", flush=True)
    C, _ = _run(c.A, c.B, c.mask, c.tile_mask, c.G)
    assert_C_close(C, og.gemm_oracle(c.A, c.B, c.mask), og.abs_bound(c.A, c.B, c.mask))


@pytest.mark.parametrize("shape_index", [0, 1, 2])
def test_config3_full_size_sampled(shape_index):
    c = wl.make_case(3, shape_index)
    print(f"case {c.name}", flush=True)
    C, raw = _run(c.A, c.B, c.mask, c.tile_mask, c.G)
    rows = np.r_[0:8, 120:136, 2040:2056, c.M - 8:c.M, np.arange(3, c.M, 257)]
    assert_C_close(C[rows], og.gemm_oracle(c.A[rows], c.B, c.mask), og.abs_bound(c.A[rows], c.B, c.mask))
    assert not raw[~c.mask.any(0)].view(np.uint16).any()
    assert np.isfinite(C).all()


def test_unsupported_tile_width_is_an_error_not_a_fallback():
    rng = np.random.default_rng(40)
    mask, tm = random_tvw_mask(rng, 64, 64, 32)
    p = tw.tw_pack(wl.make_B(1, 64, 64, 1.0), mask, 32, tw.PATTERN_TVW, tile_mask=tm)
    import torch
    At = torch.zeros((64, 8), dtype=torch.float16, device="cuda")
    Ct = torch.zeros((64, 8), dtype=torch.float16, device="cuda")
    with pytest.raises(tw.TwError) as e:
        tw.tw_gemm(At.data_ptr(), 8, 8, tw.LAYOUT_KM, p, Ct.data_ptr(), 8, 0)
    assert e.value.status == 3
    p.free()
