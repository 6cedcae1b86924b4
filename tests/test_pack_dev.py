"""Device-side packer (tw_pack_dev): the handle it builds from device buffers equals the oracle's
canonical packed form bit for bit (index lists, values, 2:4 positions and valid bits), refuses
what the host packer refuses, multiplies like a host-packed handle, and moves no weight to the host."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from oracle import pack as opk
from tests.helpers import assert_C_close, random_tw_mask, random_tvw_mask
from tests.test_cabi_packer import _same
import workloads as wl

pytestmark = pytest.mark.gpu


def _pack_dev(B, mask, G, pattern, tile_mask=None, ldb=None):
    import torch
    K, N = B.shape
    ldb = ldb or N
    Bp = np.full((K, ldb), 7.0, np.float16)
    Bp[:, :N] = B
    Bd = torch.from_numpy(Bp).cuda()
    md = torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).cuda()
    td = None if tile_mask is None else torch.from_numpy(np.ascontiguousarray(tile_mask, dtype=np.uint8)).cuda()
    return tw.tw_pack_dev(Bd.data_ptr(), ldb, md.data_ptr(), None if td is None else td.data_ptr(), K, N, G, pattern,
                          torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("seed", range(10))
def test_tw_equals_oracle_pack(seed):
    rng = np.random.default_rng(seed)
    K, N = int(rng.integers(1, 300)), int(rng.integers(1, 400))
    G = int(rng.choice([32, 64, 128]))
    mask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.1, 1.0))
    B = wl.rng_fp16(seed, (K, N))
    print(f"case pack_dev tw seed={seed} K={K} N={N} G={G}", flush=True)
    p = _pack_dev(B, mask, G, tw.PATTERN_TW, ldb=N + 8 * (seed % 2))
    _same(p.export(), opk.ref_pack(B, mask, G, opk.PATTERN_TW))
    Bm, m2 = p.unpack()
    assert np.array_equal(m2, mask) and np.array_equal(Bm, np.where(mask != 0, B.view(np.uint16), 0))
    p.free()


@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("with_tile_mask", [True, False])
def test_tvw_equals_oracle_pack(seed, with_tile_mask):
    rng = np.random.default_rng(100 + seed)
    K, N = int(rng.integers(1, 300)), int(rng.integers(1, 400))
    G = int(rng.choice([32, 64, 128]))
    mask, tm = random_tvw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.2, 1.0),
                               full=bool(seed % 2))                 # odd seeds: groups with fewer than two kept
    B = wl.rng_fp16(seed, (K, N))
    B[rng.random((K, N)) < 0.05] = 0                                 # kept zeros: valid bits cannot come from values
    print(f"case pack_dev tvw seed={seed} K={K} N={N} G={G} tile_mask={with_tile_mask}", flush=True)
    tmask = tm if with_tile_mask else None
    try:
        want = opk.ref_pack(B, mask, G, opk.PATTERN_TVW, tile_mask=tmask)
    except opk.MaskError:
        with pytest.raises(tw.TwError) as ei:
            _pack_dev(B, mask, G, tw.PATTERN_TVW, tile_mask=tmask)
        assert ei.value.status == 2
        return
    p = _pack_dev(B, mask, G, tw.PATTERN_TVW, tile_mask=tmask)
    _same(p.export(), want)
    p.free()


def test_masks_the_host_packer_refuses_are_refused():
    rng = np.random.default_rng(1)
    K, N, G = 40, 100, 32
    B = wl.rng_fp16(1, (K, N))
    mask = random_tw_mask(rng, K, N, G)
    hole = mask.copy()
    k, n = np.argwhere(hole)[7]
    hole[k, n] = 0                                                   # a kept row of a tile with a hole
    with pytest.raises(tw.TwError) as ei:
        _pack_dev(B, hole, G, tw.PATTERN_TW)
    assert ei.value.status == 2
    vm, tm = random_tvw_mask(rng, K, N, G)
    three = vm.copy()
    cols = np.flatnonzero(tm.any(0))
    rows = np.flatnonzero(tm[:, cols[0]])
    three[rows[:3], cols[0]] = 1                                     # three kept in one group of four
    with pytest.raises(tw.TwError) as ei:
        _pack_dev(B, three, G, tw.PATTERN_TVW, tile_mask=tm)
    assert ei.value.status == 2
    outside = vm.copy()
    outside[np.argwhere(tm == 0)[0][0], np.argwhere(tm == 0)[0][1]] = 1   # element mask leaves the tile mask
    with pytest.raises(tw.TwError) as ei:
        _pack_dev(B, outside, G, tw.PATTERN_TVW, tile_mask=tm)
    assert ei.value.status == 2
    empty = _pack_dev(B, np.zeros((K, N), np.uint8), G, tw.PATTERN_TW)      # nothing kept: a valid, empty weight
    assert empty.export()["n_tiles"] == 0
    empty.free()


@pytest.mark.parametrize("pattern", ["tw", "tvw"])
def test_device_packed_handle_multiplies_concats_and_binds(pattern):
    from tests import gpu_util as gu
    rng = np.random.default_rng(9)
    M, K, N, G = 300, 288, 330, 128
    B = wl.make_B(9, K, N, 0.1)
    A = wl.make_A(9, M, K)
    if pattern == "tw":
        mask = tm = random_tw_mask(rng, K, N, G)
        pat = tw.PATTERN_TW
    else:
        mask, tm = random_tvw_mask(rng, K, N, G)
        pat = tw.PATTERN_TVW
    pd = _pack_dev(B, mask, G, pat, tile_mask=tm if pattern == "tvw" else None)
    ph = tw.tw_pack(B, mask, G, pat, tile_mask=tm if pattern == "tvw" else None)
    Cd, rawd = gu.run_tw(tw, pd, A, N)
    Ch, rawh = gu.run_tw(tw, ph, A, N)
    assert np.array_equal(rawd.view(np.uint16)[:, :M], rawh.view(np.uint16)[:, :M])      # same image, same launch
    assert_C_close(Cd, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    both = tw.tw_concat([pd, ph])                                                         # fetches pd's values
    Cc, _ = gu.run_tw(tw, both, A, 2 * N)
    assert np.array_equal(Cc[:, :N], Cd) and np.array_equal(Cc[:, N:], Cd)
    g = wl.same_geom(32, 3, 3, 1, 10, 10)                                                 # K = 288
    X = wl.make_conv_input(10, g)
    Cw, _ = gu.run_conv(tw, pd, X, g, N)
    Cw2, _ = gu.run_conv(tw, ph, X, g, N)
    assert np.array_equal(Cw, Cw2)
    for p in (both, pd, ph):
        p.free()


def test_bert_base_ffn1_device_prune_then_pack_equals_host_pack():
    """768 x 3072 at the configured sparsity, pruned and packed on the device, against the host
    packer on the same masks, list by list and value by value."""
    import torch
    c = wl.make_case(3, 1, with_A=False)
    p_dev = _pack_dev(c.B, c.mask, c.G, tw.PATTERN_TVW, tile_mask=c.tile_mask)
    _same(p_dev.export(), opk.ref_pack(c.B, c.mask, c.G, opk.PATTERN_TVW, tile_mask=c.tile_mask))
    p_dev.free()
