"""Convolution through the implicit img2col gather: host checks (CPU) and parity of the HIP
path against the img2col-GEMM oracle over the wide grid (-m gpu)."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import conv as oc
from oracle import gemm as og
from tests.helpers import assert_C_close, random_tw_mask, random_tvw_mask
import workloads as wl


def _status(fn, *a):
    with pytest.raises(tw.TwError) as ei:
        fn(*a)
    return ei.value.status


def test_bind_argument_errors_need_no_device():
    g = wl.same_geom(4, 3, 3, 1, 6, 6)
    K, N, G = g.K, 64, 64
    p = tw.tw_pack_host(np.ones((K, N), np.float16), np.ones((K, N), np.uint8), G, tw.PATTERN_TW)
    ldx = wl.conv_ldx(g)
    assert _status(tw.tw_conv_bind, p, g, ldx) == 6                         # not uploaded
    assert _status(tw.tw_conv_bind, p, g, ldx - 8) == 1                     # windows would leave the row
    assert _status(tw.tw_conv_bind, p, wl.ConvGeom(4, 3, 3, 1, 6, 6, 7, 8), ldx) == 1     # P < W+S-1
    assert _status(tw.tw_conv_bind, p, wl.ConvGeom(4, 3, 3, 1, 6, 6, 8, 7), ldx) == 1     # L < H+R-1
    assert _status(tw.tw_conv_bind, p, wl.same_geom(5, 3, 3, 1, 6, 6), ldx) == 1          # K != C*R*S
    p32 = tw.tw_pack_host(np.ones((K, 32), np.float16), np.ones((K, 32), np.uint8), 32, tw.PATTERN_TW)
    assert _status(tw.tw_conv_bind, p32, g, ldx) == 3                       # G = 32
    p8 = tw.tw_pack_i8_host(np.ones((K, N), np.int8), np.ones((K, N), np.uint8), G)
    assert _status(tw.tw_conv_bind, p8, g, wl.conv_ldx(g, 16)) == 6         # int8 binds too, once uploaded
    assert _status(tw.tw_conv_bind, p8, g, wl.conv_ldx(g, 16) + 8) == 1     # int8 rows: multiples of 16
    assert tw.lib().tw_conv_gemm(0x10000, None, 0x20000, 64, None) == 1     # a launch needs a binding
    assert tw.lib().tw_conv_free(None) == 0
    for q in (p, p32, p8):
        q.free()


def _check(g, N, G, pattern, seed, tile_m=0, ldc=None):
    from tests import gpu_util as gu
    rng = np.random.default_rng(seed)
    X = wl.make_conv_input(seed, g)
    Bw = wl.rng_fp16(seed + 1, (g.K, N), 0.05)
    if pattern == "tw":
        mask = tmask = random_tw_mask(rng, g.K, N, G, col_keep=0.85, row_keep=0.4)
        p = tw.tw_pack(Bw, mask, G, tw.PATTERN_TW)
    else:
        mask, tmask = random_tvw_mask(rng, g.K, N, G, col_keep=0.85, row_keep=0.5)
        p = tw.tw_pack(Bw, mask, G, tw.PATTERN_TVW, tile_mask=tmask)
    print(f"conv {pattern} C={g.C} {g.R}x{g.S} B={g.B} {g.H}x{g.W} P={g.P} L={g.L} N={N} G={G} tile_m={tile_m}",
          flush=True)
    tw.tw_set_option("tile_m", tile_m)
    try:
        Cw, raw = gu.run_conv(tw, p, X, g, N, ldc=ldc, fill=7.0)
    finally:
        tw.tw_set_option("tile_m", 0)
        p.free()
    assert_C_close(Cw, oc.conv_wide_oracle(X, Bw, mask, **g.ints()), oc.conv_wide_abs_bound(X, Bw, mask, **g.ints()))
    valid = oc.valid_positions(B=g.B, H=g.H, W=g.W, P=g.P, L=g.L)
    assert (raw[:, :g.Mp][:, ~valid].view(np.uint16) == 0).all()            # padding lanes: +0
    assert (raw[:, g.Mp:] == 7.0).all()                                     # beyond the grid: untouched
    return Cw


@pytest.mark.gpu
@pytest.mark.parametrize("pattern", ["tw", "tvw"])
@pytest.mark.parametrize("G,tile_m", [(64, 128), (128, 64), (128, 128), (128, 256)])
def test_conv3x3_parity(pattern, G, tile_m):
    if pattern == "tvw" and G == 64 and tile_m != 128:
        pytest.skip("one TVW instance for G = 64")
    g = wl.same_geom(24, 3, 3, 2, 13, 11)                    # Mp = 2*15*13 = 390: several M-tiles, ragged
    _check(g, 150, G, pattern, 100 + G + tile_m, tile_m, ldc=400)


@pytest.mark.gpu
@pytest.mark.parametrize("R,S,pitch", [(1, 1, 1), (5, 3, 1), (3, 3, 8), (1, 7, 1)])
def test_conv_other_filters_and_pitches(R, S, pitch):
    g = wl.same_geom(16, R, S, 3, 9, 10, pitch)
    _check(g, 130, 128, "tw", 7 * R + S + pitch)


@pytest.mark.gpu
def test_conv_equals_the_launch_on_the_materialised_matrix():
    """The same handle on the explicit img2col matrix (tw_gemm) and on the wide input
    (tw_conv_gemm): same products in the same order, so the valid positions agree bit for bit."""
    from tests import gpu_util as gu
    g = wl.same_geom(32, 3, 3, 2, 12, 12)
    N, G = 128, 128
    rng = np.random.default_rng(5)
    X = wl.make_conv_input(5, g)
    Bw = wl.rng_fp16(6, (g.K, N), 0.05)
    mask = random_tw_mask(rng, g.K, N, G)
    p = tw.tw_pack(Bw, mask, G, tw.PATTERN_TW)
    A = oc.im2col_wide(X, **g.ints())                                      # layout only, no arithmetic
    _, raw_gemm = gu.run_tw(tw, p, A, N)
    _, raw_conv = gu.run_conv(tw, p, X, g, N)
    p.free()
    assert np.array_equal(raw_gemm[:, :g.Mp].view(np.uint16), raw_conv[:, :g.Mp].view(np.uint16))


@pytest.mark.gpu
@pytest.mark.parametrize("layer,G", [(1, 64), (1, 128), (0, 128)])
def test_conv_vgg_layer_on_sampled_positions(layer, G):
    """The configured 3x3 layers at full size (512 -> 512 at 14 x 14 and 256 -> 256 at 56 x 56, batch
    8; the launch configuration the benchmark times), checked on sampled positions the oracle computes
    one by one."""
    from tests import gpu_util as gu
    name, g, N = wl.CONV_LAYERS[layer]
    X = wl.make_conv_input(11, g)
    Bw = wl.make_B(12, g.K, N, 0.02)
    mask = wl.tw_mask(Bw, G, density=0.25, col_frac=0.10)
    p = tw.tw_pack(Bw, mask, G, tw.PATTERN_TW)
    print(f"conv {name} Mp={g.Mp} G={G}", flush=True)
    Cw, raw = gu.run_conv(tw, p, X, g, N)
    p.free()
    valid = np.flatnonzero(oc.valid_positions(B=g.B, H=g.H, W=g.W, P=g.P, L=g.L))
    rng = np.random.default_rng(13)
    pos = np.concatenate([valid[:3], valid[-3:], rng.choice(valid, 58, replace=False)])
    A_rows = oc.im2col_wide(X, rows=pos, **g.ints())             # those rows of the img2col matrix
    assert_C_close(Cw[pos], og.gemm_oracle(A_rows, Bw, mask), og.abs_bound(A_rows, Bw, mask))
    inval = ~oc.valid_positions(B=g.B, H=g.H, W=g.W, P=g.P, L=g.L)
    assert (raw[:, :g.Mp][:, inval].view(np.uint16) == 0).all()


@pytest.mark.gpu
@pytest.mark.parametrize("pattern", ["tw", "tvw"])
@pytest.mark.parametrize("G,tile_m,c_dtype", [(128, 128, 0), (128, 64, 1), (64, 128, 1), (128, 256, 0)])
def test_conv_int8_parity(pattern, G, tile_m, c_dtype):
    """int8 input and weight: the img2col GEMM over integers, bit for bit, int32 or requantised."""
    from tests import gpu_util as gu
    g = wl.same_geom(24, 3, 3, 2, 13, 11)
    N = 150
    rng = np.random.default_rng(300 + G + tile_m + c_dtype)
    X = wl.make_conv_input(20, g, int8=True)
    Bw = wl.rng_i8(21, (g.K, N))
    if pattern == "tw":
        mask = tmask = random_tw_mask(rng, g.K, N, G, col_keep=0.85, row_keep=0.4)
    else:
        mask, tmask = random_tvw_mask(rng, g.K, N, G, col_keep=0.85, row_keep=0.5)
    scale = 1.0 / 700.0
    print(f"conv int8 {pattern} G={G} tile_m={tile_m} c_dtype={c_dtype}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack_i8(Bw, mask, G, tw.PATTERN_TVW if pattern == "tvw" else tw.PATTERN_TW,
                      tile_mask=tmask if pattern == "tvw" else None)
    try:
        Cw, raw = gu.run_conv_i8(tw, p, X, g, N, c_dtype=c_dtype, scale=scale)
    finally:
        tw.tw_set_option("tile_m", 0)
        p.free()
    want = og.gemm_i8_oracle(oc.im2col_wide(X, **g.ints()), Bw, mask)
    if c_dtype:
        want = og.requantize_i8(want, scale).astype(np.int64)
    assert np.abs(want).max() > 20
    assert np.array_equal(Cw, want)
    valid = oc.valid_positions(B=g.B, H=g.H, W=g.W, P=g.P, L=g.L)
    assert (raw[:, :g.Mp][:, ~valid] == 0).all()
    assert (raw[:, g.Mp:] == -77).all()
