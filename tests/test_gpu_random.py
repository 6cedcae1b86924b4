"""Seeded random cases over every launch entry point (-m gpu): shapes, tile widths, patterns,
leading dimensions and tuning options drawn together, each case checked against the oracle.
The targeted tests cover the corners one at a time; this one covers their combinations."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import conv as oc
from oracle import gemm as og
from tests import gpu_util as gu
from tests.helpers import assert_C_close, random_tw_mask, random_tvw_mask
import workloads as wl

pytestmark = pytest.mark.gpu

OPTS = (("tile_m", 0), ("xcd_map", 1), ("kernel", 0), ("depth", 3), ("waves", 4), ("ksplit", 0))


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    for k, v in OPTS:
        tw.tw_set_option(k, v)


def _draw_options(rng):
    o = dict(tile_m=int(rng.choice([0, 64, 128, 256])), xcd_map=int(rng.integers(0, 3)),
             depth=int(rng.choice([3, 4])), waves=int(rng.choice([4, 8])), ksplit=int(rng.integers(0, 3)))
    for k, v in o.items():
        tw.tw_set_option(k, v)
    return o


@pytest.mark.parametrize("seed", range(24))
def test_random_fp16_case(seed):
    rng = np.random.default_rng(9000 + seed)
    M, K, N = int(rng.integers(1, 700)), int(rng.integers(1, 900)), int(rng.integers(1, 600))
    G = int(rng.choice([32, 64, 128]))
    pattern = str(rng.choice(["tw", "tvw", "tew"]))
    A, B = wl.make_A(seed, M, K), wl.make_B(seed, K, N, 1.0)
    if pattern == "tw":
        mask = tmask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.05, 1.0))
        pat = tw.PATTERN_TW
    elif pattern == "tvw":
        mask, tmask = random_tvw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.1, 1.0),
                                      full=bool(rng.integers(0, 2)))
        pat = tw.PATTERN_TVW
    else:
        tmask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.05, 1.0))
        mask = (tmask | (rng.random((K, N)) < 0.01)).astype(np.uint8)
        pat = tw.PATTERN_TEW
    o = _draw_options(rng)
    lda = (M + 7) // 8 * 8 + 8 * int(rng.integers(0, 3))
    ldc = (M + 7) // 8 * 8 + 8 * int(rng.integers(0, 3))
    print(f"random fp16 seed={seed} {pattern} M={M} K={K} N={N} G={G} lda={lda} ldc={ldc} {o}", flush=True)
    p = tw.tw_pack(B, mask, G, pat, tile_mask=None if pattern == "tw" else tmask)
    try:
        C, raw = gu.run_tw(tw, p, A, N, lda=lda, ldc=ldc, fill=3.0)
    except tw.TwError as e:
        assert e.status == 3 and pattern != "tw" and G == 32, e     # TVW / TEW have no kernel for G = 32
        return
    finally:
        p.free()
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    assert (raw[:, M:] == 3.0).all()


@pytest.mark.parametrize("seed", range(12))
def test_random_int8_case(seed):
    rng = np.random.default_rng(9100 + seed)
    M, K, N = int(rng.integers(1, 700)), int(rng.integers(1, 900)), int(rng.integers(1, 600))
    G = int(rng.choice([64, 128]))
    tvw = bool(rng.integers(0, 2))
    A, B = wl.rng_i8(seed, (M, K)), wl.rng_i8(seed + 1, (K, N))
    if tvw:
        mask, tmask = random_tvw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.1, 1.0),
                                      full=bool(rng.integers(0, 2)))
    else:
        mask = tmask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.05, 1.0))
    c_dtype = int(rng.integers(0, 2))
    scale = float(np.float32(rng.uniform(1e-4, 1e-2)))
    tile_m = int(rng.choice([0, 64, 128, 256]))
    lda = (M + 15) // 16 * 16 + 16 * int(rng.integers(0, 2))
    ldc = (M + 15) // 16 * 16 + 16 * int(rng.integers(0, 2))
    print(f"random int8 seed={seed} tvw={tvw} M={M} K={K} N={N} G={G} c_dtype={c_dtype} tile_m={tile_m}", flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack_i8(B, mask, G, tw.PATTERN_TVW if tvw else tw.PATTERN_TW, tile_mask=tmask if tvw else None)
    try:
        C, raw = gu.run_tw_i8(tw, p, A, N, c_dtype=c_dtype, scale=scale, lda=lda, ldc=ldc)
    except tw.TwError as e:
        assert e.status == 3 and tile_m in (64, 256), e      # forced tile height without an instance
        return
    finally:
        p.free()
    want = og.gemm_i8_oracle(A, B, mask)
    if c_dtype:
        want = og.requantize_i8(want, scale).astype(np.int64)
    assert np.array_equal(C, want)
    assert (raw[:, M:] == -77).all()


@pytest.mark.parametrize("seed", range(8))
def test_random_conv_case(seed):
    rng = np.random.default_rng(9200 + seed)
    R, S = int(rng.choice([1, 3, 5])), int(rng.choice([1, 3, 5]))
    g = wl.same_geom(int(rng.integers(1, 40)), R, S, int(rng.integers(1, 4)), int(rng.integers(1, 20)),
                     int(rng.integers(1, 20)), int(rng.choice([1, 4, 8])))
    N, G = int(rng.integers(1, 300)), int(rng.choice([64, 128]))
    tvw = bool(rng.integers(0, 2))
    X, Bw = wl.make_conv_input(seed, g), wl.rng_fp16(seed + 1, (g.K, N), 0.1)
    if tvw:
        mask, tmask = random_tvw_mask(rng, g.K, N, G, col_keep=0.8, row_keep=0.6)
    else:
        mask = tmask = random_tw_mask(rng, g.K, N, G, col_keep=0.8, row_keep=0.5)
    tile_m = int(rng.choice([0, 64, 128]))
    print(f"random conv seed={seed} tvw={tvw} C={g.C} {R}x{S} B={g.B} {g.H}x{g.W} P={g.P} N={N} G={G} tile_m={tile_m}",
          flush=True)
    tw.tw_set_option("tile_m", tile_m)
    p = tw.tw_pack(Bw, mask, G, tw.PATTERN_TVW if tvw else tw.PATTERN_TW, tile_mask=tmask if tvw else None)
    try:
        Cw, raw = gu.run_conv(tw, p, X, g, N, fill=5.0)
    finally:
        p.free()
    assert_C_close(Cw, oc.conv_wide_oracle(X, Bw, mask, **g.ints()), oc.conv_wide_abs_bound(X, Bw, mask, **g.ints()))
    valid = oc.valid_positions(B=g.B, H=g.H, W=g.W, P=g.P, L=g.L)
    assert (raw[:, :g.Mp][:, ~valid].view(np.uint16) == 0).all()
    assert (raw[:, g.Mp:] == 5.0).all()
