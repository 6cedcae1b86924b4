"""Host side of the C ABI (no GPU): the library loads, exports every declared
symbol, and its packer agrees bit for bit with the oracle's canonical form."""
import ctypes as C
import re
import os

import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import pack as opk
from tests.helpers import random_tw_mask, random_tvw_mask
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "twgemm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(tw_[a-z0-9_]+)\s*\(", header)))
    assert declared == sorted(tw.EXPORTED_SYMBOLS)
    L = C.CDLL(tw.lib_path())
    for name in declared:
        assert getattr(L, name) is not None


def test_header_is_plain_c(tmp_path):
    """include/twgemm.h is the boundary: it must compile as C99 on its own, warnings as errors."""
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "twgemm.h"\nint main(void) { tw_conv_geom g = {1, 1, 1, 1, 1, 1, 1, 1}; tw_packed_view v;\n'
                   '  (void)g; (void)v; return (int)TW_OK; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I" + os.path.join(ROOT, "include"),
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def _same(e, r):
    assert e["n_kept"] == r["n_kept"] and e["n_tiles"] == r["n_tiles"]
    assert np.array_equal(e["col_idx"], r["col_idx"])
    assert np.array_equal(e["cto_n"], r["cto_n"])
    for t in range(r["n_tiles"]):
        assert np.array_equal(e["row_idx"][t], r["row_idx"][t])
        assert np.array_equal(e["cto_k"][t], r["cto_k"][t])
        assert np.array_equal(e["values"][t], r["values"][t])
        if r["pattern"] == opk.PATTERN_TVW:
            assert np.array_equal(e["meta"][t], r["meta"][t])
            assert np.array_equal(e["valid"][t], r["valid"][t])


@pytest.mark.parametrize("seed", range(8))
def test_tw_export_equals_oracle_pack(seed):
    rng = np.random.default_rng(seed)
    K, N = int(rng.integers(1, 90)), int(rng.integers(1, 200))
    G = int(rng.choice([32, 64, 128]))
    mask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.3, 1.0), row_keep=rng.uniform(0.1, 1.0))
    B = wl.rng_fp16(seed, (K, N))
    p = tw.tw_pack_host(B, mask, G, tw.PATTERN_TW)
    _same(p.export(), opk.ref_pack(B, mask, G, opk.PATTERN_TW))
    Bm, m2 = p.unpack()
    assert np.array_equal(m2, mask)
    assert np.array_equal(Bm, np.where(mask != 0, B.view(np.uint16), 0))
    skw, sk, ku = p.flop_counts()
    assert skw == int(mask.sum()) and sk == sum(len(r) for r in p.export()["row_idx"])
    assert ku == int(mask.any(axis=1).sum())
    p.free()


@pytest.mark.parametrize("seed,full,with_tm", [(0, True, True), (1, True, True), (2, False, True),
                                                (3, False, True), (4, True, False), (5, True, True)])
def test_tvw_export_equals_oracle_pack(seed, full, with_tm):
    rng = np.random.default_rng(100 + seed)
    K, N = int(rng.integers(4, 120)), int(rng.integers(1, 200))
    G = int(rng.choice([32, 64, 128]))
    mask, tm = random_tvw_mask(rng, K, N, G, full=full)
    B = wl.rng_fp16(seed, (K, N))
    if not with_tm:
        # without the TW-level mask the structure is derived from the element mask
        # itself; only usable when that derivation is conformant
        try:
            r = opk.ref_pack(B, mask, G, opk.PATTERN_TVW)
        except opk.MaskError:
            with pytest.raises(tw.TwError):
                tw.tw_pack_host(B, mask, G, tw.PATTERN_TVW)
            return
        p = tw.tw_pack_host(B, mask, G, tw.PATTERN_TVW)
    else:
        r = opk.ref_pack(B, mask, G, opk.PATTERN_TVW, tile_mask=tm)
        p = tw.tw_pack_host(B, mask, G, tw.PATTERN_TVW, tile_mask=tm)
    _same(p.export(), r)
    Bm, m2 = p.unpack()
    assert np.array_equal(m2, mask)
    assert np.array_equal(Bm, np.where(mask != 0, B.view(np.uint16), 0))
    p.free()


def test_worked_example_through_the_c_abi(golden_dir):
    # Section V: tiles keep rows (1,2,4) and (0,3); offsets (1,1,2) and (0,2)
    K, G = 5, 32
    mask = np.zeros((K, 2 * G), np.uint8)
    mask[[1, 2, 4], :G] = 1
    mask[[0, 3], G:] = 1
    p = tw.tw_pack_host(wl.rng_fp16(0, mask.shape), mask, G, tw.PATTERN_TW)
    e = p.export()
    assert [r.tolist() for r in e["row_idx"]] == [[1, 2, 4], [0, 3]]
    assert [r.tolist() for r in e["cto_k"]] == [[1, 1, 2], [0, 2]]
    p.free()


def test_configured_workloads_pack_bit_exactly():
    for cfg, pat in ((1, "tw"), (2, "tw"), (3, "tvw")):
        c = wl.make_case(cfg, 0, with_A=False)
        pattern = tw.PATTERN_TW if pat == "tw" else tw.PATTERN_TVW
        tm = c.tile_mask if pat == "tvw" else None
        p = tw.tw_pack_host(c.B, c.mask, c.G, pattern, tile_mask=tm)
        _same(p.export(), opk.ref_pack(c.B, c.mask, c.G, pattern, tile_mask=tm))
        p.free()


def test_error_codes():
    B = wl.rng_fp16(0, (8, 8))
    ones = np.ones((8, 8), np.uint8)
    with pytest.raises(tw.TwError) as e:
        tw.tw_pack_host(B, ones, 48, tw.PATTERN_TW)           # bad G
    assert e.value.status == 1
    with pytest.raises(tw.TwError) as e:
        tw.tw_pack_host(B, ones, 32, 7)                       # bad pattern
    assert e.value.status == 1
    holed = ones.copy(); holed[3, 2] = 0
    with pytest.raises(tw.TwError) as e:
        tw.tw_pack_host(B, holed, 32, tw.PATTERN_TW)
    assert e.value.status == 2
    with pytest.raises(tw.TwError) as e:                      # 4 of 4 kept in a group
        tw.tw_pack_host(B, ones, 32, tw.PATTERN_TVW)
    assert e.value.status == 2
    L = tw.lib()
    assert L.tw_pack_host(None, None, None, 8, 8, 32, 0, C.byref(C.c_void_p())) == 1
    assert L.tw_free(None) == 0
    assert L.tw_status_str(2) == b"mask is not TW/TVW conformant"
    # gemm on a handle that was never uploaded
    p = tw.tw_pack_host(B, ones, 32, tw.PATTERN_TW)
    assert L.tw_gemm(C.c_void_p(256), 8, 8, 0, p.handle, C.c_void_p(512), 8, None) == 6
    assert L.tw_gemm(C.c_void_p(256), 8, 7, 0, p.handle, C.c_void_p(512), 8, None) == 1   # lda % 8
    assert L.tw_gemm(C.c_void_p(258), 8, 8, 0, p.handle, C.c_void_p(512), 8, None) == 1   # alignment
    p.free()
    with pytest.raises(tw.TwError):
        tw.tw_set_option("no_such_knob", 1)


def test_empty_and_full_masks():
    B = wl.rng_fp16(0, (6, 70))
    p = tw.tw_pack_host(B, np.zeros((6, 70), np.uint8), 32, tw.PATTERN_TW)
    e = p.export()
    assert e["n_kept"] == 0 and e["n_tiles"] == 0
    p.free()
    p = tw.tw_pack_host(B, np.ones((6, 70), np.uint8), 32, tw.PATTERN_TW)
    e = p.export()
    assert e["n_tiles"] == 3 and [v.shape for v in e["values"]] == [(6, 32), (6, 32), (6, 6)]
    p.free()
