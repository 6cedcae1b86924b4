"""tw_concat: weights packed one by one and placed side by side along N behave as
the weight [B_0 | B_1 | ...] with the mask [mask_0 | mask_1 | ...]; the host
part runs without a GPU, the product is compared with the oracle on the GPU."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from oracle import pack as opk
from tests.helpers import assert_C_close, random_tw_mask, random_tvw_mask
import workloads as wl


def _members(seed, K, Ns, G, pattern):
    rng = np.random.default_rng(seed)
    out = []
    for i, N in enumerate(Ns):
        B = wl.make_B(seed * 10 + i, K, N, 1.0)
        if pattern == "tw":
            mask = random_tw_mask(rng, K, N, G, col_keep=rng.uniform(0.5, 1.0), row_keep=rng.uniform(0.2, 0.9))
            tm = None
        else:
            mask, tm = random_tvw_mask(rng, K, N, G, full=bool(i % 2))
        out.append((B, mask, tm))
    return out


@pytest.mark.parametrize("pattern", ["tw", "tvw"])
@pytest.mark.parametrize("seed", range(4))
def test_concat_host_is_the_side_by_side_weight(seed, pattern):
    rng = np.random.default_rng(100 + seed)
    K = int(rng.integers(1, 120))
    Ns = [int(n) for n in rng.integers(1, 200, size=int(rng.integers(1, 5)))]
    G = int(rng.choice([32, 64, 128]))
    pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
    mem = _members(seed, K, Ns, G, pattern)
    parts = [tw.tw_pack_host(B, m, G, pat, tile_mask=t) for B, m, t in mem]
    cat = tw.tw_concat(parts, upload=False)
    Bm, m2 = cat.unpack()
    B_all = np.concatenate([B for B, _, _ in mem], axis=1)
    m_all = np.concatenate([m for _, m, _ in mem], axis=1)
    assert np.array_equal(m2, m_all)
    assert np.array_equal(Bm, np.where(m_all != 0, B_all.view(np.uint16), 0))
    # the members' tiles, one after the other, with shifted columns
    e = cat.export()
    refs = [opk.ref_pack(B, m, G, pat, tile_mask=t) for B, m, t in mem]
    assert e["n_tiles"] == sum(r["n_tiles"] for r in refs)
    assert e["n_kept"] == sum(r["n_kept"] for r in refs)
    t0, n0, c0 = 0, 0, 0
    for r in refs:
        assert np.array_equal(e["col_idx"][c0:c0 + r["n_kept"]], r["col_idx"] + n0)
        for t in range(r["n_tiles"]):
            assert e["tile_col_off"][t0 + t] == c0 + min(t * G, r["n_kept"])
            assert np.array_equal(e["row_idx"][t0 + t], r["row_idx"][t])
            assert np.array_equal(e["values"][t0 + t], r["values"][t])
            if pattern == "tvw":
                assert np.array_equal(e["meta"][t0 + t], r["meta"][t])
                assert np.array_equal(e["valid"][t0 + t], r["valid"][t])
        t0 += r["n_tiles"]; n0 += r["N"]; c0 += r["n_kept"]
    assert e["tile_col_off"][-1] == e["n_kept"]
    assert np.array_equal(e["cto_n"], e["col_idx"] - np.arange(e["n_kept"]))
    skw, sk, ku = cat.flop_counts()
    assert skw == sum(p.flop_counts()[0] for p in parts)
    used = np.concatenate([(t if t is not None else m) for _, m, t in mem], axis=1).any(axis=1)
    assert ku == int(used.sum())
    for p in parts + [cat]:
        p.free()


def test_concat_rejects_mismatched_members():
    B = wl.make_B(1, 40, 64, 1.0)
    m = np.ones((40, 64), np.uint8)
    a = tw.tw_pack_host(B, m, 32, tw.PATTERN_TW)
    b = tw.tw_pack_host(B, m, 64, tw.PATTERN_TW)
    c = tw.tw_pack_host(B[:20], m[:20], 32, tw.PATTERN_TW)
    for parts in ([a, b], [a, c], []):
        with pytest.raises(tw.TwError) as ei:
            tw.tw_concat(parts, upload=False)
        assert ei.value.status == 1
    for p in (a, b, c):
        p.free()


@pytest.mark.gpu
@pytest.mark.parametrize("pattern,G,tile_m", [("tw", 128, 0), ("tw", 64, 128), ("tw", 128, 64), ("tvw", 128, 0), ("tvw", 64, 0)])
def test_concat_gemm_matches_oracle(pattern, G, tile_m):
    from tests import gpu_util as gu
    print(f"concat {pattern} G={G} tile_m={tile_m}", flush=True)
    M, K, Ns = 200, 260, [150, 300, 77]
    pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
    mem = _members(7, K, Ns, G, pattern)
    parts = [tw.tw_pack_host(B, m, G, pat, tile_mask=t) for B, m, t in mem]
    cat = tw.tw_concat(parts)
    A = wl.make_A(3, M, K)
    tw.tw_set_option("tile_m", tile_m)
    try:
        C, raw = gu.run_tw(tw, cat, A, sum(Ns))
    finally:
        tw.tw_set_option("tile_m", 0)
    B_all = np.concatenate([B for B, _, _ in mem], axis=1)
    m_all = np.concatenate([m for _, m, _ in mem], axis=1)
    assert_C_close(C, og.gemm_oracle(A, B_all, m_all), og.abs_bound(A, B_all, m_all))
    # member i's rows of C^T are what its own handle gives, bit for bit
    n0 = 0
    for (B, m, t), p, N in zip(mem, parts, Ns):
        p.upload()
        tw.tw_set_option("tile_m", tile_m)
        try:
            _, raw_i = gu.run_tw(tw, p, A, N)
        finally:
            tw.tw_set_option("tile_m", 0)
        assert np.array_equal(raw[n0:n0 + N, :M].view(np.uint16), raw_i[:, :M].view(np.uint16))
        n0 += N
    for p in parts + [cat]:
        p.free()
