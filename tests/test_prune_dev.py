"""Device-side one-shot pruner (tw_prune_dev) against the oracle's Algorithm 3 with exact
integer scores, and the device-to-handle path (tw_pack_dev)."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from oracle import prune as op
from tests.helpers import assert_C_close
import workloads as wl


def test_workspace_size_and_argument_errors():
    n = tw.tw_prune_workspace_bytes(768, 3072, 128)
    assert n >= 24 * 768 * 28 and n % 256 == 0
    with pytest.raises(tw.TwError) as ei:
        tw.tw_prune_workspace_bytes(0, 8, 128)
    assert ei.value.status == 1
    dummy = 4096                                   # never dereferenced: every call below fails its checks first
    bad = [dict(K=0), dict(N=0), dict(ldb=7), dict(G=48), dict(n_cols_pruned=9), dict(rows_per_tile=9),
           dict(n_cols_pruned=-1), dict(pattern=7), dict(workspace_bytes=16)]
    for kw in bad:
        a = dict(B_ptr=dummy, K=8, N=8, ldb=8, G=32, pattern=tw.PATTERN_TW, n_cols_pruned=1, rows_per_tile=4,
                 mask_ptr=dummy, tile_mask_ptr=None, workspace_ptr=dummy, workspace_bytes=1 << 20)
        a.update(kw)
        with pytest.raises(tw.TwError) as ei:
            tw.tw_prune_dev(**a)
        assert ei.value.status == 1, kw
    a = dict(B_ptr=dummy, K=8, N=8, ldb=8, G=32, pattern=tw.PATTERN_TEW, n_cols_pruned=1, rows_per_tile=4,
             mask_ptr=dummy, tile_mask_ptr=None, workspace_ptr=dummy, workspace_bytes=1 << 20)
    with pytest.raises(tw.TwError) as ei:
        tw.tw_prune_dev(**a)
    assert ei.value.status == 3


def _prune_on_device(B, G, pattern, n_cols_pruned, rows_per_tile, ldb=None, want_tile_mask=True):
    import torch
    K, N = B.shape
    ldb = ldb or N
    Bp = np.full((K, ldb), 7.0, np.float16)
    Bp[:, :N] = B
    Bd = torch.from_numpy(Bp).cuda()
    mask = torch.full((K, N), 9, dtype=torch.uint8, device="cuda")
    tmask = torch.full((K, N), 9, dtype=torch.uint8, device="cuda") if want_tile_mask else None
    ws = torch.empty(tw.tw_prune_workspace_bytes(K, N, G), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    tw.tw_prune_dev(Bd.data_ptr(), K, N, ldb, G, pattern, n_cols_pruned, rows_per_tile, mask.data_ptr(),
                    tmask.data_ptr() if want_tile_mask else None, ws.data_ptr(), ws.numel(), st)
    torch.cuda.synchronize()
    return mask.cpu().numpy(), (tmask.cpu().numpy() if want_tile_mask else None), (Bd, mask, tmask)


@pytest.mark.gpu
@pytest.mark.parametrize("seed,K,N,G,cp,rk", [(0, 40, 36, 32, 4, 10), (1, 33, 150, 64, 0, 7), (2, 64, 70, 32, 9, 16),
                                               (3, 100, 300, 128, 41, 28), (4, 7, 5, 32, 5, 3), (5, 50, 64, 64, 0, 50),
                                               (6, 30, 90, 32, 3, 0)])
def test_tw_mask_equals_oracle(seed, K, N, G, cp, rk):
    B = wl.rng_fp16(seed, (K, N))
    print(f"case prune tw seed={seed}", flush=True)
    mask, tmask, _ = _prune_on_device(B, G, tw.PATTERN_TW, cp, rk, ldb=N + 8)
    want = op.tw(B, G, n_cols_pruned=cp, rows_kept_per_tile=rk, exact=True)
    assert np.array_equal(mask, want) and np.array_equal(tmask, want)


@pytest.mark.gpu
@pytest.mark.parametrize("seed,K,N,G,cp,rk", [(0, 40, 36, 32, 4, 12), (1, 64, 150, 64, 10, 20), (2, 33, 70, 32, 0, 30),
                                               (3, 100, 200, 128, 20, 28)])
def test_tvw_mask_equals_oracle(seed, K, N, G, cp, rk):
    B = wl.rng_fp16(10 + seed, (K, N))
    B[:8, :] = np.float16(0.5) * np.sign(B[:8, :]).astype(np.float16)                # equal magnitudes: tie rule
    print(f"case prune tvw seed={seed}", flush=True)
    mask, tmask, _ = _prune_on_device(B, G, tw.PATTERN_TVW, cp, rk)
    want_tm = op.tw(B, G, n_cols_pruned=cp, rows_kept_per_tile=rk, exact=True)
    assert np.array_equal(tmask, want_tm)
    assert np.array_equal(mask, op.vw24_condensed(B, want_tm, G))
    mask2, _, _ = _prune_on_device(B, G, tw.PATTERN_TVW, cp, rk, want_tile_mask=False)
    assert np.array_equal(mask2, mask)


@pytest.mark.gpu
def test_equal_scores_lose_the_lower_index_first():
    B = np.ones((12, 40), np.float16)
    mask, _, _ = _prune_on_device(B, 32, tw.PATTERN_TW, 5, 4)
    want = np.zeros((12, 40), np.uint8)
    want[8:, 5:] = 1                       # columns 0..4 and rows 0..7 of every tile go
    assert np.array_equal(mask, want)
    assert np.array_equal(mask, op.tw(B, 32, n_cols_pruned=5, rows_kept_per_tile=4, exact=True))


@pytest.mark.gpu
def test_decision_that_needs_exact_sums():
    """One large and many tiny values against the large value alone: an fp64 running sum cannot
    tell the two columns apart, the exact scores can."""
    K = 40
    B = np.zeros((K, 2), np.float16)
    B[0, :] = 64.0
    B[1:, 0] = 2.0 ** -24
    mask, _, _ = _prune_on_device(B, 32, tw.PATTERN_TW, 1, K)
    assert mask[:, 0].all() and not mask[:, 1].any()


@pytest.mark.gpu
@pytest.mark.parametrize("pattern", ["tw", "tvw"])
def test_bert_base_shape_equals_the_workload_generator_and_multiplies(pattern):
    """768 x 3072 at the configured sparsity: the device mask equals the seeded generator's
    (same recipe, fp64 scores: no near-ties in this data), and prune -> pack -> multiply, all
    from device buffers, matches the oracle on sampled rows."""
    import torch
    from tests import gpu_util as gu
    c = wl.make_case(2 if pattern == "tw" else 3, 1, M=256)
    n_cols_pruned = int(np.floor(0.10 * c.N))
    rows = int(c.tile_mask[:, c.tile_mask.any(0)][:, 0].sum())
    pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
    print(f"case prune {c.name} rows_per_tile={rows}", flush=True)
    mask, tmask, (Bd, md, tmd) = _prune_on_device(c.B, c.G, pat, n_cols_pruned, rows)
    assert np.array_equal(tmask, c.tile_mask) and np.array_equal(mask, c.mask)
    p = tw.tw_pack_dev(Bd.data_ptr(), c.N, md.data_ptr(), tmd.data_ptr() if pattern == "tvw" else None,
                       c.K, c.N, c.G, pat, torch.cuda.current_stream().cuda_stream)
    C, _ = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    assert_C_close(C, og.gemm_oracle(c.A, c.B, c.mask), og.abs_bound(c.A, c.B, c.mask))
