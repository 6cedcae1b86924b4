"""tw_prune_dev_static (the entry point that allocates nothing: its scratch is a fixed device array
inside the library) against tw_prune_dev with a caller workspace, bit for bit, on two calls in a
row, the second on a smaller input that leaves the first call's contents in most of the array."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
import workloads as wl


def test_static_entry_point_rejects_what_does_not_fit():
    dummy = 4096                          # never dereferenced: the size check comes first
    with pytest.raises(tw.TwError) as ei:
        tw.tw_prune_dev_static(dummy, 8192, 8192, 8192, 32, tw.PATTERN_TW, 0, 8192, dummy, None)
    assert ei.value.status == 7 and "static scratch" in str(ei.value)
    with pytest.raises(tw.TwError) as ei:
        tw.tw_prune_dev_static(dummy, 8, 8, 7, 32, tw.PATTERN_TW, 0, 8, dummy, None)
    assert ei.value.status == 1


def _both(B, G, pattern, cp, rk):
    import torch
    K, N = B.shape
    Bd = torch.from_numpy(B).cuda()
    st = torch.cuda.current_stream().cuda_stream
    out = []
    for static in (False, True):
        mask = torch.full((K, N), 9, dtype=torch.uint8, device="cuda")
        tmask = torch.full((K, N), 9, dtype=torch.uint8, device="cuda")
        if static:
            tw.tw_prune_dev_static(Bd.data_ptr(), K, N, N, G, pattern, cp, rk, mask.data_ptr(), tmask.data_ptr(), st)
        else:
            ws = torch.empty(tw.tw_prune_workspace_bytes(K, N, G), dtype=torch.uint8, device="cuda")
            tw.tw_prune_dev(Bd.data_ptr(), K, N, N, G, pattern, cp, rk, mask.data_ptr(), tmask.data_ptr(),
                            ws.data_ptr(), ws.numel(), st)
        torch.cuda.synchronize()
        out.append((mask.cpu().numpy(), tmask.cpu().numpy()))
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("pattern", ["tw", "tvw"])
def test_static_scratch_equals_workspace_twice_in_a_row(pattern):
    pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
    for seed, K, N, G, cp, rk in [(1, 768, 1000, 128, 100, 212), (2, 100, 300, 64, 41, 28)]:   # large, then small
        print(f"case static prune {pattern} K={K} N={N} G={G}", flush=True)
        B = wl.rng_fp16(seed, (K, N))
        (m0, t0), (m1, t1) = _both(B, G, pat, cp, rk)
        assert np.array_equal(m0, m1) and np.array_equal(t0, t1)
        assert m1.max() == 1 and m1.sum() > 0
        kept_cols = t1.any(0).sum()
        assert kept_cols == N - cp and (t1.sum(0)[t1.any(0)] == rk).all()
