"""Seeded random shapes, masks and launch options through tw_gemm_ex against the oracle (-m gpu):
combinations of tile height, index route, K split, pipeline depth and tiles per workgroup that the
targeted tests do not pair up, on ragged shapes down to a single row, column or kept element."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import gemm as og
from tests.helpers import assert_C_close, random_tw_mask, random_tvw_mask
from tests import gpu_util as gu
import workloads as wl


def _case(seed):
    rng = np.random.default_rng(9000 + seed)
    pattern = "tvw" if rng.random() < 0.35 else "tw"
    G = int(rng.choice([64, 128] if pattern == "tvw" else [32, 64, 128, 128]))
    M = int(rng.choice([1, 7, 64, 129, 300, 517, 700]))
    K = int(rng.choice([1, 5, 33, 100, 257, 640, 900]))
    N = int(rng.choice([1, 9, 128, 131, 300, 500]))
    col_keep, row_keep = float(rng.choice([0.3, 0.8, 1.0])), float(rng.choice([0.1, 0.5, 1.0]))
    opts = dict(tile_m=int(rng.choice([0, 0, 64, 128, 256])), idx_route=int(rng.integers(0, 3)),
                ksplit=int(rng.integers(0, 3)), depth=int(rng.choice([0, 3, 4])),
                tiles_per_wg=int(rng.choice([0, 1, 2, 3])), waves=int(rng.choice([0, 4, 8])),
                xcd_map=int(rng.choice([-1, 0, 1, 2])))
    return rng, pattern, G, M, K, N, col_keep, row_keep, opts


@pytest.mark.gpu
@pytest.mark.parametrize("seed", range(96))
def test_random_shape_mask_and_options(seed):
    import torch
    rng, pattern, G, M, K, N, col_keep, row_keep, opts = _case(seed)
    if pattern == "tw":
        mask = random_tw_mask(rng, K, N, G, col_keep=col_keep, row_keep=row_keep)
        tmask = None
    else:
        mask, tmask = random_tvw_mask(rng, K, N, G, col_keep=col_keep, row_keep=row_keep)
    A, B = wl.make_A(seed, M, K), wl.make_B(seed + 1, K, N, 0.1)
    print(f"case seed={seed} {pattern} G={G} M={M} K={K} N={N} keep={col_keep}/{row_keep} opts={opts}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TVW if pattern == "tvw" else tw.PATTERN_TW, tile_mask=tmask)
    At, lda = gu.to_dev_KM(A)
    Ct, ldc = gu.new_C(N, M, fill=3.0)
    try:
        tw.tw_gemm_ex(At.data_ptr(), M, lda, tw.LAYOUT_KM, p, Ct.data_ptr(), ldc, tw.tw_launch_opts(**opts),
                      torch.cuda.current_stream().cuda_stream)
    except tw.TwError as e:
        assert e.status == 3, e                       # a forced instance that does not exist for this G
        pytest.skip("no such instance")
    finally:
        torch.cuda.synchronize()
        p.free()
    raw = Ct.cpu().numpy()
    assert_C_close(raw[:, :M].T.astype(np.float64), og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    assert (raw[:, M:] == 3.0).all()                  # the padding of the row pitch stays untouched
