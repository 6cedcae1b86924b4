"""Row-major compatibility layout, both pipelines, and the remaining configured
workloads (BERT-large sweep, VGG-16 im2col shapes) against the oracle (-m gpu)."""
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


def _oracle(c, rows=None):
    A = c.A if rows is None else c.A[rows]
    return og.gemm_oracle(A, c.B, c.mask), og.abs_bound(A, c.B, c.mask)


def _pack(c):
    if c.pattern == "tvw":
        return tw.tw_pack(c.B, c.mask, c.G, tw.PATTERN_TVW, tile_mask=c.tile_mask)
    return tw.tw_pack(c.B, c.mask, c.G, tw.PATTERN_TW)


@pytest.mark.parametrize("G", [32, 64, 128])
def test_row_major_layout_tw(G):
    rng = np.random.default_rng(50 + G)
    M, K, N = 203, 150, 300
    mask = random_tw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.5)
    A, B = wl.make_A(G, M, K), wl.make_B(G, K, N, 1.0)
    print(f"case row-major G={G}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    C, raw = gu.run_tw_mk(tw, p, A, N, ldc=312, fill=5.0)
    p.free()
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    assert not raw[:, :N][:, ~mask.any(0)].view(np.uint16).any()
    assert (raw[:, N:] == 5.0).all()


def test_row_major_equals_transposed_layout_bitwise():
    c = wl.make_case(1, M=200)
    p = _pack(c)
    C_mk, _ = gu.run_tw_mk(tw, p, c.A, c.N)
    tw.tw_set_option("kernel", 1)                 # same register-staged kernel, other layout
    tw.tw_set_option("tile_m", 128)
    C_km, _ = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    assert np.array_equal(C_mk, C_km)


def test_row_major_dense():
    A, B = wl.make_A(3, 130, 96), wl.make_B(3, 96, 200, 0.1)
    C = gu.run_dense_mk(tw, A, B)
    ones = np.ones(B.shape, np.uint8)
    assert_C_close(C, og.gemm_oracle(A, B, ones), og.abs_bound(A, B, ones))


@pytest.mark.parametrize("kernel,depth", [(1, 3), (2, 3), (2, 4)])
@pytest.mark.parametrize("tile_m", [64, 128, 256])
def test_both_pipelines_agree_with_oracle(kernel, depth, tile_m):
    tw.tw_set_option("kernel", kernel); tw.tw_set_option("depth", depth); tw.tw_set_option("tile_m", tile_m)
    c = wl.make_case(2, 0, M=520, recipe="global")
    print(f"case {c.name} kernel={kernel} depth={depth} tile_m={tile_m}", flush=True)
    p = _pack(c)
    C, _ = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    ref, S = _oracle(c)
    assert_C_close(C, ref, S)
    # dense baseline on the same pipeline
    Cd, _ = gu.run_dense(tw, c.A, c.B)
    ones = np.ones_like(c.mask)
    assert_C_close(Cd, og.gemm_oracle(c.A, c.B, ones), og.abs_bound(c.A, c.B, ones))


@pytest.mark.parametrize("tile_m,depth", [(128, 3), (128, 4), (256, 3)])
def test_eight_wave_workgroups(tile_m, depth):
    for k, v in (("kernel", 2), ("waves", 8), ("tile_m", tile_m), ("depth", depth)):
        tw.tw_set_option(k, v)
    c = wl.make_case(2, 2, M=520, recipe="global")
    print(f"case {c.name} waves=8 tile_m={tile_m} depth={depth}", flush=True)
    p = _pack(c)
    C, _ = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    ref, S = _oracle(c)
    assert_C_close(C, ref, S)
    Cd, _ = gu.run_dense(tw, c.A, c.B)
    ones = np.ones_like(c.mask)
    assert_C_close(Cd, og.gemm_oracle(c.A, c.B, ones), og.abs_bound(c.A, c.B, ones))


@pytest.mark.parametrize("tile_m,depth,G", [(128, 3, 128), (64, 3, 128), (64, 4, 128), (128, 3, 64)])
@pytest.mark.parametrize("K_keep", ["odd", "even"])
def test_k_split_inside_the_workgroup(tile_m, depth, G, K_keep):
    """Two wave groups share one output tile; an odd number of 32-row stages
    leaves the second group idle on the last stage."""
    for k, v in (("kernel", 2), ("ksplit", 2), ("tile_m", tile_m), ("depth", depth)):
        tw.tw_set_option(k, v)
    rng = np.random.default_rng(70 + tile_m + G)
    M, K, N = 333, 800, 300
    mask = random_tw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.42 if K_keep == "odd" else 0.5)
    A, B = wl.make_A(7, M, K), wl.make_B(7, K, N, 0.1)
    print(f"case ksplit tile_m={tile_m} depth={depth} G={G} {K_keep}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    C, _ = gu.run_tw(tw, p, A, N)
    p.free()
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    A2, B2 = wl.make_A(8, 200, 448), wl.make_B(8, 448, 260, 0.1)     # dense, K % 64 == 0
    Cd, _ = gu.run_dense(tw, A2, B2)
    ones = np.ones(B2.shape, np.uint8)
    assert_C_close(Cd, og.gemm_oracle(A2, B2, ones), og.abs_bound(A2, B2, ones))


@pytest.mark.parametrize("pattern,sparsity", [("tw", 0.0), ("tw", 0.5), ("tw", 0.75), ("tw", 0.875), ("tw", 0.9375),
                                              ("tvw", 0.5), ("tvw", 0.75), ("tvw", 0.875), ("tvw", 0.9375)])
@pytest.mark.parametrize("shape_index", [0, 1])
def test_config4_bert_large_sweep_reduced_M(shape_index, pattern, sparsity):
    cf = 0.0 if sparsity in (0.0,) or (pattern == "tvw" and sparsity == 0.5) else None
    c = wl.make_case(4, shape_index, pattern=pattern, sparsity=sparsity, col_frac=cf, M=384)
    print(f"case {c.name}", flush=True)
    p = _pack(c)
    C, _ = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    ref, S = _oracle(c)
    assert_C_close(C, ref, S)
    if sparsity == 0.0:                           # 0 % is the dense GEMM
        Cd, _ = gu.run_dense(tw, c.A, c.B)
        assert_C_close(Cd, ref, S)


_A_DEV = {}


def _config4_A_on_device(shape_index):
    """A^T of a BERT-large FFN shape at full M, made and uploaded once for all its rows."""
    import torch
    if shape_index not in _A_DEV:
        _A_DEV.clear()                                  # one shape resident at a time
        shp = wl.SHAPES[4][shape_index]
        A = wl.make_A(wl.seed_for(4, shape_index), shp.M, shp.K)
        _A_DEV[shape_index] = (A, torch.from_numpy(np.ascontiguousarray(A.T)).cuda())
    return _A_DEV[shape_index]


@pytest.mark.parametrize("pattern,sparsity", [("tw", 0.0), ("tw", 0.5), ("tw", 0.75), ("tw", 0.875), ("tw", 0.9375),
                                              ("tvw", 0.5), ("tvw", 0.75), ("tvw", 0.875), ("tvw", 0.9375)])
@pytest.mark.parametrize("shape_index", [0, 1])
def test_config4_bert_large_sweep_full_size(shape_index, pattern, sparsity):
    """Every row of the BERT-large FFN sweep at M = 8192, in the launch configuration the heuristics
    pick there (the one the benchmark times), against the oracle on sampled rows of A."""
    import torch
    cf = 0.0 if sparsity == 0.0 or (pattern == "tvw" and sparsity == 0.5) else None
    c = wl.make_case(4, shape_index, pattern=pattern, sparsity=sparsity, col_frac=cf, with_A=False)
    A, At = _config4_A_on_device(shape_index)
    M = A.shape[0]
    print(f"case {c.name} M={M}", flush=True)
    p = _pack(c)
    Ct = torch.full((c.N, M), float("nan"), dtype=torch.float16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    tw.tw_gemm(At.data_ptr(), M, M, tw.LAYOUT_KM, p, Ct.data_ptr(), M, st)
    torch.cuda.synchronize()
    p.free()
    raw = Ct.cpu().numpy()
    rows = np.r_[0:8, 4090:4100, M - 8:M, np.arange(5, M, 257)]
    ref = og.gemm_oracle(A[rows], c.B, c.mask)
    S = og.abs_bound(A[rows], c.B, c.mask)
    assert_C_close(raw[:, rows].T, ref, S)
    assert np.isfinite(raw).all() and not raw[~c.mask.any(0)].view(np.uint16).any()
    if sparsity == 0.0:                           # 0 % is the dense GEMM, also at this size
        Bd = torch.from_numpy(c.B).cuda()
        Ct.fill_(float("nan"))
        tw.tw_dense_gemm(At.data_ptr(), Bd.data_ptr(), Ct.data_ptr(), M, c.K, c.N, M, c.N, M, tw.LAYOUT_KM, st)
        torch.cuda.synchronize()
        assert_C_close(Ct[:, torch.from_numpy(rows).cuda()].T.cpu().numpy(), ref, S)


@pytest.mark.parametrize("pattern,sparsity,G", [("tw", 0.75, 64), ("tw", 0.75, 128), ("tvw", 0.875, 64), ("tvw", 0.875, 128)])
def test_config5_vgg_conv_512_full_size(pattern, sparsity, G):
    c = wl.make_case(5, 1, pattern=pattern, sparsity=sparsity, G=G)      # M = 1568: M tail
    print(f"case {c.name}", flush=True)
    p = _pack(c)
    C, raw = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    rows = np.r_[0:8, 1560:1568, np.arange(3, c.M, 97)]
    ref, S = _oracle(c, rows)
    assert_C_close(C[rows], ref, S)
    assert np.isfinite(C).all()


@pytest.mark.parametrize("pattern,sparsity,G", [("tw", 0.75, 64), ("tvw", 0.875, 64), ("tw", 0.75, 128), ("tvw", 0.875, 128)])
def test_config5_vgg_conv_256_full_size_sampled(pattern, sparsity, G):
    c = wl.make_case(5, 0, pattern=pattern, sparsity=sparsity, G=G)      # M = 25088
    print(f"case {c.name}", flush=True)
    p = _pack(c)
    C, raw = gu.run_tw(tw, p, c.A, c.N)
    p.free()
    rows = np.r_[0:8, 25080:25088, np.arange(11, c.M, 1571)]
    ref, S = _oracle(c, rows)
    assert_C_close(C[rows], ref, S)
    assert np.isfinite(C).all()


@pytest.mark.parametrize("pattern", ["tw", "tvw", "dense"])
def test_A_beyond_4_GiB_takes_the_64_bit_path(pattern):
    """K * lda * 2 bytes >= 2^32: the asynchronous TW kernel (32-bit byte offsets into A) must
    not be chosen; the kernels with 64-bit addressing give the oracle's values on sampled m."""
    import torch
    from tests.helpers import random_tvw_mask
    K, N, G = 1032, 130, 128
    M = (1 << 21) + 8
    assert K * M * 2 >= 1 << 32
    rng = np.random.default_rng(3)
    if pattern == "dense":
        mask = np.ones((K, N), np.uint8)
        tm, pat = mask, None
    elif pattern == "tw":
        mask = random_tw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.3)
        tm, pat = mask, tw.PATTERN_TW
    else:
        mask, tm = random_tvw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.3)
        pat = tw.PATTERN_TVW
    B = wl.make_B(3, K, N, 1.0)
    print(f"case A beyond 4 GiB, {pattern}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(5)
    At = torch.empty((K, M), dtype=torch.float16, device="cuda")
    for k0 in range(0, K, 129):                       # in slabs: no 8 GiB fp32 temporary
        At[k0:k0 + 129].copy_(torch.randn((min(129, K - k0), M), generator=gen, device="cuda", dtype=torch.float32))
    Ct = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    if pattern == "dense":
        Bd = torch.from_numpy(np.ascontiguousarray(np.pad(B, ((0, 0), (0, 6))))).cuda()     # ldb = 136
        tw.tw_dense_gemm(At.data_ptr(), Bd.data_ptr(), Ct.data_ptr(), M, K, N, M, 136, M, tw.LAYOUT_KM, st)
        torch.cuda.synchronize()
    else:
        p = tw.tw_pack(B, mask, G, pat, tile_mask=tm if pattern == "tvw" else None)
        tw.tw_gemm(At.data_ptr(), M, M, tw.LAYOUT_KM, p, Ct.data_ptr(), M, st)
        torch.cuda.synchronize()
        p.free()
    idx = torch.from_numpy(np.concatenate([[0, 1, M - 1, M - 8, (1 << 20) + 3],
                                           rng.integers(0, M, 43)])).cuda()
    A_s = At[:, idx].T.contiguous().cpu().numpy()          # 48 x K
    C_s = Ct[:, idx].T.contiguous().cpu().numpy().astype(np.float64)
    del At, Ct
    assert_C_close(C_s, og.gemm_oracle(A_s, B, mask), og.abs_bound(A_s, B, mask))
