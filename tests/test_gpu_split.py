"""K split across workgroups (tw_gemm_ex with a workspace), per-call launch options and
convolution bindings: parity with the oracle, determinism, and concurrent use of one handle (-m gpu)."""
import threading

import numpy as np
import pytest

import paper_2402_10876_amd as tw
from oracle import conv as oc
from oracle import gemm as og
from tests.helpers import assert_C_close, random_tw_mask
from tests import gpu_util as gu
import workloads as wl


def test_option_and_workspace_errors_need_no_device():
    p = tw.tw_pack_host(np.ones((64, 128), np.float16), np.ones((64, 128), np.uint8), 128, tw.PATTERN_TW)
    assert tw.tw_gemm_workspace_bytes(p, 100) >= 4096 + 2 * 8 * 64 * 128 * 4
    for bad in (dict(tile_m=100), dict(depth=5), dict(waves=3), dict(wg_split=9), dict(tiles_per_wg=9), dict(kernel=3), dict(xcd_map=7),
                dict(workspace_dev=0x1010, workspace_bytes=1 << 20)):
        o = tw.tw_launch_opts(**bad)
        with pytest.raises(tw.TwError) as ei:
            tw.tw_gemm_ex(0x10000, 8, 8, tw.LAYOUT_KM, p, 0x20000, 8, o)
        assert ei.value.status in (1, 6), bad          # not uploaded (6) is checked before the options
    with pytest.raises(tw.TwError) as ei:
        tw.tw_workspace_init(0x1010, 1 << 20)
    assert ei.value.status == 1
    p.free()


def _run_ex(p, A16, N, opts):
    import torch
    M = A16.shape[0]
    At, lda = gu.to_dev_KM(A16)
    Ct, ldc = gu.new_C(N, M)
    tw.tw_gemm_ex(At.data_ptr(), M, lda, tw.LAYOUT_KM, p, Ct.data_ptr(), ldc, opts, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = Ct.cpu().numpy()
    return raw[:, :M].T.astype(np.float64), raw


def _workspace(p, M):
    import torch
    n = tw.tw_gemm_workspace_bytes(p, M)
    ws = torch.full((n,), 0x5A, dtype=torch.uint8, device="cuda")      # garbage: init must clear what matters
    tw.tw_workspace_init(ws.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
    return ws, n


@pytest.mark.gpu
@pytest.mark.parametrize("G,tile_m,S", [(128, 128, 2), (128, 128, 3), (128, 64, 4), (128, 64, 8), (64, 128, 2), (64, 128, 5)])
def test_wg_split_parity_and_determinism(G, tile_m, S):
    rng = np.random.default_rng(900 + G + tile_m + S)
    M, K, N = 333, 1500, 300
    mask = random_tw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.45)
    A, B = wl.make_A(31, M, K), wl.make_B(31, K, N, 0.1)
    print(f"case wg_split G={G} tile_m={tile_m} S={S}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    ws, n = _workspace(p, M)
    o = tw.tw_launch_opts(tile_m=tile_m, wg_split=S, workspace_dev=ws.data_ptr(), workspace_bytes=n)
    ref, Sb = og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask)
    C1, raw1 = _run_ex(p, A, N, o)
    assert_C_close(C1, ref, Sb)
    assert not raw1[~mask.any(0)].view(np.uint16)[:, :M].any()               # pruned columns: +0
    for _ in range(3):                       # same workspace again: counters are back at zero, same bits
        _, raw = _run_ex(p, A, N, o)
        assert np.array_equal(raw.view(np.uint16)[:, :M], raw1.view(np.uint16)[:, :M])
    p.free()


@pytest.mark.gpu
def test_wg_split_short_tiles_and_small_workspace():
    """Tiles with fewer stages than workgroups per pair (some shares are empty), and a workspace
    that cannot hold the split that was asked for."""
    import torch
    rng = np.random.default_rng(5)
    M, K, N, G = 200, 96, 260, 128
    mask = random_tw_mask(rng, K, N, G, col_keep=0.9, row_keep=0.5)            # ~48 rows: 2 stages
    A, B = wl.make_A(32, M, K), wl.make_B(32, K, N, 0.1)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    ws, n = _workspace(p, M)
    C, _ = _run_ex(p, A, N, tw.tw_launch_opts(tile_m=128, wg_split=4, workspace_dev=ws.data_ptr(), workspace_bytes=n))
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    small = tw.tw_launch_opts(tile_m=128, wg_split=4, workspace_dev=ws.data_ptr(), workspace_bytes=8192)
    At, lda = gu.to_dev_KM(A)
    Ct, ldc = gu.new_C(N, M)
    with pytest.raises(tw.TwError) as ei:
        tw.tw_gemm_ex(At.data_ptr(), M, lda, tw.LAYOUT_KM, p, Ct.data_ptr(), ldc, small, torch.cuda.current_stream().cuda_stream)
    assert ei.value.status == 1
    p.free()


@pytest.mark.gpu
@pytest.mark.parametrize("cfg,si,G,S", [(5, 1, 128, 4), (5, 1, 64, 3), (2, 2, 128, 2)])
def test_split_on_the_few_tile_shapes_at_full_size(cfg, si, G, S):
    """512 -> 512 convolution GEMM (M = 1568, K = 4608) and BERT-base FFN2 at full size, K shared
    out over S workgroups per tile, against the oracle on sampled rows."""
    c = wl.make_case(cfg, si, G=G)
    print(f"case {c.name} wg_split={S}", flush=True)
    p = tw.tw_pack(c.B, c.mask, c.G, tw.PATTERN_TW)
    ws, n = _workspace(p, c.M)
    C, raw = _run_ex(p, c.A, c.N, tw.tw_launch_opts(wg_split=S, workspace_dev=ws.data_ptr(), workspace_bytes=n))
    p.free()
    rows = np.r_[0:8, c.M - 8:c.M, np.arange(3, c.M, 97)]
    assert_C_close(C[rows], og.gemm_oracle(c.A[rows], c.B, c.mask), og.abs_bound(c.A[rows], c.B, c.mask))
    assert np.isfinite(C).all()


@pytest.mark.gpu
@pytest.mark.parametrize("depth,tile_m,G", [(6, 128, 128), (8, 128, 128), (6, 64, 128), (8, 64, 128), (6, 128, 64), (8, 128, 64),
                                            (4, 128, 128), (3, 256, 64)])
@pytest.mark.parametrize("K", [100, 1700])
def test_pipeline_depths(depth, tile_m, G, K):
    """Stages in flight 3 .. 8; K = 1700 keeps about 25 stages (the kept-row list passes through its
    LDS ring three times), K = 100 fewer stages than the pipeline is deep."""
    rng = np.random.default_rng(depth * 100 + tile_m + G + K)
    M, N = 300, 270
    mask = random_tw_mask(rng, K, N, G, col_keep=0.85, row_keep=0.48)
    A, B = wl.make_A(51, M, K), wl.make_B(51, K, N, 0.1)
    print(f"case depth={depth} tile_m={tile_m} G={G} K={K}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    C, _ = _run_ex(p, A, N, tw.tw_launch_opts(tile_m=tile_m, depth=depth, kernel=2, ksplit=1))
    p.free()
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))


@pytest.mark.gpu
@pytest.mark.parametrize("route", [1, 2])
@pytest.mark.parametrize("tile_m,waves,G,depth", [(128, 4, 128, 3), (64, 4, 128, 4), (256, 8, 128, 3), (128, 8, 128, 3), (256, 4, 64, 3),
                                                 (128, 4, 64, 4)])
def test_both_routes_of_the_kept_row_list(route, tile_m, waves, G, depth):
    """Scalar loads and the LDS ring give the same bits (same products in the same order); K = 1300
    sends the list through the ring twice."""
    rng = np.random.default_rng(tile_m + waves + G + depth)
    M, K, N = 290, 1300, 200
    mask = random_tw_mask(rng, K, N, G, col_keep=0.85, row_keep=0.5)
    A, B = wl.make_A(61, M, K), wl.make_B(61, K, N, 0.1)
    print(f"case idx_route={route} tile_m={tile_m} waves={waves} G={G} depth={depth}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    C, raw = _run_ex(p, A, N, tw.tw_launch_opts(tile_m=tile_m, waves=waves, depth=depth, kernel=2, ksplit=1, idx_route=route))
    C2, raw2 = _run_ex(p, A, N, tw.tw_launch_opts(tile_m=tile_m, waves=waves, depth=depth, kernel=2, ksplit=1, idx_route=3 - route))
    p.free()
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    assert np.array_equal(raw.view(np.uint16)[:, :M], raw2.view(np.uint16)[:, :M])


@pytest.mark.gpu
@pytest.mark.parametrize("tpw", [2, 3, 8])
@pytest.mark.parametrize("tile_m,waves,ksplit,G,route", [(64, 4, 1, 128, 2), (64, 4, 1, 128, 1), (128, 4, 1, 128, 1), (128, 4, 1, 128, 2),
                                                        (256, 8, 1, 128, 1), (128, 4, 2, 128, 2), (128, 4, 1, 64, 2)])
def test_several_tiles_per_workgroup(tpw, tile_m, waves, ksplit, G, route):
    """A workgroup that computes several tiles one after the other (pruned columns and the ragged
    last M-tile among its jobs, fewer jobs than tpw x workgroups at the end) gives the bits of one
    tile per workgroup, and those match the oracle; instances without the loop ignore the option."""
    rng = np.random.default_rng(tpw * 1000 + tile_m + waves + ksplit + G)
    M, K, N = 490, 330, 530
    mask = random_tw_mask(rng, K, N, G, col_keep=0.8, row_keep=0.5)
    A, B = wl.make_A(71, M, K), wl.make_B(71, K, N, 0.1)
    print(f"case tiles_per_wg={tpw} tile_m={tile_m} waves={waves} ksplit={ksplit} G={G} idx_route={route}", flush=True)
    p = tw.tw_pack(B, mask, G, tw.PATTERN_TW)
    kw = dict(tile_m=tile_m, waves=waves, kernel=2, ksplit=ksplit, idx_route=route)
    C, raw = _run_ex(p, A, N, tw.tw_launch_opts(tiles_per_wg=tpw, **kw))
    C1, raw1 = _run_ex(p, A, N, tw.tw_launch_opts(tiles_per_wg=1, **kw))
    p.free()
    assert_C_close(C, og.gemm_oracle(A, B, mask), og.abs_bound(A, B, mask))
    assert np.array_equal(raw.view(np.uint16), raw1.view(np.uint16))


@pytest.mark.gpu
def test_one_handle_two_threads_different_options_and_geometries():
    """Per-call options and bindings: two host threads launch the same handle at the same time
    with different tile heights (on their own streams), and two convolution geometries bound to
    one handle run side by side; every result equals the single-threaded one bit for bit."""
    import torch
    rng = np.random.default_rng(11)
    g1, g2 = wl.same_geom(16, 3, 3, 2, 12, 10), wl.same_geom(16, 3, 3, 3, 7, 9)
    N, G = 200, 128
    Bw = wl.rng_fp16(40, (g1.K, N), 0.1)
    mask = random_tw_mask(rng, g1.K, N, G)
    p = tw.tw_pack(Bw, mask, G, tw.PATTERN_TW)
    M = 700
    A = wl.make_A(41, M, g1.K)
    At, lda = gu.to_dev_KM(A)
    X1, X2 = wl.make_conv_input(42, g1), wl.make_conv_input(43, g2)
    Xd = [torch.from_numpy(X1).cuda(), torch.from_numpy(X2).cuda()]
    bind = [tw.tw_conv_bind(p, g1, X1.shape[1]), tw.tw_conv_bind(p, g2, X2.shape[1])]     # both alive at once
    geoms = [g1, g2]

    def gemm(tile_m, stream, Ct):
        tw.tw_gemm_ex(At.data_ptr(), M, lda, tw.LAYOUT_KM, p, Ct.data_ptr(), Ct.shape[1], tw.tw_launch_opts(tile_m=tile_m), stream)

    def conv(i, stream, Ct):
        tw.tw_conv_gemm(Xd[i].data_ptr(), bind[i], Ct.data_ptr(), Ct.shape[1], stream)

    def outputs():
        return ([gu.new_C(N, M)[0] for _ in range(2)] + [gu.new_C(N, g.Mp)[0] for g in geoms])
    st0 = torch.cuda.current_stream().cuda_stream
    want = outputs()
    gemm(64, st0, want[0]); gemm(256, st0, want[1]); conv(0, st0, want[2]); conv(1, st0, want[3])
    torch.cuda.synchronize()
    want = [w.cpu().numpy().view(np.uint16) for w in want]
    ref, Sb = og.gemm_oracle(A, Bw, mask), og.abs_bound(A, Bw, mask)
    for w in want[:2]:
        assert_C_close(w.view(np.float16)[:, :M].T, ref, Sb)
    for w, g, X in zip(want[2:], geoms, (X1, X2)):
        assert_C_close(w.view(np.float16)[:, :g.Mp].T, oc.conv_wide_oracle(X, Bw, mask, **g.ints()),
                       oc.conv_wide_abs_bound(X, Bw, mask, **g.ints()))

    streams = [torch.cuda.Stream() for _ in range(2)]
    errors = []

    def worker(t, got):
        try:
            s = streams[t].cuda_stream
            for rep in range(20):
                gemm(64 if t == 0 else 256, s, got[t])
                conv(t, s, got[2 + t])
            streams[t].synchronize()
        except Exception as e:          # noqa: BLE001
            errors.append(e)
    got = outputs()
    torch.cuda.synchronize()
    th = [threading.Thread(target=worker, args=(t, got)) for t in range(2)]
    for t in th:
        t.start()
    for t in th:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for w, gt in zip(want, got):
        assert np.array_equal(w, gt.cpu().numpy().view(np.uint16))
    for b in bind:
        b.free()
    p.free()
