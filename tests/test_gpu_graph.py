"""The launches under HIP graph capture (-m gpu): they allocate nothing and record no memset, so a
captured step replays; every replay is checked bit for bit against the eager results, with eager
work and synchronisations of the program between the replays."""
import numpy as np
import pytest

import paper_2402_10876_amd as tw
from tests.helpers import random_tw_mask, random_tvw_mask
import workloads as wl

pytestmark = pytest.mark.gpu


def test_captured_step_replays_bit_exactly():
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    M, K, N, G = 300, 260, 330, 128
    mask = random_tw_mask(rng, K, N, G)
    vmask, vtmask = random_tvw_mask(rng, K, N, G)
    B16, B8 = wl.make_B(1, K, N, 1.0), wl.rng_i8(2, (K, N))
    g = wl.same_geom(20, 3, 3, 2, 9, 9)
    Bc = wl.rng_fp16(3, (g.K, N), 0.1)
    cmask = random_tw_mask(rng, g.K, N, G)
    p_tw = tw.tw_pack(B16, mask, G, tw.PATTERN_TW)
    p_tvw = tw.tw_pack(B16, vmask, G, tw.PATTERN_TVW, tile_mask=vtmask)
    p_i8 = tw.tw_pack_i8(B8, mask, G)
    p_cv = tw.tw_pack(Bc, cmask, G, tw.PATTERN_TW)
    ldx = wl.conv_ldx(g)
    b_cv = tw.tw_conv_bind(p_cv, g, ldx)
    ld, ld8 = 304, 304
    A16 = torch.randn((K, ld), dtype=torch.float16, device=dev)
    A8 = torch.randint(-127, 128, (K, ld8), dtype=torch.int8, device=dev)
    X = torch.from_numpy(wl.make_conv_input(4, g, ldx)).to(dev)
    ldc_cv = (g.Mp + 7) // 8 * 8
    outs = [torch.zeros((N, ld), dtype=torch.float16, device=dev), torch.zeros((N, ld), dtype=torch.float16, device=dev),
            torch.zeros((N, ld8), dtype=torch.int8, device=dev), torch.zeros((N, ldc_cv), dtype=torch.float16, device=dev)]

    def step(stream):
        tw.tw_gemm(A16.data_ptr(), M, ld, tw.LAYOUT_KM, p_tw, outs[0].data_ptr(), ld, stream)
        tw.tw_gemm(A16.data_ptr(), M, ld, tw.LAYOUT_KM, p_tvw, outs[1].data_ptr(), ld, stream)
        tw.tw_gemm_i8(A8.data_ptr(), M, ld8, p_i8, outs[2].data_ptr(), ld8, 1, 1.0 / 300.0, stream)
        tw.tw_conv_gemm(X.data_ptr(), b_cv, outs[3].data_ptr(), ldc_cv, stream)

    step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    assert all(bool(e.any()) for e in eager)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(side.cuda_stream)
    torch.cuda.synchronize()
    for replay in range(4):
        for o in outs:                       # the program's own eager work between the replays
            o.fill_(0)
        scratch = torch.randn((256, 256), device=dev) @ torch.randn((256, 256), device=dev)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        print(f"replay {replay}", flush=True)
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), f"replay {replay} differs from the eager launch"
        assert bool(torch.isfinite(scratch).all())
    for p in (p_tw, p_tvw, p_i8, p_cv):
        p.free()


def test_concurrent_launches_on_two_streams():
    """The launches keep no state outside their arguments: the same handle on two streams with
    distinct outputs, interleaved many times, gives the single-stream result bit for bit."""
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(78)
    M, K, N, G = 1000, 512, 640, 128
    mask = random_tw_mask(rng, K, N, G)
    p = tw.tw_pack(wl.make_B(9, K, N, 1.0), mask, G, tw.PATTERN_TW)
    A1 = torch.randn((K, M), dtype=torch.float16, device=dev)
    A2 = torch.randn((K, M), dtype=torch.float16, device=dev)
    ref1, ref2 = (torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(2))
    cur = torch.cuda.current_stream().cuda_stream
    tw.tw_gemm(A1.data_ptr(), M, M, tw.LAYOUT_KM, p, ref1.data_ptr(), M, cur)
    tw.tw_gemm(A2.data_ptr(), M, M, tw.LAYOUT_KM, p, ref2.data_ptr(), M, cur)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    C1 = [torch.zeros((N, M), dtype=torch.float16, device=dev) for _ in range(8)]
    C2 = [torch.zeros((N, M), dtype=torch.float16, device=dev) for _ in range(8)]
    torch.cuda.synchronize()
    for i in range(8):
        tw.tw_gemm(A1.data_ptr(), M, M, tw.LAYOUT_KM, p, C1[i].data_ptr(), M, s1.cuda_stream)
        tw.tw_gemm(A2.data_ptr(), M, M, tw.LAYOUT_KM, p, C2[i].data_ptr(), M, s2.cuda_stream)
    torch.cuda.synchronize()
    for i in range(8):
        assert torch.equal(C1[i], ref1) and torch.equal(C2[i], ref2), i
    p.free()
