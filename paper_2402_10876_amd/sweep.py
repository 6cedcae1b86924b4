"""Timing sweep over the configured workloads: python -m paper_2402_10876_amd.sweep [--configs 2,3,4,5]

For every (layer shape, pattern, sparsity, G) it times the sparse launch and our
dense baseline back to back on rotating buffer sets (operands from HBM) and
prints one JSON line with dense-equivalent TFLOP/s, condensed-FLOP matrix-core
utilisation, speed-up over the dense baseline and the fraction of the binding
roofline (vendor peaks: 8 TB/s, 2.5 PFLOP/s fp16 dense).  `--cube` adds the
paper's 4096 x 4096 x 4096 sparsity sweep (Section VI-B; TVW at 50 % is plain
2:4).  `--imbalance` times uneven tiles (one magnitude threshold over all
tile rows of the matrix instead of one per tile: Section IV "global weight
pruning", Section V "load imbalance") with the tiles launched longest first and
in column order.  `--tew` adds the TEW pattern (TW plus delta restored elements).
`--conv` times config 5's convolutions with the img2col matrix never materialised
(`tw_conv_gemm` on the wide input) against the same handle on the materialised matrix.
`--i8` times the int8 TW path (Section VI-B "Int8 Quantization") against the dense
int8 baseline and the fp16 TW launch of the same mask.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

HBM = 8.0e12
MFMA = 2.5e15


def alg_bytes(M, K_union, N, pattern, skw, sk):
    """A rows kept by some tile + all of C + condensed weight + kept-row lists."""
    w = 2 * skw if pattern == "tw" else skw + skw // 8
    return 2 * M * K_union + 2 * M * N + w + 4 * sk


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="2,3,4,5")
    ap.add_argument("--cube", action="store_true")
    ap.add_argument("--imbalance", action="store_true")
    ap.add_argument("--tew", action="store_true",
                    help="TEW at 75 % with delta = 0.5, 1.5 and 5 % on the BERT shapes (Section VI, impact of delta)")
    ap.add_argument("--conv", action="store_true",
                    help="implicit img2col (tw_conv_gemm) vs the materialised matrix on the VGG layers")
    ap.add_argument("--i8", action="store_true",
                    help="int8 TW at 75 % (int8 and int32 outputs) vs the dense int8 baseline")
    ap.add_argument("--reps", type=int, default=24)
    ap.add_argument("--sets", type=int, default=6)
    args = ap.parse_args()

    import torch
    import paper_2402_10876_amd as tw
    import workloads as wl

    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream

    def timed(fn, reps, rounds=3):
        vals = []
        for _ in range(rounds):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for r in range(reps):
                fn(r)
            e1.record()
            torch.cuda.synchronize()
            vals.append(e0.elapsed_time(e1) / reps * 1e-3)
        return float(np.median(vals))

    plan = []
    cfgs = [int(c) for c in args.configs.split(",") if c]
    for cfg in cfgs:
        for si in range(len(wl.SHAPES[cfg])):
            if cfg == 2:
                plan.append((cfg, si, "tw", 0.75, 128))
            elif cfg == 3:
                plan.append((cfg, si, "tvw", 0.875, 128))
            elif cfg == 4:
                for sp in (0.0, 0.5, 0.75, 0.875, 0.9375):
                    plan.append((cfg, si, "tw", sp, 128))
                for sp in (0.5, 0.75, 0.875, 0.9375):
                    plan.append((cfg, si, "tvw", sp, 128))
            elif cfg == 5:
                plan += [(cfg, si, "tw", 0.75, 64), (cfg, si, "tw", 0.75, 128),
                         (cfg, si, "tvw", 0.875, 64), (cfg, si, "tvw", 0.875, 128)]
    if args.cube:
        wl.SHAPES[6] = [wl.Shape("cube_4096", 4096, 4096, 4096, 0.02)]
        wl.CONFIGS[6] = dict(G=128, pattern="tw", sparsity=0.75, col_frac=0.10)
        for sp in (0.0, 0.1, 0.25, 0.5, 0.75, 0.875):
            plan.append((6, 0, "tw", sp, 128))
            plan.append((6, 0, "tw", sp, 64))
        for sp in (0.5, 0.75, 0.875):
            plan.append((6, 0, "tvw", sp, 128))

    if args.cube or args.imbalance:
        wl.SHAPES[6] = [wl.Shape("cube_4096", 4096, 4096, 4096, 0.02)]
        wl.CONFIGS[6] = dict(G=128, pattern="tw", sparsity=0.75, col_frac=0.10)
    if args.imbalance:
        for cfg, si in ((4, 0), (4, 1), (6, 0)):
            shp = wl.SHAPES[cfg][si]
            M, K, N = shp.M, shp.K, shp.N
            nsets = max(2, min(args.sets, int(600e6 // (2 * M * (K + N)))))
            A = [torch.randn((K, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
            C = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
            for recipe in ("per_tile", "global", "global, column blocks rescaled"):
                if recipe.startswith("global,"):
                    # i.i.d. weights give nearly even tiles under one threshold; trained layers do
                    # not: rescale each block of 128 columns by exp(N(0, 0.6^2)) before thresholding
                    Bs = wl.make_B(wl.seed_for(cfg, si), K, N, shp.sigma).astype(np.float32)
                    f = np.exp(0.6 * np.random.default_rng(wl.seed_for(cfg, si) + 7).standard_normal((N + 127) // 128))
                    Bs = (Bs * np.repeat(f, 128)[:N]).astype(np.float16)
                    mask = wl.tw_mask(Bs, 128, density=0.25, col_frac=0.10, recipe="global")
                    c = wl.Case("rescaled", M, K, N, 128, "tw", 0.75, 0, None, Bs, mask, mask)
                else:
                    c = wl.make_case(cfg, si, pattern="tw", sparsity=0.75, G=128, recipe=recipe, with_A=False)
                row = dict(shape=shp.name, M=M, K=K, N=N, G=128, pattern="tw", sparsity=0.75, recipe=recipe)
                for order in (1, 0):
                    tw.tw_set_option("tile_order", order)
                    packed = [tw.tw_pack(c.B, c.mask, 128, tw.PATTERN_TW) for _ in range(nsets)]
                    t = timed(lambda r: tw.tw_gemm(A[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % nsets],
                                                   C[r % nsets].data_ptr(), M, stream), args.reps)
                    e = packed[0].export()
                    kt = np.array([len(r) for r in e["row_idx"]])
                    row.update({("us_longest_first" if order else "us_column_order"): round(t * 1e6, 2),
                                "K_t_min": int(kt.min()), "K_t_mean": round(float(kt.mean()), 1), "K_t_max": int(kt.max())})
                    for p in packed:
                        p.free()
                tw.tw_set_option("tile_order", 1)
                print(json.dumps(row), flush=True)
            del A, C

    if args.conv:
        for si, (name, g, N) in enumerate(wl.CONV_LAYERS):
            M, K, Mp, ldx = g.B * g.H * g.W, g.K, g.Mp, wl.conv_ldx(g)
            ns_conv = max(2, min(24, int(600e6 // (2 * (g.C * ldx + N * Mp)))))
            ns_mat = max(2, min(args.sets, int(600e6 // (2 * M * (K + N)))))
            X = [torch.randn((g.C, ldx), dtype=torch.float16, device=dev) for _ in range(ns_conv)]
            Cw = [torch.empty((N, Mp), dtype=torch.float16, device=dev) for _ in range(ns_conv)]
            A = [torch.randn((K, M), dtype=torch.float16, device=dev) for _ in range(ns_mat)]
            Cm = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(ns_mat)]
            for pattern, sp, G in (("tw", 0.75, 128), ("tw", 0.75, 64), ("tvw", 0.875, 128), ("tw", 0.0, 128)):
                c = wl.make_case(5, si, pattern=pattern, sparsity=sp, G=G, col_frac=0.0 if sp == 0.0 else None,
                                 with_A=False)
                pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
                packed = [tw.tw_pack(c.B, c.mask, G, pat, tile_mask=c.tile_mask if pattern != "tw" else None)
                          for _ in range(ns_conv)]
                for p in packed:
                    tw.tw_conv_bind(p, g, ldx)
                skw, sk, ku = packed[0].flop_counts()
                t_conv = timed(lambda r: tw.tw_conv_gemm(X[r % ns_conv].data_ptr(), packed[r % ns_conv],
                                                         Cw[r % ns_conv].data_ptr(), Mp, stream), args.reps)
                t_mat = timed(lambda r: tw.tw_gemm(A[r % ns_mat].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % ns_mat],
                                                   Cm[r % ns_mat].data_ptr(), M, stream), args.reps)
                wbytes = 2 * skw if pattern == "tw" else skw + skw // 8
                ab = 2 * g.C * Mp + 2 * N * Mp + wbytes + 4 * sk       # the input once, C over the wide grid, weight
                print(json.dumps(dict(
                    shape=name, positions=M, wide_grid=Mp, K=K, N=N, G=G, pattern=pattern, sparsity=sp,
                    us_implicit=round(t_conv * 1e6, 2), us_materialised=round(t_mat * 1e6, 2),
                    speedup_vs_materialised=round(t_mat / t_conv, 3),
                    dense_eq_tflops=round(2.0 * M * K * N / t_conv / 1e12, 1),
                    input_MB=round(2 * g.C * Mp / 1e6, 2), materialised_A_MB=round(2 * M * ku / 1e6, 2),
                    alg_MB=round(ab / 1e6, 2), alg_GBps=round(ab / t_conv / 1e9, 1),
                    roofline_frac=round(max(ab / HBM, (1.0 if pattern == "tvw" else 2.0) * Mp * skw / MFMA) / t_conv, 4))),
                    flush=True)
                for p in packed:
                    p.free()
            del X, Cw, A, Cm

    if args.i8:
        shapes = [(2, si) for si in range(len(wl.SHAPES[2]))] + [(4, 0), (4, 1)]
        if args.cube:
            shapes.append((6, 0))
        for cfg, si in shapes:
            shp = wl.SHAPES[cfg][si]
            M, K, N, G = shp.M, shp.K, shp.N, 128
            nsets = max(2, min(args.sets, int(600e6 // (M * (K + 4 * N)))))
            B8 = wl.rng_i8(wl.seed_for(cfg, si) + 1, (K, N))
            cases = [("tw", sp) for sp in ((0.75, 0.875) if cfg != 6 else (0.5, 0.75, 0.875))] + [("tvw", 0.875)]
            for pattern, sp in cases:
                B16 = B8.astype(np.float16)
                if pattern == "tw":
                    mask = tmask = wl.tw_mask(B16, G, density=1.0 - sp, col_frac=0.10)
                else:
                    mask, tmask = wl.tvw_mask(B16, G, sparsity=sp, col_frac=0.10)
                pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
                tmk = tmask if pattern == "tvw" else None
                packed = [tw.tw_pack_i8(B8, mask, G, pat, tile_mask=tmk) for _ in range(nsets)]
                p16 = [tw.tw_pack(B16, mask, G, pat, tile_mask=tmk) for _ in range(nsets)]
                A8 = [torch.randint(-127, 128, (K, M), dtype=torch.int8, device=dev) for _ in range(nsets)]
                A16 = [a.to(torch.float16) for a in A8]
                C32 = [torch.empty((N, M), dtype=torch.int32, device=dev) for _ in range(nsets)]
                C8 = [torch.empty((N, M), dtype=torch.int8, device=dev) for _ in range(nsets)]
                C16 = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
                Bd = torch.from_numpy(B8).to(dev)
                skw, sk, ku = packed[0].flop_counts()
                t8 = timed(lambda r: tw.tw_gemm_i8(A8[r % nsets].data_ptr(), M, M, packed[r % nsets],
                                                   C8[r % nsets].data_ptr(), M, 1, 1e-3, stream), args.reps)
                t32 = timed(lambda r: tw.tw_gemm_i8(A8[r % nsets].data_ptr(), M, M, packed[r % nsets],
                                                    C32[r % nsets].data_ptr(), M, 0, 1.0, stream), args.reps)
                td8 = timed(lambda r: tw.tw_dense_gemm_i8(A8[r % nsets].data_ptr(), Bd.data_ptr(), C8[r % nsets].data_ptr(),
                                                          M, K, N, M, N, M, 1, 1e-3, stream), args.reps)
                t16 = timed(lambda r: tw.tw_gemm(A16[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, p16[r % nsets],
                                                 C16[r % nsets].data_ptr(), M, stream), args.reps)
                # int8 A rows, int8 C, condensed bytes (TVW: the kept half + 2 bits per stored value), row lists
                ab8 = M * ku + M * N + (skw if pattern == "tw" else skw // 2 + skw // 8) + 4 * sk
                issued = (2.0 if pattern == "tw" else 1.0) * M * skw        # TVW: skw counts the rows before 2:4
                print(json.dumps(dict(
                    shape=shp.name, M=M, K=K, N=N, G=G, pattern=pattern + "_i8", sparsity=sp, K_union=ku,
                    us_i8_out=round(t8 * 1e6, 2), us_i32_out=round(t32 * 1e6, 2), dense_i8_us=round(td8 * 1e6, 2),
                    fp16_us=round(t16 * 1e6, 2), speedup_vs_dense_i8=round(td8 / t8, 3),
                    speedup_vs_fp16=round(t16 / t8, 3),
                    dense_eq_tops=round(2.0 * M * K * N / t8 / 1e12, 1),
                    condensed_mfma_util=round(issued / t8 / 5.0e15, 4),
                    alg_MB=round(ab8 / 1e6, 2), alg_GBps=round(ab8 / t8 / 1e9, 1),
                    roofline_frac=round(max(ab8 / HBM, issued / 5.0e15) / t8, 4))), flush=True)
                for p in packed + p16:
                    p.free()
                del A8, A16, C32, C8, C16

    if args.tew:
        for cfg, si in ((2, 0), (2, 1), (2, 2), (4, 0), (4, 1)):
            for delta in (0.005, 0.015, 0.05):
                plan.append((cfg, si, "tew", 0.75, 128, delta))

    dense_cache = {}
    for entry in plan:
        cfg, si, pattern, sp, G = entry[:5]
        delta = entry[5] if len(entry) > 5 else 0.0
        shp = wl.SHAPES[cfg][si]
        M, K, N = shp.M, shp.K, shp.N
        nsets = max(2, min(args.sets, int(600e6 // (2 * M * (K + N)))))
        cf = 0.0 if sp == 0.0 or (pattern == "tvw" and sp == 0.5) else None
        c = wl.make_case(cfg, si, pattern=pattern, sparsity=sp, G=G, col_frac=cf, with_A=False, delta=delta)
        pat = {"tw": tw.PATTERN_TW, "tvw": tw.PATTERN_TVW, "tew": tw.PATTERN_TEW}[pattern]
        packed = [tw.tw_pack(c.B, c.mask, G, pat, tile_mask=c.tile_mask if pattern != "tw" else None)
                  for _ in range(nsets)]
        nnz_ew = int(c.mask.sum() - c.tile_mask.sum()) if pattern == "tew" else 0
        A = [torch.randn((K, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
        C = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
        skw, sk, ku = packed[0].flop_counts()
        t = timed(lambda r: tw.tw_gemm(A[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % nsets],
                                       C[r % nsets].data_ptr(), M, stream), args.reps)
        key = (cfg, si)
        if key not in dense_cache:
            Bd = torch.from_numpy(c.B).to(dev)
            dense_cache[key] = timed(lambda r: tw.tw_dense_gemm(A[r % nsets].data_ptr(), Bd.data_ptr(),
                                                                C[r % nsets].data_ptr(), M, K, N, M, N, M,
                                                                tw.LAYOUT_KM, stream), args.reps)
        td = dense_cache[key]
        ab = alg_bytes(M, ku, N, "tw" if pattern == "tew" else pattern, skw, sk) + 4 * nnz_ew + (4 * (N + 1) if nnz_ew else 0)
        issued = 1.0 * M * skw if pattern == "tvw" else 2.0 * M * skw
        t_hbm, t_mfma = ab / HBM, issued / MFMA
        print(json.dumps(dict(
            shape=shp.name, M=M, K=K, N=N, G=G, pattern=pattern, sparsity=sp, K_union=ku,
            **(dict(delta=delta, restored=nnz_ew, ew_gather_MB=round(2.0 * M * nnz_ew / 1e6, 1)) if pattern == "tew" else {}),
            us=round(t * 1e6, 2), dense_us=round(td * 1e6, 2), speedup_vs_dense=round(td / t, 3),
            dense_eq_tflops=round(2.0 * M * K * N / t / 1e12, 1),
            condensed_mfma_util=round(2.0 * M * skw / t / MFMA, 4),
            alg_MB=round(ab / 1e6, 2), alg_GBps=round(ab / t / 1e9, 1),
            bound="hbm" if t_hbm >= t_mfma else "mfma",
            roofline_frac=round(max(t_hbm, t_mfma) / t, 4))), flush=True)
        for p in packed:
            p.free()
        del A, C


if __name__ == "__main__":
    sys.exit(main())
