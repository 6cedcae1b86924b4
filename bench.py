#!/usr/bin/env python3
"""Benchmark of the TW / TVW sparse GEMM hot path on one MI355X.

A step = the six linear-layer GEMMs of one BERT-base encoder layer at batch 32 x
sequence 128 (M = 4096): four 768x768 (Q, K, V, output), 768x3072 (FFN1) and
3072x768 (FFN2), with synthetic seeded weights pruned tile-wise (G = 128).
Q, K and V multiply the same activations and do not depend on one another: their
three separately pruned and packed weights are placed side by side with
tw_concat and run as ONE launch that reads A once and writes the three outputs
(4 launches per step).  `--separate-qkv` launches them one by one instead (6
launches per step, each with activations of its own); the default run reports
that variant too, under detail.separate_qkv.  Patterns:
  --pattern tw  : 75 % sparsity, 10 % of the columns plus magnitude-scored rows
                  per tile (the default, the configuration the metric is quoted on)
  --pattern tvw : the same tile-wise part plus 2:4 along the kept rows, 87.5 %
Each step works on its own set of activations, outputs and packed weights out of
`--sets` rotating sets (12 = one per encoder layer, about 1.4 GB in total), so
operands come from HBM rather than from the 256 MB last-level cache.

Prints ONE JSON line: dense-equivalent TFLOP/s of the whole step, plus
  roofline      the grouped GEMM kernel against the HBM roof, from the same timed loop
                (HIP events on the launch stream around the K steps);
  calibration   what this machine sustains for plain streams and register-only matrix-core
                loops (tw_calibrate kernels timed with events);
  rows          every other configured workload as one row each (BERT-base TVW, the
                BERT-large FFN sparsity sweep, the VGG-16 im2col GEMMs): time, our dense
                kernel's time, binding roof and the fraction of it (outside the timed region);
  cpu_baseline  the fp64 oracle timed on the host cores.
`--extra cube,imbalance,tew,i8,conv,options` adds opt-in sweeps (the 4096^3 sparsity sweep, uneven
tiles, TEW, int8, convolutions without a materialised img2col matrix) under `extra`.
`--calibrate` runs the calibration kernels alone (the command the rocprofv3 summary in
profiles/ was taken with).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PREWARM_S = 0.05            # untimed launches before each measurement (see main)
FP16_PEAK_TFLOPS = 2500.0
PLAN = [(0, 4), (1, 1), (2, 1)]          # (shape index in the config, copies per layer)
# HBM-side bytes per launch (average over the launches of a step), NOT measured by this run:
# they come from the two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this same command
# summarised in the file named beside them, scaled by what the same counters read for a plain
# 256 MiB device copy.  None where no such run has been made.
PROFILED_TRAFFIC = {("tw", True): (32.46e6, "profiles/tw_gemm_km_dma_kernel_bert_base_tw75.md"),
                    ("tvw", True): (29.45e6, "profiles/tvw_gemm_km_kernel_bert_base_tvw875.md")}


def algorithmic_bytes(M, K_union, N, pattern, sum_kw, sum_k):
    """Bytes one launch must move: the rows of A that some tile keeps, once; all
    of C (pruned columns are written as zeros); the condensed weight (TVW: half
    the values plus 4 position bits per group and column) and its kept-row list."""
    w = 2 * sum_kw if pattern == "tw" else sum_kw + sum_kw // 8
    return 2 * M * K_union + 2 * M * N + w + 4 * sum_k


def issued_flops(M, sum_kw, pattern):
    """Matrix-core work of a launch: 2 M sum(K_t W_t); the 2:4 instruction issues half of it."""
    return (1.0 if pattern == "tvw" else 2.0) * M * sum_kw


def roof(alg_bytes, flops, seconds):
    """Which published roof binds and the fraction of it that was reached."""
    t_hbm, t_mfma = alg_bytes / (HBM_PEAK_GBS * 1e9), flops / (FP16_PEAK_TFLOPS * 1e12)
    return ("hbm" if t_hbm >= t_mfma else "mfma"), max(t_hbm, t_mfma) / seconds


def calibration(tw, torch, dev, stream, quick=False):
    """Times the tw_calibrate kernels: GB/s of plain streams, TFLOP/s of register-only loops."""
    nbytes = (256 << 20) if quick else (1 << 30)
    src = torch.ones(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
    out = {}

    def timed(kind, n, iters=0, reps=5, chain=1):
        """units per second; chain > 1: that many launches back to back between the two events
        (per-launch time as in a stream of launches: the host-side launch latency of a single
        launch, about 4 us here, is hidden as it is in the benchmark's steps)"""
        best, units = None, 0.0
        for r in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(chain):
                units = tw.tw_calibrate(kind, dst.data_ptr(), src.data_ptr(), n, iters, stream)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / chain
            if r > 0 and (best is None or t < best):      # first round is a warm-up
                best = t
        return units / best
    out["copy_GBps"] = timed(tw.CAL_COPY, nbytes) / 1e9            # read + write bytes
    out["read_GBps"] = timed(tw.CAL_READ, nbytes) / 1e9
    out["write_GBps"] = timed(tw.CAL_WRITE, nbytes) / 1e9
    # What a launch that only writes C costs: zero fills in the epilogue's pattern at four sizes,
    # 16 launches back to back; time = fixed + bytes / rate by least squares.
    sizes = [768 * 4096 * 2, 3072 * 4096 * 2, 4 * 3072 * 4096 * 2, 8 * 3072 * 4096 * 2]
    us = [s / timed(tw.CAL_STORE_CT, s, reps=5, chain=16) * 1e6 for s in sizes]          # units == bytes written
    A = np.vstack([np.ones(len(sizes)), np.array(sizes, dtype=np.float64)]).T
    fixed_us, us_per_byte = np.linalg.lstsq(A, np.array(us), rcond=None)[0]
    out["store_ct_us_by_MB"] = {f"{s / 1e6:.1f}": round(t, 2) for s, t in zip(sizes, us)}
    out["store_ct_fixed_us"] = float(fixed_us)
    out["store_ct_fit_GBps"] = float(1e-3 / us_per_byte)
    out["single_launch_25MB_store_us"] = 3072 * 4096 * 2 / timed(tw.CAL_STORE_CT, 3072 * 4096 * 2, reps=10) * 1e6
    iters = 2000 if quick else 8000
    out["mfma_f16_TFLOPs"] = timed(tw.CAL_MFMA_F16, nbytes, iters) / 1e12
    out["smfmac_f16_dense_eq_TFLOPs"] = timed(tw.CAL_SMFMAC_F16, nbytes, iters) / 1e12
    out["mfma_i8_TOPs"] = timed(tw.CAL_MFMA_I8, nbytes, iters) / 1e12
    out["bytes"] = nbytes
    out["note"] = ("best of 5 rounds between HIP events (single launches; the store pattern as 16 launches "
                   "back to back); copy counts bytes read + written; matrix loops: 2048 workgroups x 4 waves x "
                   "4 accumulators, operands in registers")
    del src, dst
    return out


def extra_rows(tw, wl, torch, dev, stream, skip_cfg, reps=24, sets=24):
    """One row per other configured workload (launch configuration as the heuristics pick it),
    timed on enough rotating buffer sets (about 600 MB) that operands come from HBM."""
    def timed(fn, rounds=5):
        t_w = time.perf_counter()      # untimed: first touch of fresh buffers, clocks up after host-side packing
        while time.perf_counter() - t_w < PREWARM_S:
            for r in range(reps):
                fn(r)
            torch.cuda.synchronize()
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
    for cfg in (2, 3, 4, 5):
        if cfg == skip_cfg:
            continue
        for si in range(len(wl.SHAPES[cfg])):
            if cfg == 2:
                plan.append((cfg, si, "tw", 0.75, 128))
            elif cfg == 3:
                plan.append((cfg, si, "tvw", 0.875, 128))
            elif cfg == 4:
                plan += [(cfg, si, "tw", sp, 128) for sp in (0.0, 0.5, 0.75, 0.875, 0.9375)]
                plan += [(cfg, si, "tvw", sp, 128) for sp in (0.5, 0.75, 0.875, 0.9375)]
            else:
                plan += [(cfg, si, "tw", 0.75, 64), (cfg, si, "tw", 0.75, 128),
                         (cfg, si, "tvw", 0.875, 64), (cfg, si, "tvw", 0.875, 128)]
    rows, dense_us, bufs = [], {}, {}
    for cfg, si, pattern, sp, G in plan:
        shp = wl.SHAPES[cfg][si]
        M, K, N = shp.M, shp.K, shp.N
        nsets = max(2, min(sets, int(600e6 // (2 * M * (K + N)))))
        if (cfg, si) not in bufs:
            bufs.clear()                                   # one shape's buffers alive at a time
            bufs[(cfg, si)] = ([torch.randn((K, M), dtype=torch.float16, device=dev) for _ in range(nsets)],
                               [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(nsets)])
        A, C = bufs[(cfg, si)]
        cf = 0.0 if sp == 0.0 or (pattern == "tvw" and sp == 0.5) else None
        c = wl.make_case(cfg, si, pattern=pattern, sparsity=sp, G=G, col_frac=cf, with_A=False)
        pat = tw.PATTERN_TW if pattern == "tw" else tw.PATTERN_TVW
        packed = [tw.tw_pack(c.B, c.mask, G, pat, tile_mask=c.tile_mask if pattern == "tvw" else None)
                  for _ in range(nsets)]
        skw, sk, ku = packed[0].flop_counts()
        t = timed(lambda r: tw.tw_gemm(A[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % nsets],
                                       C[r % nsets].data_ptr(), M, stream))
        if (cfg, si) not in dense_us:
            Bd = torch.from_numpy(c.B).to(dev)
            dense_us[(cfg, si)] = timed(lambda r: tw.tw_dense_gemm(A[r % nsets].data_ptr(), Bd.data_ptr(),
                                                                   C[r % nsets].data_ptr(), M, K, N, M, N, M,
                                                                   tw.LAYOUT_KM, stream))
        td = dense_us[(cfg, si)]
        ab = algorithmic_bytes(M, ku, N, pattern, skw, sk)
        fl = issued_flops(M, skw, pattern)
        bound, frac = roof(ab, fl, t)
        rows.append(dict(config=cfg, shape=shp.name, M=M, K=K, N=N, G=G, pattern=pattern, sparsity=sp,
                         us=round(t * 1e6, 2), dense_us=round(td * 1e6, 2), speedup_vs_dense=round(td / t, 3),
                         dense_eq_tflops=round(2.0 * M * K * N / t / 1e12, 1),
                         # issued matrix-core work over the peak of the instruction that issues it
                         # (TVW: useful flops over the dense peak, the same number)
                         condensed_mfma_util=round(fl / t / 1e12 / FP16_PEAK_TFLOPS, 4),
                         alg_bytes=int(ab), alg_GBps=round(ab / t / 1e9, 1), bound=bound, frac=round(frac, 4)))
        for p in packed:
            p.free()
    bufs.clear()
    return rows


def extra_sweeps(tw, wl, torch, dev, stream, which, reps=24, sets=6):
    """Opt-in measurements beyond the configured workloads (`--extra cube,imbalance,tew,i8,conv`; `options` is handled in main, on the step's own buffers):
    the 4096^3 sparsity sweep of Section VI-B (TVW at 50 % is plain 2:4), uneven tiles from one
    magnitude threshold over all tile rows (Section V "load imbalance") launched longest first
    and in column order, TEW at 75 % with delta restored elements (Section VI, impact of delta),
    int8 TW / TVW against the dense int8 kernel and the fp16 launch of the same mask (Section
    VI-B), and config 5's convolutions on the wide input against the materialised matrix."""
    def timed(fn, rounds=5):
        t_w = time.perf_counter()      # untimed: first touch of fresh buffers, clocks up after host-side packing
        while time.perf_counter() - t_w < PREWARM_S:
            for r in range(reps):
                fn(r)
            torch.cuda.synchronize()
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
    out = {}
    wl.SHAPES[6] = [wl.Shape("cube_4096", 4096, 4096, 4096, 0.02)]
    wl.CONFIGS[6] = dict(G=128, pattern="tw", sparsity=0.75, col_frac=0.10)

    def gemm_rows(plan):
        rows, dense = [], {}
        for entry in plan:
            cfg, si, pattern, sp, G = entry[:5]
            delta = entry[5] if len(entry) > 5 else 0.0
            shp = wl.SHAPES[cfg][si]
            M, K, N = shp.M, shp.K, shp.N
            nsets = max(2, min(sets, int(600e6 // (2 * M * (K + N)))))
            cf = 0.0 if sp == 0.0 or (pattern == "tvw" and sp == 0.5) else None
            c = wl.make_case(cfg, si, pattern=pattern, sparsity=sp, G=G, col_frac=cf, with_A=False, delta=delta)
            pat = {"tw": tw.PATTERN_TW, "tvw": tw.PATTERN_TVW, "tew": tw.PATTERN_TEW}[pattern]
            packed = [tw.tw_pack(c.B, c.mask, G, pat, tile_mask=c.tile_mask if pattern != "tw" else None)
                      for _ in range(nsets)]
            A = [torch.randn((K, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
            C = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
            skw, sk, ku = packed[0].flop_counts()
            t = timed(lambda r: tw.tw_gemm(A[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % nsets],
                                           C[r % nsets].data_ptr(), M, stream))
            if (cfg, si) not in dense:
                Bd = torch.from_numpy(c.B).to(dev)
                dense[(cfg, si)] = timed(lambda r: tw.tw_dense_gemm(A[r % nsets].data_ptr(), Bd.data_ptr(),
                                                                    C[r % nsets].data_ptr(), M, K, N, M, N, M,
                                                                    tw.LAYOUT_KM, stream))
            td = dense[(cfg, si)]
            nnz_ew = int(c.mask.sum() - c.tile_mask.sum()) if pattern == "tew" else 0
            ab = algorithmic_bytes(M, ku, N, "tvw" if pattern == "tvw" else "tw", skw, sk) + 4 * nnz_ew
            bound, frac = roof(ab, issued_flops(M, skw, pattern), t)
            row = dict(shape=shp.name, M=M, K=K, N=N, G=G, pattern=pattern, sparsity=sp, us=round(t * 1e6, 2),
                       dense_us=round(td * 1e6, 2), speedup_vs_dense=round(td / t, 3),
                       dense_eq_tflops=round(2.0 * M * K * N / t / 1e12, 1), bound=bound, frac=round(frac, 4))
            if pattern == "tew":
                row.update(delta=delta, restored=nnz_ew)
            rows.append(row)
            for p in packed:
                p.free()
        return rows

    if "cube" in which:
        plan = [(6, 0, "tw", sp, G) for sp in (0.0, 0.1, 0.25, 0.5, 0.75, 0.875) for G in (128, 64)]
        plan += [(6, 0, "tvw", sp, 128) for sp in (0.5, 0.75, 0.875)]
        out["cube"] = gemm_rows(plan)
    if "tew" in which:
        out["tew"] = gemm_rows([(cfg, si, "tew", 0.75, 128, delta) for cfg, si in ((2, 0), (2, 1), (2, 2), (4, 0), (4, 1))
                                for delta in (0.005, 0.015, 0.05)])
    if "imbalance" in which:
        rows = []
        for cfg, si in ((4, 0), (4, 1), (6, 0)):
            shp = wl.SHAPES[cfg][si]
            M, K, N = shp.M, shp.K, shp.N
            nsets = max(2, min(sets, int(600e6 // (2 * M * (K + N)))))
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
                else:
                    c = wl.make_case(cfg, si, pattern="tw", sparsity=0.75, G=128, recipe=recipe, with_A=False)
                    Bs, mask = c.B, c.mask
                row = dict(shape=shp.name, M=M, K=K, N=N, G=128, pattern="tw", sparsity=0.75, recipe=recipe)
                for order in (1, 0):
                    tw.tw_set_option("tile_order", order)
                    packed = [tw.tw_pack(Bs, mask, 128, tw.PATTERN_TW) for _ in range(nsets)]
                    t = timed(lambda r: tw.tw_gemm(A[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % nsets],
                                                   C[r % nsets].data_ptr(), M, stream))
                    kt = np.array([len(r) for r in packed[0].export()["row_idx"]])
                    row.update({("us_longest_first" if order else "us_column_order"): round(t * 1e6, 2),
                                "K_t_min": int(kt.min()), "K_t_mean": round(float(kt.mean()), 1), "K_t_max": int(kt.max())})
                    for p in packed:
                        p.free()
                tw.tw_set_option("tile_order", 1)
                rows.append(row)
            del A, C
        out["imbalance"] = rows
    if "conv" in which:
        rows = []
        for si, (name, g, N) in enumerate(wl.CONV_LAYERS):
            M, K, Mp, ldx = g.B * g.H * g.W, g.K, g.Mp, wl.conv_ldx(g)
            ns_conv = max(2, min(24, int(600e6 // (2 * (g.C * ldx + N * Mp)))))
            ns_mat = max(2, min(sets, int(600e6 // (2 * M * (K + N)))))
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
                bound_ = [tw.tw_conv_bind(p, g, ldx) for p in packed]
                skw, sk, ku = packed[0].flop_counts()
                t_conv = timed(lambda r: tw.tw_conv_gemm(X[r % ns_conv].data_ptr(), bound_[r % ns_conv],
                                                         Cw[r % ns_conv].data_ptr(), Mp, stream))
                t_mat = timed(lambda r: tw.tw_gemm(A[r % ns_mat].data_ptr(), M, M, tw.LAYOUT_KM, packed[r % ns_mat],
                                                   Cm[r % ns_mat].data_ptr(), M, stream))
                wbytes = 2 * skw if pattern == "tw" else skw + skw // 8
                ab = 2 * g.C * Mp + 2 * N * Mp + wbytes + 4 * sk       # the input once, C over the wide grid, weight
                rows.append(dict(shape=name, positions=M, wide_grid=Mp, K=K, N=N, G=G, pattern=pattern, sparsity=sp,
                                 us_implicit=round(t_conv * 1e6, 2), us_materialised=round(t_mat * 1e6, 2),
                                 input_MB=round(2 * g.C * Mp / 1e6, 2), materialised_A_MB=round(2 * M * ku / 1e6, 2),
                                 alg_MB=round(ab / 1e6, 2), alg_GBps=round(ab / t_conv / 1e9, 1)))
                for b in bound_:
                    b.free()
                for p in packed:
                    p.free()
            del X, Cw, A, Cm
        out["conv"] = rows
    if "i8" in which:
        rows = []
        for cfg, si in [(2, 0), (2, 1), (2, 2), (4, 0), (4, 1)]:
            shp = wl.SHAPES[cfg][si]
            M, K, N, G = shp.M, shp.K, shp.N, 128
            nsets = max(2, min(sets, int(600e6 // (M * (K + 4 * N)))))
            B8 = wl.rng_i8(wl.seed_for(cfg, si) + 1, (K, N))
            for pattern, sp in (("tw", 0.75), ("tw", 0.875), ("tvw", 0.875)):
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
                C8 = [torch.empty((N, M), dtype=torch.int8, device=dev) for _ in range(nsets)]
                C16 = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(nsets)]
                Bd = torch.from_numpy(B8).to(dev)
                t8 = timed(lambda r: tw.tw_gemm_i8(A8[r % nsets].data_ptr(), M, M, packed[r % nsets],
                                                   C8[r % nsets].data_ptr(), M, 1, 1e-3, stream))
                td8 = timed(lambda r: tw.tw_dense_gemm_i8(A8[r % nsets].data_ptr(), Bd.data_ptr(), C8[r % nsets].data_ptr(),
                                                          M, K, N, M, N, M, 1, 1e-3, stream))
                t16 = timed(lambda r: tw.tw_gemm(A16[r % nsets].data_ptr(), M, M, tw.LAYOUT_KM, p16[r % nsets],
                                                 C16[r % nsets].data_ptr(), M, stream))
                rows.append(dict(shape=shp.name, M=M, K=K, N=N, G=G, pattern=pattern + "_i8", sparsity=sp,
                                 us_i8_out=round(t8 * 1e6, 2), dense_i8_us=round(td8 * 1e6, 2), fp16_us=round(t16 * 1e6, 2),
                                 speedup_vs_dense_i8=round(td8 / t8, 3), speedup_vs_fp16=round(t16 / t8, 3),
                                 dense_eq_tops=round(2.0 * M * K * N / t8 / 1e12, 1)))
                for p in packed + p16:
                    p.free()
                del A8, A16, C8, C16
        out["i8"] = rows
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--sets", type=int, default=12)
    ap.add_argument("--pattern", default="tw", choices=["tw", "tvw"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-rows", action="store_true", help="skip the rows of the other configured workloads")
    ap.add_argument("--no-calibration", action="store_true")
    ap.add_argument("--extra", default="", help="comma list of opt-in sweeps, printed under `extra`: "
                                                "cube, imbalance, tew, i8, conv, options (each takes 10-60 s)")
    ap.add_argument("--calibrate", action="store_true", help="run the calibration kernels only and print their rates")
    ap.add_argument("--separate-qkv", action="store_true",
                    help="time the step with Q, K and V as three launches (6 launches per step)")
    ap.add_argument("--xcd-map", type=int, default=1, choices=[0, 1],
                    help="0 switches the XCD-aware workgroup order off (for counter comparisons)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of 256 MiB (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2402_10876_amd import build as _build
    _build.ensure_built()                   # compiles only if the library does not match the sources
    import paper_2402_10876_amd as tw
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    if args.calibrate:
        print(json.dumps(dict(calibration=calibration(tw, torch, dev, stream), library=_build.describe())))
        return
    tw.tw_set_option("xcd_map", args.xcd_map)
    cfg = 2 if args.pattern == "tw" else 3
    shapes = wl.SHAPES[cfg]
    M = shapes[0].M
    pat = tw.PATTERN_TW if args.pattern == "tw" else tw.PATTERN_TVW

    # ---- rotating sets: packed weights, A^T, C^T ----------------------------
    # An op is (key, packed, A^T, C^T); key = shape index, or "qkv" for the grouped launch.
    t_pack = 0.0
    sets_sep, sets_grp, meta, case_cache = [], [], {}, {}
    gen = torch.Generator(device="cpu").manual_seed(1234)
    for s in range(args.sets):
        ops = []
        for si, copies in PLAN:
            shp = shapes[si]
            for cidx in range(copies):
                variant = (s * 4 + cidx) % 10
                if (si, variant) not in case_cache:
                    case_cache[(si, variant)] = wl.make_case(cfg, si, variant=variant, with_A=False)
                c = case_cache[(si, variant)]
                t0 = time.perf_counter()
                packed = tw.tw_pack(c.B, c.mask, c.G, pat, tile_mask=c.tile_mask if args.pattern == "tvw" else None)
                t_pack += time.perf_counter() - t0
                skw, sk, ku = packed.flop_counts()
                meta[si] = dict(K=shp.K, N=shp.N, sum_kw=skw, sum_k=sk, k_union=ku, name=shp.name,
                                alg=algorithmic_bytes(M, ku, shp.N, args.pattern, skw, sk))
                At = torch.randn((shp.K, M), generator=gen, dtype=torch.float32).to(torch.float16).to(dev)
                Ct = torch.empty((shp.N, M), dtype=torch.float16, device=dev)
                ops.append((si, packed, At, Ct))
        sets_sep.append(ops)
        # Q, K, V (the first three 768x768 weights of the set) side by side, on Q's activations
        qkv = tw.tw_concat([o[1] for o in ops[:3]])
        skw, sk, ku = qkv.flop_counts()
        Nq = 3 * shapes[0].N
        meta["qkv"] = dict(K=shapes[0].K, N=Nq, sum_kw=skw, sum_k=sk, k_union=ku, name="bert_base_qkv_grouped",
                           alg=algorithmic_bytes(M, ku, Nq, args.pattern, skw, sk))
        sets_grp.append([("qkv", qkv, ops[0][2], torch.empty((Nq, M), dtype=torch.float16, device=dev))] + ops[3:])
    torch.cuda.synchronize()
    grouped = not args.separate_qkv
    sets = sets_grp if grouped else sets_sep

    def launch(o):
        tw.tw_gemm(o[2].data_ptr(), M, M, tw.LAYOUT_KM, o[1], o[3].data_ptr(), M, stream)

    def step(i, which=None):
        for o in (which or sets)[i % args.sets]:
            launch(o)

    # ---- the timed region -------------------------------------------------------
    # Wall clock between two synchronisations around exactly `steps` steps gives ms_per_step and
    # `value`; one pair of HIP events recorded on the launch stream inside the same region
    # (first thing after the opening synchronisation, last thing before the closing one) gives
    # the device-side span of the same launches: span / launches is the average launch duration
    # of the roofline (back-to-back launches, so the gap between two kernels is part of it).
    # Before the W warm-up steps: the same steps, untimed, for PREWARM_S seconds.  The weights were
    # just packed on the host, the GPU sat idle meanwhile, and its clocks take tens of milliseconds
    # of work to come back up; a short run (few steps, few warm-up steps) would time that ramp.
    t_w = time.perf_counter()
    prewarm_steps = 0
    while time.perf_counter() - t_w < PREWARM_S:
        for i in range(args.sets):
            step(i)
        prewarm_steps += args.sets
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    sec_per_step = (time.perf_counter() - t0) / args.steps
    launches = len(sets[0])
    avg_launch_ms = ev0.elapsed_time(ev1) / (args.steps * launches)
    alg_per_launch = sum(meta[o[0]]["alg"] for o in sets[0]) / launches

    # ---- the other variant of the step, for the record (outside the timed region) ----
    def time_steps(which):
        for i in range(args.warmup):
            step(i, which)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, which)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps
    sec_other = time_steps(sets_sep if grouped else sets_grp)

    # ---- per shape: 24 back-to-back launches between two events, rotating sets ----
    def time_shape(key, fn, reps=24, rounds=5, which=None):
        best = []
        for _ in range(rounds):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for r in range(reps):
                pool = which or sets_sep
                fn([x for x in pool[r % len(pool)] if x[0] == key][0])
            e1.record()
            torch.cuda.synchronize()
            best.append(e0.elapsed_time(e1) / reps)
        return float(np.median(best))
    per_shape_ms = {si: time_shape(si, launch) for si, _ in PLAN}
    per_shape_ms["qkv"] = time_shape("qkv", launch, which=sets_grp)
    # the same launches on ONE set of buffers: operands stay in the 256 MB last-level cache
    hot_ms = {si: time_shape(si, launch, which=sets_sep[:1]) for si, _ in PLAN}
    hot_ms["qkv"] = time_shape("qkv", launch, which=sets_grp[:1])

    dense_flops_step = sum(2.0 * M * shapes[si].K * shapes[si].N * c for si, c in PLAN)
    issued_step = sum(issued_flops(M, meta[si]["sum_kw"], args.pattern) * c for si, c in PLAN)
    value = dense_flops_step / sec_per_step / 1e12

    # ---- our own dense MFMA GEMM at the same shapes (outside the timed region) -----
    # The dense counterpart of the grouped launch is one 768 x 2304 GEMM on [Wq | Wk | Wv].
    detail = {}
    for key in [si for si, _ in PLAN] + ["qkv"]:
        mt = meta[key]
        Kk, Nn, which = mt["K"], mt["N"], (sets_grp if key == "qkv" else sets_sep)
        t_sp = per_shape_ms[key] * 1e-3
        fl = issued_flops(M, mt["sum_kw"], args.pattern)
        bound, frac = roof(mt["alg"], fl, t_sp)
        d = dict(sparse_us=t_sp * 1e6, dense_eq_tflops=2.0 * M * Kk * Nn / t_sp / 1e12,
                 condensed_mfma_util=fl / t_sp / 1e12 / FP16_PEAK_TFLOPS,
                 alg_GBps=mt["alg"] / t_sp / 1e9, alg_bytes=mt["alg"], bound=bound, frac=frac,
                 sparse_us_cache_resident=hot_ms[key] * 1e3)
        if not args.no_dense:
            Bd = torch.from_numpy(wl.make_B(wl.seed_for(cfg, 0 if key == "qkv" else key), Kk, Nn, 0.02)).to(dev)
            t_d = time_shape(key, lambda o: tw.tw_dense_gemm(o[2].data_ptr(), Bd.data_ptr(), o[3].data_ptr(), M, Kk,
                                                             Nn, M, Nn, M, tw.LAYOUT_KM, stream), which=which) * 1e-3
            d.update(dense_us=t_d * 1e6, dense_tflops=2.0 * M * Kk * Nn / t_d / 1e12,
                     speedup_vs_dense=t_d / t_sp)
            # context only, never the baseline: the vendor GEMM behind torch.matmul on the
            # same shape (row-major A, M x K), timed the same way
            Arm = [y for y in which[0] if y[0] == key][0][2].t().contiguous()
            out_rm = torch.empty((M, Nn), dtype=torch.float16, device=dev)
            t_v = time_shape(key, lambda o: torch.matmul(Arm, Bd, out=out_rm), which=which) * 1e-3
            d.update(vendor_gemm_us=t_v * 1e6)
        detail[mt["name"]] = d
    if not args.no_dense:
        keys_grp, keys_sep = ["qkv", 0, 1, 2], [0, 0, 0, 0, 1, 2]
        us = lambda keys, f: sum(detail[meta[k]["name"]][f] for k in keys)
        detail["step_speedup_vs_own_dense"] = (us(keys_grp, "dense_us") / us(keys_grp, "sparse_us") if grouped
                                               else us(keys_sep, "dense_us") / us(keys_sep, "sparse_us"))
    other = dict(launches_per_step=len((sets_sep if grouped else sets_grp)[0]), ms_per_step=sec_other * 1e3,
                 value=dense_flops_step / sec_other / 1e12)
    detail["separate_qkv" if grouped else "grouped_qkv"] = other

    options_sweep = None
    if "options" in set(args.extra.split(",")):
        # the step itself with one process-wide launch option forced at a time (the value
        # listed first is the default), values interleaved over 7 rounds of `steps` steps
        plan = [("idx_route", (0, 1, 2)), ("xcd_map", (1, 2, 0)), ("depth", (3, 4)), ("tile_m", (0, 64, 128, 256)),
                ("ksplit", (0, 1, 2)), ("waves", (4, 8))]
        res = {}
        for name, values in plan:
            t = {v: [] for v in values}
            for _ in range(7):
                for v in values:
                    tw.tw_set_option(name, v)
                    for i in range(args.warmup):
                        step(i)
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for i in range(args.steps):
                        step(i)
                    e1.record()
                    torch.cuda.synchronize()
                    t[v].append(e0.elapsed_time(e1) / args.steps * 1e3)
            tw.tw_set_option(name, values[0])
            res[name] = {str(v): round(float(np.median(t[v])), 2) for v in values}
        options_sweep = dict(us_per_step=res, note="median of 7 interleaved rounds; first value = default")

    # release the step's buffers before the other workloads allocate theirs
    for ops in sets_grp:
        ops[0][1].free()
    for ops in sets_sep:
        for o in ops:
            o[1].free()
    del sets, sets_sep, sets_grp
    torch.cuda.empty_cache()

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cal = None if args.no_calibration else calibration(tw, torch, dev, stream, quick=True)
    rows = None if args.no_rows else extra_rows(tw, wl, torch, dev, stream, skip_cfg=cfg)

    achieved = alg_per_launch / (avg_launch_ms * 1e-3) / 1e9
    kern = "tw_gemm_km_dma_kernel" if args.pattern == "tw" else "tvw_gemm_km_kernel"
    traffic, traffic_src = PROFILED_TRAFFIC.get((args.pattern, grouped), (None, None))
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBS, traffic=traffic, traffic_source=traffic_src,
                    kernel=f"{kern} (all {launches} launches of a step; the step runs nothing else)",
                    avg_launch_us=avg_launch_ms * 1e3, wall_us_per_launch=sec_per_step * 1e6 / launches,
                    algorithmic_bytes_per_launch=alg_per_launch,
                    timing="HIP events on the launch stream around the same K steps that ms_per_step times")
    if cal:
        roofline.update(measured_copy_GBps=cal["copy_GBps"], frac_vs_measured_copy=achieved / cal["copy_GBps"])
    util = issued_step / sec_per_step / 1e12 / FP16_PEAK_TFLOPS
    roofline["note"] = (f"HBM-bound at this sparsity: the matrix-core roof of the step is "
                        f"{issued_step / (FP16_PEAK_TFLOPS * 1e12) * 1e6:.1f} us against "
                        f"{alg_per_launch * launches / (HBM_PEAK_GBS * 1e9) * 1e6:.1f} us for its bytes; "
                        f"condensed-FLOP matrix-core utilisation {util:.3f} (goal 0.60 not met: it is capped "
                        f"by the byte roof on these shapes)")

    out = dict(metric=f"{args.pattern.upper()} sparse GEMM effective (dense-equivalent) TFLOP/s, BERT-base layer",
               value=value, unit="TFLOP/s", n_gpus=1, steps=args.steps, warmup=args.warmup, prewarm_steps=prewarm_steps,
               ms_per_step=sec_per_step * 1e3, higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16", data="synthetic",
               config=dict(workload=f"BERT-base linear layers as {args.pattern.upper()} GEMM (config {cfg}): M=4096, "
                                    "4x 768x768 + 768x3072 + 3072x768, "
                                    + ("Q/K/V as one grouped launch (4 launches per step), " if grouped else
                                       "6 launches per step, ") + "G=128, "
                                    + ("75 % sparsity (10 % columns + per-tile rows)" if args.pattern == "tw" else
                                       "87.5 % sparsity (tile-wise 75 % + 2:4)") + ", layout K x M / N x M",
                           sets=args.sets, pattern=args.pattern, launches_per_step=launches),
               condensed_flop_mfma_util=util,
               pack_seconds_per_weight=t_pack / (args.sets * 6), library=_build.describe(),
               roofline=roofline, detail=detail)
    if cal:
        out["calibration"] = cal
        out["condensed_flop_util_vs_measured_mfma_loop"] = (
            issued_step / sec_per_step / 1e12 /
            (cal["mfma_f16_TFLOPs"] if args.pattern == "tw" else cal["smfmac_f16_dense_eq_TFLOPs"] / 2.0))
    if rows is not None:
        out["rows"] = rows
    if args.extra:
        which_extra = set(args.extra.split(","))
        out["extra"] = extra_sweeps(tw, wl, torch, dev, stream, which_extra - {"options"})
        if options_sweep is not None:
            out["extra"]["options"] = options_sweep

    if not args.no_cpu_baseline:
        from oracle import gemm as og
        cases = [(wl.make_case(cfg, si), copies) for si, copies in PLAN]
        reps = []
        for _ in range(3):
            t0 = time.perf_counter()
            for c, copies in cases:
                for _ in range(copies):
                    og.gemm_oracle(c.A, c.B, c.mask)
            reps.append(time.perf_counter() - t0)
        tcpu = float(np.median(reps))
        try:
            import threadpoolctl
            cores = max(p["num_threads"] for p in threadpoolctl.threadpool_info()) or os.cpu_count()
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = dict(value=dense_flops_step / tcpu / 1e12, unit="TFLOP/s", cores=int(cores),
                                   kind="oracle", sample="one full step (6 GEMMs, full M=4096), fp64 NumPy matmul on the "
                                                         "masked dense weight, median of 3", seconds=tcpu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
