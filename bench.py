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
`roofline` (the grouped GEMM kernel, HBM-bound at this sparsity) and
`cpu_baseline` (the fp64 oracle timed on the host cores).
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
FP16_PEAK_TFLOPS = 2500.0
# fp16 matrix-core rate reached on the box by a register-only v_mfma_f32_32x32x16_f16 loop
# (a microbenchmark, not part of this script): context for the utilisation figures
MEASURED_MFMA_LOOP_TFLOPS = 1970.0
PLAN = [(0, 4), (1, 1), (2, 1)]          # (shape index in the config, copies per layer)
# HBM-side bytes per launch (average over the launches of a step) from the two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) summarised under profiles/, scaled by
# what the same counters read for a plain 256 MiB device copy.  A measurement that
# cannot be taken from inside this script: None where no such run has been made.
MEASURED_TRAFFIC_BYTES = {("tw", False): None, ("tvw", False): None,
                          ("tw", True): 32.47e6, ("tvw", True): 29.45e6}   # key: (pattern, Q/K/V grouped)


def algorithmic_bytes(M, K_union, N, pattern, sum_kw, sum_k):
    """Bytes one launch must move: the rows of A that some tile keeps, once; all
    of C (pruned columns are written as zeros); the condensed weight (TVW: half
    the values plus 4 position bits per group and column) and its kept-row list."""
    w = 2 * sum_kw if pattern == "tw" else sum_kw + sum_kw // 8
    return 2 * M * K_union + 2 * M * N + w + 4 * sum_k


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--sets", type=int, default=12)
    ap.add_argument("--pattern", default="tw", choices=["tw", "tvw"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
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
    _build.ensure_built()                   # compiles only if no library has been built
    import paper_2402_10876_amd as tw
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    tw.tw_set_option("xcd_map", args.xcd_map)
    dev = torch.device("cuda:0")
    cfg = 2 if args.pattern == "tw" else 3
    shapes = wl.SHAPES[cfg]
    M = shapes[0].M
    stream = torch.cuda.current_stream().cuda_stream
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
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    sec_per_step = (time.perf_counter() - t0) / args.steps

    # ---- the same steps again, one pair of HIP events around the launches of each
    # step, recorded on the stream the kernels run on: elapsed / launches is the
    # average launch duration (back-to-back launches, so the gap between two
    # kernels is part of it)
    ev = []
    for i in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); step(i); e1.record()
        ev.append((e0, e1))
    torch.cuda.synchronize()
    launches = len(sets[0])
    avg_launch_ms = float(np.mean([a.elapsed_time(b) for a, b in ev])) / launches
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
    cond_flops_step = sum(2.0 * M * meta[si]["sum_kw"] * c for si, c in PLAN)
    value = dense_flops_step / sec_per_step / 1e12

    # ---- our own dense MFMA GEMM at the same shapes (outside the timed region) -----
    # The dense counterpart of the grouped launch is one 768 x 2304 GEMM on [Wq | Wk | Wv].
    detail = {}
    for key in [si for si, _ in PLAN] + ["qkv"]:
        mt = meta[key]
        Kk, Nn, which = mt["K"], mt["N"], (sets_grp if key == "qkv" else sets_sep)
        t_sp = per_shape_ms[key] * 1e-3
        d = dict(sparse_us=t_sp * 1e6, dense_eq_tflops=2.0 * M * Kk * Nn / t_sp / 1e12,
                 condensed_mfma_util=2.0 * M * mt["sum_kw"] / t_sp / 1e12 / FP16_PEAK_TFLOPS,
                 alg_GBps=mt["alg"] / t_sp / 1e9, alg_bytes=mt["alg"],
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

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()

    achieved = alg_per_launch / (avg_launch_ms * 1e-3) / 1e9
    kern = "tw_gemm_km_dma_kernel" if args.pattern == "tw" else "tvw_gemm_km_kernel"
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBS, traffic=MEASURED_TRAFFIC_BYTES[(args.pattern, grouped)],
                    kernel=f"{kern} (all {launches} launches of a step; the step runs nothing else)",
                    avg_launch_us=avg_launch_ms * 1e3, algorithmic_bytes_per_launch=alg_per_launch)

    out = dict(metric=f"{args.pattern.upper()} sparse GEMM effective (dense-equivalent) TFLOP/s, BERT-base layer",
               value=value, unit="TFLOP/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=sec_per_step * 1e3, higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16", data="synthetic",
               config=dict(workload=f"BERT-base linear layers as {args.pattern.upper()} GEMM (config {cfg}): M=4096, "
                                    "4x 768x768 + 768x3072 + 3072x768, "
                                    + ("Q/K/V as one grouped launch (4 launches per step), " if grouped else
                                       "6 launches per step, ") + "G=128, "
                                    + ("75 % sparsity (10 % columns + per-tile rows)" if args.pattern == "tw" else
                                       "87.5 % sparsity (tile-wise 75 % + 2:4)") + ", layout K x M / N x M",
                           sets=args.sets, pattern=args.pattern, launches_per_step=launches),
               condensed_flop_mfma_util=cond_flops_step / sec_per_step / 1e12 / FP16_PEAK_TFLOPS,
               condensed_flop_util_vs_measured_mfma_loop=cond_flops_step / sec_per_step / 1e12 / MEASURED_MFMA_LOOP_TFLOPS,
               pack_seconds_per_weight=t_pack / (args.sets * 6),
               roofline=roofline, detail=detail)

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
