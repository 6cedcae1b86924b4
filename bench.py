#!/usr/bin/env python3
"""Benchmark of the TW sparse GEMM hot path on one MI355X.

A step = the six linear-layer GEMMs of one BERT-base encoder layer at batch 32 x
sequence 128 (M = 4096): four 768x768 (Q, K, V, output), 768x3072 (FFN1) and
3072x768 (FFN2), weights pruned tile-wise to 75 % (G = 128, 10 % of the columns
plus magnitude-scored rows per tile), synthetic seeded data.  Each step works on
its own set of activations, outputs and packed weights out of `--sets` rotating
sets (12 = one per encoder layer, about 1.4 GB in total), so operands come from
HBM rather than from the 256 MB last-level cache.

Prints ONE JSON line: dense-equivalent TFLOP/s of the whole step, plus
`roofline` (dominant kernel = the FFN1-shaped launch, HBM-bound) and
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


def layer_shapes():
    import workloads as wl
    s = wl.SHAPES[2]
    # (shape_index, copies per layer)
    return [(0, 4), (1, 1), (2, 1)], s


def algorithmic_bytes(M, K, N, sum_kw, sum_k):
    """Bytes one TW launch must move: A once, all of C (pruned columns are
    written as zeros), the condensed weight with its row index list."""
    return 2 * M * K + 2 * M * N + 2 * sum_kw + 4 * sum_k


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--sets", type=int, default=12)
    ap.add_argument("--pattern", default="tw", choices=["tw"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2402_10876_amd as tw
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    plan, shapes = layer_shapes()
    M = shapes[0].M
    stream = torch.cuda.current_stream().cuda_stream

    # ---- build the rotating sets: packed weights, A^T, C^T ------------------
    t_pack = 0.0
    sets = []
    meta = {}
    gen = torch.Generator(device="cpu").manual_seed(1234)
    case_cache = {}
    for s in range(args.sets):
        ops = []
        for si, copies in plan:
            shp = shapes[si]
            for cidx in range(copies):
                variant = (s * 4 + cidx) % 10
                if (si, variant) not in case_cache:
                    case_cache[(si, variant)] = wl.make_case(2, si, variant=variant, with_A=False)
                c = case_cache[(si, variant)]
                t0 = time.perf_counter()
                packed = tw.tw_pack(c.B, c.mask, c.G, tw.PATTERN_TW)
                t_pack += time.perf_counter() - t0
                skw, sk = packed.flop_counts()
                meta[si] = dict(K=shp.K, N=shp.N, sum_kw=skw, sum_k=sk, name=shp.name)
                At = (torch.randn((shp.K, M), generator=gen, dtype=torch.float32)).to(torch.float16).to(dev)
                Ct = torch.empty((shp.N, M), dtype=torch.float16, device=dev)
                ops.append((si, packed, At, Ct))
        sets.append(ops)
    torch.cuda.synchronize()

    def step(i, ev=None):
        for si, packed, At, Ct in sets[i % args.sets]:
            if ev is not None and si == 1:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                tw.tw_gemm(At.data_ptr(), M, M, tw.LAYOUT_KM, packed, Ct.data_ptr(), M, stream)
                e1.record()
                ev.append((e0, e1))
            else:
                tw.tw_gemm(At.data_ptr(), M, M, tw.LAYOUT_KM, packed, Ct.data_ptr(), M, stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev = []
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, ev)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps
    dom_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))

    dense_flops_step = sum(2.0 * M * shapes[si].K * shapes[si].N * copies for si, copies in plan)
    cond_flops_step = sum(2.0 * M * meta[si]["sum_kw"] * copies for si, copies in plan)
    value = dense_flops_step / sec_per_step / 1e12

    # ---- per-shape kernel times (events around back-to-back launches, rotating sets)
    def time_shape(si, fn, reps=60):
        evs = []
        for r in range(reps + 10):
            ops = [o for o in sets[r % args.sets] if o[0] == si]
            o = ops[0]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(o); e1.record()
            if r >= 10:
                evs.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e-3

    detail = {}
    dense_B = {}
    for si, copies in plan:
        shp = shapes[si]
        t_tw = time_shape(si, lambda o: tw.tw_gemm(o[2].data_ptr(), M, M, tw.LAYOUT_KM, o[1], o[3].data_ptr(), M, stream))
        d = dict(tw_us=t_tw * 1e6, dense_eq_tflops=2.0 * M * shp.K * shp.N / t_tw / 1e12,
                 condensed_mfma_util=2.0 * M * meta[si]["sum_kw"] / t_tw / 1e12 / FP16_PEAK_TFLOPS,
                 alg_GBps=algorithmic_bytes(M, shp.K, shp.N, meta[si]["sum_kw"], meta[si]["sum_k"]) / t_tw / 1e9)
        if not args.no_dense:
            Bd = wl.make_B(wl.seed_for(2, si), shp.K, shp.N, shp.sigma)
            dense_B[si] = torch.from_numpy(Bd).to(dev)
            t_d = time_shape(si, lambda o: tw.tw_dense_gemm(o[2].data_ptr(), dense_B[si].data_ptr(), o[3].data_ptr(),
                                                            M, shp.K, shp.N, M, shp.N, M, tw.LAYOUT_KM, stream))
            d.update(dense_us=t_d * 1e6, dense_tflops=2.0 * M * shp.K * shp.N / t_d / 1e12, speedup_vs_dense=t_d / t_tw)
        detail[shp.name] = d
    if not args.no_dense:
        t_dense_step = sum(detail[shapes[si].name]["dense_us"] * copies for si, copies in plan)
        t_tw_step = sum(detail[shapes[si].name]["tw_us"] * copies for si, copies in plan)
        detail["step_speedup_vs_dense_kernel_sum"] = t_dense_step / t_tw_step

    m1 = meta[1]
    alg = algorithmic_bytes(M, m1["K"], m1["N"], m1["sum_kw"], m1["sum_k"])
    achieved = alg / (dom_ms * 1e-3) / 1e9
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBS, traffic=None,
                    kernel="tw_gemm_km_kernel (bert_base_ffn1, TW 75 %)",
                    avg_launch_us=dom_ms * 1e3, algorithmic_bytes=alg)

    out = dict(metric="TW sparse GEMM effective (dense-equivalent) TFLOP/s, BERT-base layer at 75 % sparsity",
               value=value, unit="TFLOP/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=sec_per_step * 1e3, higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16", data="synthetic",
               config=dict(workload="BERT-base linear layers as TW GEMM (config 2): M=4096, 4x 768x768 + 768x3072 + 3072x768, "
                                    "G=128, 75 % sparsity (10 % columns + per-tile rows), layout K x M / N x M",
                           sets=args.sets, pattern="tw"),
               condensed_flop_mfma_util=cond_flops_step / sec_per_step / 1e12 / FP16_PEAK_TFLOPS,
               pack_seconds_per_weight=t_pack / (args.sets * 6),
               roofline=roofline, detail=detail)

    if not args.no_cpu_baseline:
        from oracle import gemm as og
        cases = [(wl.make_case(2, si), copies) for si, copies in plan]
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
