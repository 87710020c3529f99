#!/usr/bin/env python3
"""Benchmark of the SparseGemv hot path on one MI355X.

A step is one `egt_sparse_gemv` call (stage x, stream the 2bit-CSR row data,
dequantise, gather, multiply-accumulate, reduce, store) on the headline workload:
W 11008 x 4096, 2:4 sparse, INT4 group 128, 2bit-CSR; x FP16; M = 1.  Inputs are
resident in HBM before the timed region.  Consecutive steps cycle over enough
distinct device copies of the packed matrix to exceed twice the 256 MB last-level
cache, so every launch streams its weights from HBM.

Prints ONE JSON line (see README / DESIGN for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
LLC_BYTES = 256 << 20
# HBM bytes per launch of the headline kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/sparse_m1_headline_hbm_traffic.txt): 9066.7 * 2 KiB read + 21.5 KiB written.
MEASURED_TRAFFIC_BYTES = round(9066.7 * 2048 + 21.5 * 1024)


def algorithmic_bytes(rows, cols, n_keep, group, kind, m=1):
    """Bytes the method itself has to move per call: the four buffers of the
    matrix (row_ptr[R] only), x once, y once."""
    slots = rows * n_keep * cols // 4
    val = slots // 2 if kind == 0 else 2 * slots
    idx = slots // 4
    qp = 4 * rows * (cols // group) if kind == 0 else 0
    return val + idx + qp + 4 * rows + 4 + m * 2 * cols + m * 2 * rows


def dense_int4_bytes(rows, cols, group):
    return rows * cols // 2 + 4 * rows * (cols // group) + 2 * cols + 2 * rows


def time_loop(torch, fn, steps, warmup):
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return e0.elapsed_time(e1) * 1e-3 / steps, wall / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extra", action="store_true", help="also time the other configurations")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a 64 MiB device copy ten times (known traffic, for scaling rocprofv3 counters)")
    ap.add_argument("--counter-workloads", action="store_true",
                    help="also launch the other kernels 40 times each on the 11008x4096 shape, untimed "
                         "(FP16 values, 1:4, M > 1), for rocprofv3 counter runs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_11582_amd import binding as B, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    R, K, N, GRP = 11008, 4096, 2, 128
    seed = synth.seed_for(synth.HEADLINE)
    w = synth.weights(R, K, seed)
    x = synth.activations(K, seed)
    mask = B.prune_n4(w, N)
    p = B.pack_2bitcsr(w, mask, N, GRP, B.VAL_INT4)
    nbytes = algorithmic_bytes(R, K, N, GRP, 0)
    copies = max(2, -(-2 * LLC_BYTES // p.nbytes()))
    packed = [p.to(dev) for _ in range(copies)]
    xd = torch.from_numpy(x.view(np.int16)).to(dev).view(torch.float16)
    ys = [torch.empty(R, dtype=torch.float16, device=dev) for _ in range(copies)]

    calls = [B.prepared_sparse_gemv(packed[i], xd, ys[i]) for i in range(copies)]

    def step(i):
        calls[i % copies]()

    t_dev, t_wall = time_loop(torch, step, args.steps, args.warmup)

    # read ceiling: a plain 128-bit streaming read of the same number of bytes, same rotation
    pool = [torch.empty(p.nbytes(), dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(copies)]
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    nb16 = p.nbytes() // 16 * 16
    reads = [B.prepared_stream_read(pool[i], nb16, sink) for i in range(copies)]
    t_read, _ = time_loop(torch, lambda i: reads[i % copies](), args.steps, args.warmup)
    tiny = B.prepared_stream_read(pool[0], 16, sink)
    t_tiny, _ = time_loop(torch, lambda i: tiny(), args.steps, args.warmup)
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    t_big, _ = time_loop(torch, lambda i: B.stream_read(big, 1 << 30, sink), 20, 3)
    del big, pool, reads

    if args.calibrate:
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.counter_workloads:
        def launches(pk_host, Ms):
            n = max(2, -(-2 * LLC_BYTES // pk_host.nbytes()))
            pks = [pk_host.to(dev) for _ in range(n)]
            for M in Ms:
                Xm = torch.from_numpy(synth.activation_rows(M, K, seed + M).view(np.int16)).to(dev).view(torch.float16)
                Ym = torch.empty((M, R), dtype=torch.float16, device=dev)
                fs = [B.prepared_sparse_gemv(pks[i], Xm[0], Ym[0]) if M == 1 else
                      B.prepared_sparse_gemm_smallm(pks[i], Xm, Ym) for i in range(n)]
                for i in range(40):
                    fs[i % n]()
                torch.cuda.synchronize()
        launches(B.pack_2bitcsr(w, mask, N, 0, B.VAL_FP16), (1, 2, 4, 16))
        launches(B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, 0, B.VAL_FP16), (1,))
        launches(p, (2, 16, 64))
        launches(B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, GRP, B.VAL_INT4), (1, 16))

    gbps = nbytes / t_dev / 1e9
    result = {
        "metric": "SparseGemv achieved HBM GB/s, INT4 2:4 11008x4096, M=1",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "us_per_call": round(t_dev * 1e6, 3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_dev * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights x fp16 activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "headline: W 11008x4096 2:4 sparse INT4 g128 in 2bit-CSR, x FP16, M=1",
                   "rotating_copies": copies, "bytes_per_call": nbytes},
        "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": MEASURED_TRAFFIC_BYTES,
                     "kernel": "egt_sparse_gemv (headline shape)",
                     "frac_of_read_ceiling": round(t_read / t_dev * nbytes / nb16, 4)},
        "host_wall_us_per_call": round(t_wall * 1e6, 3),
        "read_ceiling": {"same_size_us": round(t_read * 1e6, 3), "same_size_gbps": round(nb16 / t_read / 1e9, 1),
                         "one_gib_gbps": round((1 << 30) / t_big / 1e9, 1),
                         "empty_kernel_us": round(t_tiny * 1e6, 3)},
    }

    if args.extra:
        extra = {}
        # the same launch on one copy only (weights stay in the last-level cache)
        t_hot, _ = time_loop(torch, lambda i: calls[0](), args.steps, args.warmup)
        extra["headline_hot_cache_us"] = round(t_hot * 1e6, 3)
        # config 3: sparse FP16 values
        p3 = B.pack_2bitcsr(w, mask, N, 0, B.VAL_FP16)
        c3 = max(2, -(-2 * LLC_BYTES // p3.nbytes()))
        pk3 = [p3.to(dev) for _ in range(c3)]
        f3 = [B.prepared_sparse_gemv(pk3[i], xd, ys[0]) for i in range(c3)]
        t3, _ = time_loop(torch, lambda i: f3[i % c3](), 1000, 100)
        b3 = algorithmic_bytes(R, K, N, 0, 1)
        extra["config3_sparse_fp16_11008x4096"] = {"us": round(t3 * 1e6, 3), "gbps": round(b3 / t3 / 1e9, 1), "bytes": b3}
        for M in (2, 4, 16):                          # the same matrix under parallel verification
            Xm = torch.from_numpy(synth.activation_rows(M, K, synth.seed_for(3) + M).view(np.int16)).to(dev).view(torch.float16)
            Ym = torch.empty((M, R), dtype=torch.float16, device=dev)
            fm = [B.prepared_sparse_gemm_smallm(pk3[i], Xm, Ym) for i in range(c3)]
            tm, _ = time_loop(torch, lambda i: fm[i % c3](), 600, 60)
            bm = algorithmic_bytes(R, K, N, 0, 1, m=M)
            extra[f"sparse_fp16_11008x4096_M{M}"] = {"us": round(tm * 1e6, 3), "gbps": round(bm / tm / 1e9, 1), "bytes": bm}
            del fm
        del pk3
        p3n = B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, 0, B.VAL_FP16)     # 1:4 with FP16 values
        c3n = max(2, -(-2 * LLC_BYTES // p3n.nbytes()))
        pk3n = [p3n.to(dev) for _ in range(c3n)]
        f3n = [B.prepared_sparse_gemv(pk3n[i], xd, ys[0]) for i in range(c3n)]
        t3n, _ = time_loop(torch, lambda i: f3n[i % c3n](), 1000, 100)
        b3n = algorithmic_bytes(R, K, 1, 0, 1)
        extra["sparse_fp16_1to4_11008x4096"] = {"us": round(t3n * 1e6, 3), "gbps": round(b3n / t3n / 1e9, 1), "bytes": b3n}
        del pk3n, f3n
        # config 2: dense INT4 4096x4096
        w2 = synth.weights(4096, 4096, synth.seed_for(2))
        q2, qp2 = B.quant_int4(w2, 128)
        c2 = max(2, -(-2 * LLC_BYTES // (q2.nbytes + qp2.nbytes)))
        q2d = [torch.from_numpy(q2).to(dev) for _ in range(c2)]
        qp2d = [torch.from_numpy(qp2.view(np.int16)).to(dev) for _ in range(c2)]
        x2 = torch.from_numpy(synth.activations(4096, synth.seed_for(2)).view(np.int16)).to(dev).view(torch.float16)
        y2 = torch.empty(4096, dtype=torch.float16, device=dev)
        f2 = [B.prepared_int4_gemv(q2d[i], qp2d[i], 4096, 4096, 128, x2, y2) for i in range(c2)]
        t2, _ = time_loop(torch, lambda i: f2[i % c2](), 2000, 200)
        b2 = dense_int4_bytes(4096, 4096, 128)
        extra["config2_dense_int4_4096x4096"] = {"us": round(t2 * 1e6, 3), "gbps": round(b2 / t2 / 1e9, 1), "bytes": b2}
        del q2d, qp2d
        # config 5: small M on both shapes
        for (r5, k5, mi) in ((11008, 4096, 0), (4096, 11008, 1)):
            w5 = synth.weights(r5, k5, synth.seed_for(5, mi))
            p5 = B.pack_2bitcsr(w5, B.prune_n4(w5, 2), 2, 128, B.VAL_INT4)
            c5 = max(2, -(-2 * LLC_BYTES // p5.nbytes()))
            pk5 = [p5.to(dev) for _ in range(c5)]
            for M in (1, 4, 16, 64):
                X = torch.from_numpy(synth.activation_rows(M, k5, 5).view(np.int16)).to(dev).view(torch.float16)
                Y = torch.empty((M, r5), dtype=torch.float16, device=dev)
                f5 = [B.prepared_sparse_gemm_smallm(pk5[i], X, Y) for i in range(c5)]
                t5, _ = time_loop(torch, lambda i: f5[i % c5](), 500, 50)
                b5 = algorithmic_bytes(r5, k5, 2, 128, 0, M)
                extra[f"config5_{r5}x{k5}_M{M}"] = {"us": round(t5 * 1e6, 3), "gbps": round(b5 / t5 / 1e9, 1),
                                                   "bytes": b5, "tflops": round(2 * M * r5 * k5 / 2 / t5 / 1e12, 2)}
            del pk5
        # M-sweep through an all-2:4 layer (q/k/v/o, gate/up, down) and the trigger cost model of
        # Sec. 3.4: verification cost ~ a + b*M, autoregressive step = t(1)
        sweep_m = (1, 2, 4, 8, 16, 32, 64)
        layer_us = {m: 0.0 for m in sweep_m}
        for (r5, k5, reps) in ((4096, 4096, 4), (11008, 4096, 2), (4096, 11008, 1)):
            w5 = synth.weights(r5, k5, synth.seed_for(5, 7))
            p5 = B.pack_2bitcsr(w5, B.prune_n4(w5, 2), 2, 128, B.VAL_INT4)
            c5 = max(2, -(-2 * LLC_BYTES // p5.nbytes()))
            pk5 = [p5.to(dev) for _ in range(c5)]
            for pass_no, M in enumerate((sweep_m[0],) + sweep_m):   # the first pass only settles clocks and caches
                X = torch.from_numpy(synth.activation_rows(M, k5, 5).view(np.int16)).to(dev).view(torch.float16)
                Y = torch.empty((M, r5), dtype=torch.float16, device=dev)
                f5 = [B.prepared_sparse_gemm_smallm(pk5[i], X, Y) for i in range(c5)]
                t5, _ = time_loop(torch, lambda i: f5[i % c5](), 600, 60)
                if pass_no > 0:
                    layer_us[M] += reps * t5 * 1e6
            del pk5
        fit_a, fit_b = B.fit_verify_cost(list(sweep_m[1:]), [layer_us[m] for m in sweep_m[1:]])
        cand = [64, 24, 9, 4, 2, 1]                      # candidates left per trie depth (wide top, narrow bottom)
        rem = [6, 5, 4, 3, 2, 1]                         # tokens still to generate (average ID length 6)
        depth, gain = B.trigger_depth(layer_us[1], fit_a, fit_b, cand, rem)
        extra["trigger_model"] = {"layer_us_by_M": {str(m): round(v, 2) for m, v in layer_us.items()},
                                  "fit_a_us": round(fit_a, 3), "fit_b_us_per_token": round(fit_b, 4),
                                  "t_ar_us": round(layer_us[1], 2), "candidates": cand, "remaining": rem,
                                  "trigger_depth": depth, "benefit_us_per_layer": round(gain, 2)}
        # 1:4 sparsity (the sparser layer-adaptive setting), same shape as the headline
        p14 = B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, GRP, B.VAL_INT4)
        c14 = max(2, -(-2 * LLC_BYTES // p14.nbytes()))
        pk14 = [p14.to(dev) for _ in range(c14)]
        f14 = [B.prepared_sparse_gemv(pk14[i], xd, ys[0]) for i in range(c14)]
        t14, _ = time_loop(torch, lambda i: f14[i % c14](), 2000, 200)
        b14 = algorithmic_bytes(R, K, 1, GRP, 0)
        extra["sparse_int4_1to4_11008x4096"] = {"us": round(t14 * 1e6, 3), "gbps": round(b14 / t14 / 1e9, 1), "bytes": b14}
        del pk14, f14
        # config 4: the 32-layer stack, 224 launches, plain and as a HIP graph
        from paper_2605_11582_amd import stack as S
        del packed, calls
        torch.cuda.empty_cache()
        stk = S.LayerStack.build(dev, distinct_layers=1)
        t4, _ = time_loop(torch, lambda i: stk.run(), 20, 3)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            stk.run(side.cuda_stream)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                stk.run(torch.cuda.current_stream().cuda_stream)
            t4g, _ = time_loop(torch, lambda i: graph.replay(), 20, 3)
        fused = stk.fuse()

        def run_fused(i):
            for c in fused:
                c()
        t4f, _ = time_loop(torch, run_fused, 20, 3)
        with torch.cuda.stream(side):
            sp = side.cuda_stream
            for c in fused:
                c(sp)
            torch.cuda.synchronize()
            graph_f = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph_f, stream=side):
                sp = torch.cuda.current_stream().cuda_stream
                for c in fused:
                    c(sp)
            t4fg, _ = time_loop(torch, lambda i: graph_f.replay(), 20, 3)
        extra["config4_stack_fused_128_launches"] = {"us_plain": round(t4f * 1e6, 1), "us_graph": round(t4fg * 1e6, 1),
                                                     "gbps_plain": round(stk.nbytes / t4f / 1e9, 1),
                                                     "gbps_graph": round(stk.nbytes / t4fg / 1e9, 1)}
        del graph_f
        extra["config4_stack_224_launches"] = {"us_plain": round(t4 * 1e6, 1), "us_graph": round(t4g * 1e6, 1),
                                               "bytes": stk.nbytes, "gbps_plain": round(stk.nbytes / t4 / 1e9, 1),
                                               "gbps_graph": round(stk.nbytes / t4g / 1e9, 1)}
        del stk, graph
        torch.cuda.empty_cache()
        # the three-way layer-adaptive mix (2:4, 1:4 and dense layers)
        stk3 = S.LayerStack.build(dev, distinct_layers=1, plan="mix3")
        t43, _ = time_loop(torch, lambda i: stk3.run(), 20, 3)
        extra["stack_mix3_224_launches"] = {"us_plain": round(t43 * 1e6, 1), "bytes": stk3.nbytes,
                                            "gbps_plain": round(stk3.nbytes / t43 / 1e9, 1)}
        result["extra"] = extra

    if not args.no_cpu_baseline:
        from oracle import egt_oracle as O
        sample = 1024
        sub_w = w[:sample]
        o = O.pack_2bitcsr(sub_w, O.prune_n4_magnitude(sub_w, N), N, GRP, O.VAL_INT4)
        reps, t0 = 0, time.perf_counter()
        while True:
            O.gemv(o, x)
            reps += 1
            if time.perf_counter() - t0 > 10.0:
                break
        t_cpu = (time.perf_counter() - t0) / reps
        sample_bytes = algorithmic_bytes(sample, K, N, GRP, 0)
        result["cpu_baseline"] = {"value": round(sample_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1,
                                  "kind": "oracle",
                                  "sample": f"oracle gemv (decode + multiply, float64 numpy) on the first {sample} "
                                            f"rows of the headline matrix, {reps} repetitions, "
                                            f"{t_cpu * 1e3:.1f} ms each; host has {os.cpu_count()} logical CPUs"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
