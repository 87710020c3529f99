#!/usr/bin/env python3
"""Benchmark of the SparseGemv hot path on one MI355X.

A step is one `egt_sparse_gemv` call (stage x, stream the 2bit-CSR row data,
dequantise, gather, multiply-accumulate, reduce, store) on the headline workload:
W 11008 x 4096, 2:4 sparse, INT4 group 128, 2bit-CSR; x FP16; M = 1.  Inputs are
resident in HBM before the timed region.  Consecutive steps cycle over enough
distinct device copies of the packed matrix to exceed twice the 256 MB last-level
cache, so every launch streams its weights from HBM.

Timing protocol: the clocks are warmed with at least 0.3 s of launches whatever
--warmup says; then `--steps` launches are enqueued back to back on one stream
behind a long filler kernel (so the queue is full when the first one starts and the
host's enqueue rate is not what is measured), bracketed by one HIP event pair; this is
repeated 5 times and the median is reported (`ms_per_step`), with the minimum beside
it.  The other configurations are timed the same way with their own launch counts and
reported under "table".

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import subprocess
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
LLC_BYTES = 256 << 20
REPEATS = 5
R, K, N, GRP = 11008, 4096, 2, 128
TRAFFIC_PROFILE = os.path.join("profiles", "sparse_m1_headline_hbm_traffic.txt")
# vector-ALU instructions and matrix-core busy cycles of one headline launch, counted by
# rocprofv3 (profiles/sparse_m1_headline_counters.txt); one wave64 vector instruction
# occupies its 16-lane SIMD for 4 cycles, the device has 1024 SIMDs at 2.4 GHz
COUNTERS_PROFILE = os.path.join("profiles", "sparse_m1_headline_counters.txt")
SIMDS, CLOCK_HZ, CYCLES_PER_VALU = 1024, 2.4e9, 4


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


def profile_number(path, key):
    """`key: <number>` from a committed profile summary, or None."""
    try:
        with open(os.path.join(ROOT, path)) as f:
            m = re.search(r"^" + re.escape(key) + r"\s*[:=]\s*([0-9.eE+]+)", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


class Timer:
    """Back-to-back launches on the current stream, one event pair, 5 repeats."""

    def __init__(self, torch, filler):
        self.torch, self.filler = torch, filler

    def __call__(self, fn, steps, warmup=None):
        torch = self.torch
        for i in range(steps if warmup is None else warmup):
            fn(i)
        per_step, wall = [], []
        for _ in range(REPEATS):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            self.filler(torch.cuda.current_stream().cuda_stream)   # keeps the GPU busy while the queue fills
            t0 = time.perf_counter()
            e0.record()
            for i in range(steps):
                fn(i)
            e1.record()
            wall.append((time.perf_counter() - t0) / steps)
            torch.cuda.synchronize()
            per_step.append(e0.elapsed_time(e1) * 1e-3 / steps)
        return {"median": statistics.median(per_step), "min": min(per_step), "all": per_step,
                "host_enqueue": statistics.median(wall)}


def entry(t, nbytes, flops=None):
    out = {"us": round(t["median"] * 1e6, 3), "us_min": round(t["min"] * 1e6, 3),
           "gbps": round(nbytes / t["median"] / 1e9, 1), "frac": round(nbytes / t["median"] / 1e9 / HBM_PEAK_GBPS, 4),
           "bytes": nbytes}
    if flops:
        out["tflops"] = round(flops / t["median"] / 1e12, 2)
    return out


# ------------------------------------------------------------------ the oracle, timed on the host
def cpu_worker(shard, nshards, reps):
    """One process of the row-sharded oracle leg: packs its rows with the oracle (untimed),
    then multiplies when told to.  Talks to the parent over stdin/stdout."""
    from oracle import egt_oracle as O
    from paper_2605_11582_amd import synth
    seed = synth.seed_for(synth.HEADLINE)
    w = synth.weights(R, K, seed)
    x = synth.activations(K, seed)
    r0, r1 = shard * R // nshards, (shard + 1) * R // nshards
    sub = np.ascontiguousarray(w[r0:r1])
    del w
    o = O.pack_2bitcsr(sub, O.prune_n4_magnitude(sub, N), N, GRP, O.VAL_INT4)
    O.gemv(o, x)
    print("ready", flush=True)
    sys.stdin.readline()
    times = []
    for _ in range(reps):
        t0 = time.perf_counter()
        O.gemv(o, x)
        times.append(time.perf_counter() - t0)
    print(json.dumps({"rows": r1 - r0, "times": times}), flush=True)


def cpu_baseline(w, x):
    from oracle import egt_oracle as O
    sample = 1024
    sub = w[:sample]
    o = O.pack_2bitcsr(sub, O.prune_n4_magnitude(sub, N), N, GRP, O.VAL_INT4)
    sample_bytes = algorithmic_bytes(sample, K, N, GRP, 0)

    def median_of(fn, budget_s=4.0):
        times, t_end = [], time.perf_counter() + budget_s
        while len(times) < 3 or time.perf_counter() < t_end:
            t0 = time.perf_counter()
            fn()
            times.append(time.perf_counter() - t0)
        return statistics.median(times), len(times)

    t_one, n_one = median_of(lambda: O.gemv(o, x))
    col, w_hat, _ = O.decode_2bitcsr(o)
    x64 = x.astype(np.float64)
    t_hoist, n_hoist = median_of(lambda: O.gemv_decoded(col, w_hat, x64))
    del col, w_hat
    # all host cores: the rows of the whole matrix sharded over one process per core
    avail = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = max(1, min(avail, 16))
    env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    reps = 3
    procs = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--cpu-worker", f"{s},{cores},{reps}"],
                              stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True, env=env, cwd=ROOT)
             for s in range(cores)]
    try:
        for p in procs:
            assert p.stdout.readline().strip() == "ready"
        for p in procs:
            p.stdin.write("go\n")
            p.stdin.flush()
        results = [json.loads(p.stdout.readline()) for p in procs]
    finally:
        for p in procs:
            p.stdin.close()
            p.wait(timeout=60)
    assert sum(r["rows"] for r in results) == R
    t_all = statistics.median([max(r["times"][k] for r in results) for k in range(reps)])
    full_bytes = algorithmic_bytes(R, K, N, GRP, 0)
    return {"value": round(full_bytes / t_all / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"oracle gemv (decode + multiply, float64 numpy) on all {R} rows of the headline matrix, "
                      f"row-sharded over {cores} processes (one thread each), median of {reps}: {t_all * 1e3:.1f} ms "
                      f"per product; host shows {os.cpu_count()} logical CPUs, {avail} usable",
            "one_core": {"value": round(sample_bytes / t_one / 1e9, 4), "unit": "GB/s", "cores": 1,
                         "sample": f"first {sample} rows, decode included, median of {n_one}: {t_one * 1e3:.1f} ms"},
            "one_core_decode_hoisted": {"value": round(sample_bytes / t_hoist / 1e9, 4), "unit": "GB/s", "cores": 1,
                                        "sample": f"first {sample} rows, decoded once outside the timed region, "
                                                  f"median of {n_hoist}: {t_hoist * 1e3:.1f} ms"}}


# ------------------------------------------------------------------ main
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-table", action="store_true", help="time the headline workload only")
    ap.add_argument("--extra", action="store_true", help="kept for compatibility: the table is on by default")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a 64 MiB device copy ten times (known traffic, for scaling rocprofv3 counters)")
    ap.add_argument("--counter-workloads", action="store_true",
                    help="also launch the other kernels 40 times each, untimed (dense INT4, FP16 values, 1:4, "
                         "M = 16 / 64), for rocprofv3 counter runs")
    ap.add_argument("--counter-run", action="store_true",
                    help="a short run for rocprofv3 --pmc: --steps headline launches without clock warm-up, read "
                         "ceilings, table or oracle, then the --counter-workloads launches, five whole-stack launches and five "
                         "verification-step launches at 16 and at 64 tokens")
    ap.add_argument("--only-stack", action="store_true",
                    help="time the whole-stack launch of configuration 4 only (for sweeps of a tuning build)")
    ap.add_argument("--only-verify-stack", type=int, default=0, metavar="M",
                    help="time the one-launch verification step of M tokens through the 2:4 layers of configuration 4 only")
    ap.add_argument("--cpu-worker", default=None, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.cpu_worker:
        cpu_worker(*[int(v) for v in args.cpu_worker.split(",")])
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    from paper_2605_11582_amd import synth
    seed = synth.seed_for(synth.HEADLINE)
    w = synth.weights(R, K, seed)
    x = synth.activations(K, seed)

    if args.counter_run:
        args.no_cpu_baseline = args.no_table = args.counter_workloads = True
    # the oracle on the host cores first: its worker processes start before this process
    # touches the GPU
    cpu = None if args.no_cpu_baseline else cpu_baseline(w, x)

    import torch
    from paper_2605_11582_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    mask = B.prune_n4(w, N)
    p = B.pack_2bitcsr(w, mask, N, GRP, B.VAL_INT4)
    nbytes = algorithmic_bytes(R, K, N, GRP, 0)
    copies = max(2, -(-2 * LLC_BYTES // p.nbytes()))
    packed = [p.to(dev) for _ in range(copies)]
    xd = torch.from_numpy(x.view(np.int16)).to(dev).view(torch.float16)
    ys = [torch.empty(R, dtype=torch.float16, device=dev) for _ in range(copies)]
    calls = [B.prepared_sparse_gemv(packed[i], xd, ys[i]) for i in range(copies)]

    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    filler = B.prepared_stream_read(big, 1 << 30, sink)
    timer = Timer(torch, filler)

    if args.only_stack:
        from paper_2605_11582_amd import stack as S
        del packed[:], calls[:]
        stk = S.LayerStack.build(dev, distinct_layers=1)     # the traffic of all 224 matrices; the numbers repeat
        whole = stk.one_launch()
        plan = whole.plan
        row = entry(timer(lambda i: whole(), 30, 5), stk.nbytes)
        row.update(mode=plan.mode, grid=plan.grid_x, block_threads=plan.block_threads, lds_bytes=plan.lds_bytes, items=plan.nitems)
        print(json.dumps({"only_stack": True, "config4_whole_stack": row}))
        return

    if args.only_verify_stack:
        from paper_2605_11582_amd import stack as S
        del packed[:], calls[:]
        stk = S.LayerStack.build(dev, distinct_layers=1)     # the traffic of all matrices; the numbers repeat
        step, step_bytes = stk.verify_step(args.only_verify_stack)
        plan = step.plan
        row = entry(timer(lambda i: step(), 30, 5), step_bytes)
        row.update(M=plan.M, matrices=plan.count, grid=plan.grid_x, block_threads=plan.block_threads, lds_bytes=plan.lds_bytes)
        out = {"only_verify_stack": True, "config4_sparse_layers_one_launch": row}
        if args.only_verify_stack <= 32:              # the 1:4 layers of the three-way mix (11 layers, 77 products)
            del stk, step
            torch.cuda.empty_cache()
            stk = S.LayerStack.build(dev, distinct_layers=1, plan="mix3")
            step, step_bytes = stk.verify_step(args.only_verify_stack, "s14")
            plan = step.plan
            row = entry(timer(lambda i: step(), 30, 5), step_bytes)
            row.update(M=plan.M, matrices=plan.count, grid=plan.grid_x, block_threads=plan.block_threads, lds_bytes=plan.lds_bytes)
            out["mix3_1to4_layers_one_launch"] = row
            both, both_bytes = stk.verify_step(args.only_verify_stack, ("s24", "s14"))
            row = entry(timer(lambda i: both(), 30, 5), both_bytes)
            row.update(M=plan.M, matrices=sum(p.count for p in both.plans), launches=len(both.plans))
            out["mix3_sparse_layers_one_call"] = row
        print(json.dumps(out))
        return

    if args.counter_run:
        for i in range(args.steps):
            calls[i % copies]()
        torch.cuda.synchronize()
        reads = [B.prepared_stream_read(packed[i].values, packed[i].values.numel() // 16 * 16, sink) for i in range(copies)]
        for i in range(40):
            reads[i % copies]()
        filler()
        torch.cuda.synchronize()
        if args.calibrate:
            src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
            dst = torch.empty_like(src)
            for _ in range(10):
                dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        counter_workloads(torch, B, synth, w, mask, p, dev)
        from paper_2605_11582_amd import stack as S
        del packed[:], calls[:]
        stk = S.LayerStack.build(dev, distinct_layers=1)
        whole = stk.one_launch()
        for _ in range(5):
            whole()
        torch.cuda.synchronize()
        for m_tokens in (16, 64):                     # a verification step through the 2:4 layers in one launch
            step, _ = stk.verify_step(m_tokens)
            for _ in range(5):
                step()
            torch.cuda.synchronize()
            del step
        print(json.dumps({"counter_run": True, "headline_launches": args.steps}))
        return

    # clock warm-up: at least 0.3 s of back-to-back launches
    t_end = time.perf_counter() + 0.3
    i = 0
    while time.perf_counter() < t_end:
        for _ in range(200):
            calls[i % copies]()
            i += 1
        torch.cuda.synchronize()

    head = timer(lambda i: calls[i % copies](), args.steps, args.warmup)
    t_dev = head["median"]

    # read ceiling: a plain 128-bit streaming read of the same number of bytes, same rotation
    steps_aux = max(args.steps, 400)
    pool = [torch.empty(p.nbytes(), dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(copies)]
    nb16 = p.nbytes() // 16 * 16
    reads = [B.prepared_stream_read(pool[i], nb16, sink) for i in range(copies)]
    t_read = timer(lambda i: reads[i % copies](), steps_aux)
    tiny = B.prepared_stream_read(pool[0], 16, sink)
    t_tiny = timer(lambda i: tiny(), steps_aux)
    t_big = timer(lambda i: filler(), 10, 2)
    del pool, reads

    if args.calibrate:
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.counter_workloads:
        counter_workloads(torch, B, synth, w, mask, p, dev)

    gbps = nbytes / t_dev / 1e9
    traffic = profile_number(TRAFFIC_PROFILE, "traffic_bytes_per_launch")
    valu_insts = profile_number(COUNTERS_PROFILE, "valu_insts_per_launch")
    mfma_cycles = profile_number(COUNTERS_PROFILE, "mfma_busy_cycles_per_launch")
    result = {
        "metric": "SparseGemv achieved HBM GB/s, INT4 2:4 11008x4096, M=1",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "us_per_call": round(t_dev * 1e6, 3),
        "us_per_call_min": round(head["min"] * 1e6, 3),
        "us_per_call_repeats": [round(v * 1e6, 3) for v in head["all"]],
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_dev * 1e3,
        "ms_per_step_min": head["min"] * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights x fp16 activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "headline: W 11008x4096 2:4 sparse INT4 g128 in 2bit-CSR, x FP16, M=1",
                   "rotating_copies": copies, "bytes_per_call": nbytes, "repeats": REPEATS,
                   "protocol": "median of 5 x --steps back-to-back launches behind a filler kernel, one event pair each"},
        "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4),
                     "traffic": None if traffic is None else int(traffic),
                     "traffic_source": TRAFFIC_PROFILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the same kernel; "
                                                        "not re-measured by this run)",
                     "kernel": "egt_sparse_gemv (headline shape)",
                     "frac_of_read_ceiling": round(t_read["median"] / t_dev * nbytes / nb16, 4)},
        "host_enqueue_us_per_call": round(head["host_enqueue"] * 1e6, 3),
        "read_ceiling": {"same_size_us": round(t_read["median"] * 1e6, 3), "same_size_us_min": round(t_read["min"] * 1e6, 3),
                         "same_size_gbps": round(nb16 / t_read["median"] / 1e9, 1),
                         "one_gib_gbps": round((1 << 30) / t_big["median"] / 1e9, 1),
                         "empty_kernel_us": round(t_tiny["median"] * 1e6, 3)},
    }
    if valu_insts is not None and mfma_cycles is not None:
        issue_s = (valu_insts * CYCLES_PER_VALU + mfma_cycles) / (SIMDS * CLOCK_HZ)
        result["valu_issue_bound"] = {"us": round(issue_s * 1e6, 3), "valu_insts_per_launch": int(valu_insts),
                                      "valu_insts_per_nnz": round(valu_insts / (R * N * K // 4), 4),
                                      "mfma_busy_cycles_per_launch": int(mfma_cycles),
                                      "model": "(vector instructions x 4 cycles + matrix busy cycles) / (1024 SIMDs x 2.4 GHz), "
                                               "perfectly spread",
                                      "source": COUNTERS_PROFILE + " (not re-measured by this run)"}

    if not args.no_table:
        result["table"] = table(torch, B, synth, timer, dev, w, mask, xd, ys, calls, packed)
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


def counter_workloads(torch, B, synth, w, mask, p, dev):
    seed = synth.seed_for(synth.HEADLINE)

    def launches(pk_host, Ms, cols=K, rows=R):
        n = max(2, -(-2 * LLC_BYTES // pk_host.nbytes()))
        pks = [pk_host.to(dev) for _ in range(n)]
        for M in Ms:
            Xm = torch.from_numpy(synth.activation_rows(M, cols, seed + M).view(np.int16)).to(dev).view(torch.float16)
            Ym = torch.empty((M, rows), dtype=torch.float16, device=dev)
            fs = [B.prepared_sparse_gemv(pks[i], Xm[0], Ym[0]) if M == 1 else
                  B.prepared_sparse_gemm_smallm(pks[i], Xm, Ym) for i in range(n)]
            for i in range(40):
                fs[i % n]()
            torch.cuda.synchronize()
    launches(B.pack_2bitcsr(w, mask, N, 0, B.VAL_FP16), (1, 2, 4, 16))
    launches(B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, 0, B.VAL_FP16), (1,))
    launches(p, (2, 16, 64))
    launches(B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, GRP, B.VAL_INT4), (1, 16))
    w5 = synth.weights(4096, 11008, synth.seed_for(5, 1))
    launches(B.pack_2bitcsr(w5, B.prune_n4(w5, 2), 2, GRP, B.VAL_INT4), (1, 16, 64), cols=11008, rows=4096)
    w2 = synth.weights(4096, 4096, synth.seed_for(2))
    q2, qp2 = B.quant_int4(w2, 128)
    c2 = max(2, -(-2 * LLC_BYTES // (q2.nbytes + qp2.nbytes)))
    x2 = torch.from_numpy(synth.activations(4096, synth.seed_for(2)).view(np.int16)).to(dev).view(torch.float16)
    y2 = torch.empty(4096, dtype=torch.float16, device=dev)
    q2d = [torch.from_numpy(q2).to(dev) for _ in range(c2)]
    qp2d = [torch.from_numpy(qp2.view(np.int16)).to(dev) for _ in range(c2)]
    for i in range(40):
        B.int4_gemv(q2d[i % c2], qp2d[i % c2], 4096, 4096, 128, x2, y2)
    torch.cuda.synchronize()


def table(torch, B, synth, timer, dev, w, mask, xd, ys, calls, packed):
    """Every configuration of the benchmark spec, timed like the headline."""
    from paper_2605_11582_amd import stack as S
    t = {}
    packed_bytes_24 = packed[0].nbytes()
    up16 = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.float16)
    # the headline launch on one copy only (weights stay in the last-level cache)
    t["headline_hot_cache"] = entry(timer(lambda i: calls[0](), 1000), algorithmic_bytes(R, K, N, GRP, 0))
    # the headline matrix with its codes in the paired nibble order (one shift and four and-ors
    # per eight codes instead of four byte permutes and four and-ors)
    pp = B.pack_2bitcsr(w, mask, N, GRP, B.VAL_INT4_PAIRED)
    cpp = len(packed)
    pkp = [pp.to(dev) for _ in range(cpp)]
    fp = [B.prepared_sparse_gemv(pkp[i], xd, ys[i]) for i in range(cpp)]
    t["headline_paired_nibble_order"] = entry(timer(lambda i: fp[i % cpp](), 1000), algorithmic_bytes(R, K, N, GRP, 0))
    del pkp, fp
    # config 1: 1024 x 1024, launch-bound
    w1 = synth.weights(1024, 1024, synth.seed_for(1))
    p1 = B.pack_2bitcsr(w1, B.prune_n4(w1, 2), 2, 128, B.VAL_INT4)
    c1 = 64
    pk1 = [p1.to(dev) for _ in range(c1)]
    x1 = up16(synth.activations(1024, synth.seed_for(1)))
    y1 = torch.empty(1024, dtype=torch.float16, device=dev)
    f1 = [B.prepared_sparse_gemv(pk1[i], x1, y1) for i in range(c1)]
    t["config1_sparse_int4_1024x1024"] = entry(timer(lambda i: f1[i % c1](), 1000), algorithmic_bytes(1024, 1024, 2, 128, 0))
    # config 2: dense INT4 4096 x 4096
    w2 = synth.weights(4096, 4096, synth.seed_for(2))
    q2, qp2 = B.quant_int4(w2, 128)
    c2 = max(2, -(-2 * LLC_BYTES // (q2.nbytes + qp2.nbytes)))
    q2d = [torch.from_numpy(q2).to(dev) for _ in range(c2)]
    qp2d = [torch.from_numpy(qp2.view(np.int16)).to(dev) for _ in range(c2)]
    x2 = up16(synth.activations(4096, synth.seed_for(2)))
    y2 = torch.empty(4096, dtype=torch.float16, device=dev)
    f2 = [B.prepared_int4_gemv(q2d[i], qp2d[i], 4096, 4096, 128, x2, y2) for i in range(c2)]
    t["config2_dense_int4_4096x4096"] = entry(timer(lambda i: f2[i % c2](), 1000), dense_int4_bytes(4096, 4096, 128))
    del q2d, qp2d, f2
    # config 3: sparse FP16 values
    p3 = B.pack_2bitcsr(w, mask, N, 0, B.VAL_FP16)
    c3 = max(2, -(-2 * LLC_BYTES // p3.nbytes()))
    pk3 = [p3.to(dev) for _ in range(c3)]
    f3 = [B.prepared_sparse_gemv(pk3[i], xd, ys[0]) for i in range(c3)]
    t["config3_sparse_fp16_11008x4096"] = entry(timer(lambda i: f3[i % c3](), 600), algorithmic_bytes(R, K, N, 0, 1))
    del pk3, f3
    # 1:4 sparsity (the sparser layer-adaptive setting), same shape as the headline
    p14 = B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, GRP, B.VAL_INT4)
    c14 = max(2, -(-2 * LLC_BYTES // p14.nbytes()))
    pk14 = [p14.to(dev) for _ in range(c14)]
    f14 = [B.prepared_sparse_gemv(pk14[i], xd, ys[0]) for i in range(c14)]
    t["sparse_int4_1to4_11008x4096"] = entry(timer(lambda i: f14[i % c14](), 1000), algorithmic_bytes(R, K, 1, GRP, 0))
    del pk14, f14
    # the same kernels on a matrix six times as tall (a 65536-word output projection): one launch
    # moves 109 MB, so the launch gap that dominates the 18 MB headline weighs a sixth as much
    Rt = 65536
    wt = synth.weights(Rt, K, synth.seed_for(synth.HEADLINE, 7))
    mask_t = B.prune_n4(wt, N)
    yt = torch.empty(Rt, dtype=torch.float16, device=dev)
    for tag, kind in (("sparse_int4_65536x4096", B.VAL_INT4), ("sparse_int4_65536x4096_paired_nibble_order", B.VAL_INT4_PAIRED)):
        pt = B.pack_2bitcsr(wt, mask_t, N, GRP, kind)
        ct = max(2, -(-2 * LLC_BYTES // pt.nbytes()))
        pkt = [pt.to(dev) for _ in range(ct)]
        ft = [B.prepared_sparse_gemv(pkt[i], xd, yt) for i in range(ct)]
        t[tag] = entry(timer(lambda i: ft[i % ct](), 300), algorithmic_bytes(Rt, K, N, GRP, 0))
        del pkt, ft, pt
    del wt, mask_t
    # rows of different lengths: half of the rows keep 1 of 4 (Sec. 3.2's adaptive N inside one
    # matrix); the slot-by-slot kernel that follows row_ptr, not a matrix-core path
    rng = np.random.default_rng(synth.seed_for(synth.HEADLINE))
    nk = rng.permutation(np.repeat([1, 2], R // 2)).astype(np.int32)
    mask_r = np.where((nk == 1)[:, None], B.prune_n4(w, 1), mask).astype(np.uint8)
    pr = B.pack_2bitcsr_rows(w, mask_r, nk, GRP, B.VAL_INT4)
    cr = max(2, -(-2 * LLC_BYTES // pr.nbytes()))
    pkr = [pr.to(dev) for _ in range(cr)]
    fr = [B.prepared_sparse_gemv(pkr[i], xd, ys[0]) for i in range(cr)]
    rag_bytes = pr.nbytes() - 4 + 2 * K + 2 * R
    t["sparse_int4_rows_half_1to4_11008x4096"] = entry(timer(lambda i: fr[i % cr](), 200), rag_bytes)
    t["sparse_int4_rows_half_1to4_11008x4096"]["bytes_saved_vs_2to4"] = packed_bytes_24 - pr.nbytes()
    del pkr, fr
    # config 5: small M on both shapes; the M-sweep (every M from 1 to 64) of an all-2:4 layer
    # (q/k/v/o, gate/up, down) feeds the trigger cost model of Sec. 3.4: verification ~ a + b*M,
    # AR step = t(1).  The workspace form is used wherever the library says it is the faster one.
    sweep_m = tuple(range(1, 65))
    layer_us = {m: 0.0 for m in sweep_m}
    pools, split_wins, best_us = {}, set(), {}
    for (r5, k5, mi, reps) in ((11008, 4096, 0, 2), (4096, 11008, 1, 1), (4096, 4096, 2, 4)):
        w5 = synth.weights(r5, k5, synth.seed_for(5, mi))
        p5 = B.pack_2bitcsr(w5, B.prune_n4(w5, 2), 2, 128, B.VAL_INT4)
        c5 = max(2, -(-2 * LLC_BYTES // p5.nbytes()))
        pk5 = [p5.to(dev) for _ in range(c5)]
        pools[mi] = (r5, k5, reps, pk5)
        for M in sweep_m:
            X = up16(synth.activation_rows(M, k5, 5))
            Y = torch.empty((M, r5), dtype=torch.float16, device=dev)
            listed = mi < 2 and M in (1, 4, 16, 64)
            steps5 = 300 if listed or M in (2, 8, 32) else 60
            f5 = [B.prepared_sparse_gemm_smallm(pk5[i], X, Y) for i in range(c5)]
            t5 = timer(lambda i: f5[i % c5](), steps5)
            best = t5["median"]
            if listed:
                t[f"config5_{r5}x{k5}_M{M}"] = entry(t5, algorithmic_bytes(r5, k5, 2, 128, 0, M), flops=2 * M * r5 * k5 / 2)
            need = B.smallm_ws_bytes(pk5[0], M)
            if need:                                  # K split over workgroups, partial sums in a caller's workspace
                ws = torch.empty(need, dtype=torch.uint8, device=dev)
                f5w = [B.prepared_sparse_gemm_smallm_ws(pk5[i], X, Y, ws) for i in range(c5)]
                t5w = timer(lambda i: f5w[i % c5](), steps5)
                if t5w["median"] < best:
                    best = t5w["median"]
                    split_wins.add((mi, M))
                if mi < 2 and M in (32, 48, 64):
                    t[f"config5_{r5}x{k5}_M{M}_k_split_workspace"] = entry(
                        t5w, algorithmic_bytes(r5, k5, 2, 128, 0, M), flops=2 * M * r5 * k5 / 2)
                del f5w, ws
            layer_us[M] += reps * best * 1e6
            best_us[(mi, M)] = best * 1e6
    # the same layer with q/k/v and gate/up each packed as one matrix (their rows concatenated at packing time,
    # the usual fused projections): 4 products per layer instead of 7, and X is staged once for the three (two)
    fused_m = (1, 2, 4, 8, 16, 32, 64)
    fused_layer = {m: best_us[(2, m)] + best_us[(1, m)] for m in fused_m}          # o and down as above
    for (r5, k5, mi) in ((3 * 4096, 4096, 3), (2 * 11008, 4096, 4)):
        w5 = synth.weights(r5, k5, synth.seed_for(5, mi))
        p5 = B.pack_2bitcsr(w5, B.prune_n4(w5, 2), 2, 128, B.VAL_INT4)
        c5 = max(2, -(-2 * LLC_BYTES // p5.nbytes()))
        pk5 = [p5.to(dev) for _ in range(c5)]
        for M in fused_m:
            X = up16(synth.activation_rows(M, k5, 5))
            Y = torch.empty((M, r5), dtype=torch.float16, device=dev)
            f5 = [B.prepared_sparse_gemm_smallm(pk5[i], X, Y) for i in range(c5)]
            best = timer(lambda i: f5[i % c5](), 200)["median"]
            need = B.smallm_ws_bytes(pk5[0], M)
            if need:
                ws = torch.empty(need, dtype=torch.uint8, device=dev)
                f5w = [B.prepared_sparse_gemm_smallm_ws(pk5[i], X, Y, ws) for i in range(c5)]
                best = min(best, timer(lambda i: f5w[i % c5](), 200)["median"])
                del f5w, ws
            fused_layer[M] += best * 1e6
            if mi == 3 and M == 16:
                qkv_fused_us = best * 1e6
            del f5
        del pk5, p5, w5
    # q/k/v as three matrices under the same 16 tokens: three launches against the batched entry point
    r5, k5, _, pk5 = pools[2]
    X = up16(synth.activation_rows(16, k5, 5))
    Ys = [torch.empty((16, r5), dtype=torch.float16, device=dev) for _ in range(3)]
    nq = len(pk5) // 3
    sep = [[B.prepared_sparse_gemm_smallm(pk5[3 * i + k], X, Ys[k]) for k in range(3)] for i in range(nq)]
    bat = [B.prepared_sparse_gemm_smallm_batch(pk5[3 * i:3 * i + 3], [X] * 3, Ys) for i in range(nq)]

    def run_sep(i):
        for c in sep[i % nq]:
            c()
    t["smallm_qkv_3x4096x4096_M16"] = {"three_launches_us": round(timer(run_sep, 200)["median"] * 1e6, 3),
                                        "one_batched_launch_us": round(timer(lambda i: bat[i % nq](), 200)["median"] * 1e6, 3),
                                        "one_matrix_of_12288_rows_us": round(qkv_fused_us, 3)}
    del sep, bat
    fused_a, fused_b = B.fit_verify_cost(list(fused_m[1:]), [fused_layer[m] for m in fused_m[1:]])
    fit_a, fit_b = B.fit_verify_cost(list(sweep_m[1:]), [layer_us[m] for m in sweep_m[1:]])
    cand = [64, 24, 9, 4, 2, 1]                      # candidates left per trie depth (wide top, narrow bottom)
    rem = [6, 5, 4, 3, 2, 1]                         # tokens still to generate (average ID length 6)
    depth, gain = B.trigger_depth(layer_us[1], fit_a, fit_b, cand, rem)
    # the same products in layer order through a 32-layer all-2:4 stack (224 launches per pass)
    stack_pass, stack_one = {}, {}
    for M in (1, 2, 4, 8, 16, 32, 64):
        seq, items = [], []
        for layer in range(32):
            for mi in (2, 2, 2, 2, 0, 0, 1):          # q, k, v, o, gate, up, down
                r5, k5, _, pk5 = pools[mi]
                X = up16(synth.activation_rows(M, k5, 5))
                Y = torch.empty((M, r5), dtype=torch.float16, device=dev)
                pk = pk5[(layer * 7 + len(items)) % len(pk5)]
                items.append((pk, X, Y))
                if M not in (1, 16, 64):
                    continue                          # (the 224 single launches: at three widths only)
                if (mi, M) in split_wins:
                    ws = torch.empty(B.smallm_ws_bytes(pk, M), dtype=torch.uint8, device=dev)
                    seq.append(B.prepared_sparse_gemm_smallm_ws(pk, X, Y, ws))
                else:
                    seq.append(B.prepared_sparse_gemm_smallm(pk, X, Y))

        def run_seq(i):
            for c in seq:
                c()
        if seq:
            stack_pass[str(M)] = round(timer(run_seq, 5, 1)["median"] * 1e6, 1)
        # the same 224 products as one table, one launch (one token: the M = 1 stack of Sec. 3.3's kernels)
        whole = (B.prepared_gemm_stack(items) if M >= 2 else
                 B.prepared_gemv_stack([("sparse", pk, X.view(-1), Y.view(-1)) for pk, X, Y in items]))
        stack_one[str(M)] = round(timer(lambda i: whole(), 5, 1)["median"] * 1e6, 1)
        del whole, seq, items
    one_m = [m for m in (2, 4, 8, 16, 32, 64)]
    one_a, one_b = B.fit_verify_cost(one_m, [stack_one[str(m)] for m in one_m])
    one_depth, one_gain = B.trigger_depth(stack_one["1"], one_a, one_b, cand, rem)
    t["trigger_model"] = {"layer_us_by_M": [round(layer_us[m], 2) for m in sweep_m], "M": [sweep_m[0], sweep_m[-1]],
                          "stack_pass_us_224_launches_by_M": stack_pass,
                          "stack_pass_us_one_launch_by_M": stack_one,
                          "one_launch": {"t_ar_us": stack_one["1"], "fit_a_us": round(one_a, 2), "fit_b_us_per_token": round(one_b, 3),
                                         "trigger_depth": one_depth, "benefit_us_per_pass": round(one_gain, 1)},
                          "stack_pass_us_32_times_layer_by_M": {str(m): round(32 * layer_us[m], 1) for m in (1, 16, 64)},
                          "fit_a_us": round(fit_a, 3), "fit_b_us_per_token": round(fit_b, 4),
                          "t_ar_us": round(layer_us[1], 2), "candidates": cand, "remaining": rem,
                          "trigger_depth": depth, "benefit_us_per_layer": round(gain, 2),
                          "fused_projections": {"layer_us_by_M": {str(m): round(fused_layer[m], 2) for m in fused_m},
                                                "launches_per_layer": 4, "fit_a_us": round(fused_a, 3),
                                                "fit_b_us_per_token": round(fused_b, 4)}}
    del pools
    # config 4: the 32-layer stack (every layer its own seeded weights), 224 launches in
    # sequence, plain and as a HIP graph; then with q/k/v and gate/up fused (128 launches)
    del packed[:], calls[:]
    torch.cuda.empty_cache()
    for plan, label in (("config4", "config4_stack"), ("mix3", "stack_mix3")):
        stk = S.LayerStack.build(dev, distinct_layers=None, plan=plan)
        t4 = timer(lambda i: stk.run(), 10, 2)
        row = {"launches_224_plain": entry(t4, stk.nbytes)}
        side = torch.cuda.Stream()
        fused = stk.fuse()

        def run_fused(i):
            for c in fused:
                c()
        row["launches_128_fused_plain"] = entry(timer(run_fused, 10, 2), stk.nbytes)
        layers = stk.per_layer()

        def run_layers(i):
            for c in layers:
                c()
        row["launches_32_one_per_layer"] = entry(timer(run_layers, 10, 2), stk.nbytes)
        whole = stk.one_launch()
        row["one_call_whole_stack"] = entry(timer(lambda i: whole(), 30, 5), stk.nbytes)
        row["one_call_whole_stack"]["launches"] = whole.plan.nparts      # 1:4 layers run as a launch of their own
        if plan == "config4":
            with torch.cuda.stream(side):
                stk.run(side.cuda_stream)
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    stk.run(torch.cuda.current_stream().cuda_stream)
                row["launches_224_graph"] = entry(timer(lambda i: graph.replay(), 10, 2), stk.nbytes)
                sp = side.cuda_stream
                for c in fused:
                    c(sp)
                torch.cuda.synchronize()
                graph_f = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph_f, stream=side):
                    sp = torch.cuda.current_stream().cuda_stream
                    for c in fused:
                        c(sp)
                row["launches_128_fused_graph"] = entry(timer(lambda i: graph_f.replay(), 10, 2), stk.nbytes)
            del graph, graph_f
        t[label] = row
        del stk, fused
        torch.cuda.empty_cache()
    return t


if __name__ == "__main__":
    main()
