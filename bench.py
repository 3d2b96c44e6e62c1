#!/usr/bin/env python3
"""Benchmark of the layout-driven tensor copy on one MI355X.

A step is one pass of the whole hot path — validate, coalesce, refine, sort, vector width, tile
(all host), launch, kernel — through the C ABI call lc_copy, over one synthetic batch that is
already resident in HBM.  Buffers rotate so that a step never finds its data in the last-level cache.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c1|c3|c4a|c4b|c5|copy|gemm_tn|gemm_nt] [--no-all]

Prints ONE JSON line (see the keys below).  `roofline` is measured live with HIP events on the
launch stream; `cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak, GB/s
MFMA_PEAK_TFLOPS = 2500.0      # MI355X published dense bf16 / fp16 matrix peak, TFLOP/s
CACHE_BYTES = 256 << 20        # last-level (Infinity) cache; rotation covers at least 4x this


def dram_minimum_bytes(w):
    """HBM bytes the workload cannot avoid: every 32-byte sector of the source span that is touched,
    plus every destination byte."""
    if w.name.startswith("c4a"):
        return 3 * w.n * 4 + w.n * 4          # stride 3: all sectors of the 3n-element span are fetched
    if w.name.startswith("c4b"):
        return (w.n // 16) * 4 + w.n * 4      # the broadcast source is read once
    return w.algorithmic_bytes


def make_buffers(torch, w, dev, rotate_bytes):
    import numpy as np
    from paper_2603_02298_amd import workloads as W
    per_pair = (w.src_elems + w.dst_elems) * w.elem_bytes
    n_pairs = max(1, min(16, -(-rotate_bytes // per_pair)))
    tdt = torch.int16 if w.elem_bytes == 2 else torch.int32
    srcs, dsts = [], []
    if w.src_elems <= (1 << 26):
        bits = W.source_bits(w)
        first = torch.from_numpy(bits.view(np.int16 if w.elem_bytes == 2 else np.int32)).to(dev)
    else:  # generating 2^30 values with numpy would dominate the run: seeded device generator, same distribution
        g = torch.Generator(device=dev)
        g.manual_seed(W.SEED_BASE + int(w.name[1]))
        if w.values == "normal":
            x = torch.randn(w.src_elems, device=dev, generator=g, dtype=torch.float32)
        elif w.values == "uniform":
            x = torch.rand(w.src_elems, device=dev, generator=g, dtype=torch.float32) * 2 - 1
        else:
            x = torch.randint(0, 1 << 20, (w.src_elems,), device=dev, generator=g).to(torch.float32)
        if w.dtype == "bf16":
            x = x.to(torch.bfloat16)
        elif w.dtype == "f16":
            x = x.to(torch.float16)
        first = x.view(tdt)
    for k in range(n_pairs):
        srcs.append(first if k == 0 else first.clone())
        dsts.append(torch.zeros(w.dst_elems, dtype=tdt, device=dev))
    return srcs, dsts


def time_workload(torch, lc, w, dev, steps, warmup, stream):
    """Returns (ms per step through lc_copy by host clock, ms per launch by HIP events, plan text)."""
    srcs, dsts = make_buffers(torch, w, dev, 4 * CACHE_BYTES)
    sl, dl = lc.Layout(w.src_layout), lc.Layout(w.dst_layout)
    n = len(srcs)
    sp = [t.data_ptr() for t in srcs]
    dp = [t.data_ptr() for t in dsts]
    for k in range(warmup):
        lc.lc_copy(sp[k % n], sl, dp[k % n], dl, w.dtype, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        lc.lc_copy(sp[k % n], sl, dp[k % n], dl, w.dtype, stream)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    plan = lc.Plan(w.src_layout, w.dst_layout, w.dtype)
    ms_kernel = plan.time(sp, dp, warmup=min(warmup, 3), iters=steps, stream=stream)
    desc = plan.describe()
    graph_ms = time_in_graph(torch, plan, sp, dp, steps) if ms_kernel < 0.05 else None
    del srcs, dsts
    torch.cuda.empty_cache()
    return ms_step, ms_kernel, desc, n, graph_ms


def time_in_graph(torch, plan, sp, dp, steps):
    """ms per launch when the launches (one per buffer pair) are recorded once into a HIP graph and replayed: what a
    launch-bound caller gets (short kernels: the eager step is mostly launch overhead)."""
    side = torch.cuda.Stream()
    n = len(sp)
    with torch.cuda.stream(side):
        plan.execute(sp[0], dp[0], side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for k in range(n):
            plan.execute(sp[k], dp[k], torch.cuda.current_stream().cuda_stream)
    reps = max(3, steps // n)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / (reps * n)


def cpu_baseline(w, budget_s=15.0):
    """The oracle's element loop on the host, on a bounded prefix of the workload's integral coordinates."""
    import numpy as np
    from oracle import pyoracle as oracle
    from paper_2603_02298_amd import workloads as W
    sl, dl = oracle.Layout(w.src_layout), oracle.Layout(w.dst_layout)
    probe = min(w.n, 1 << 20)
    # the sample is a prefix [0, m): buffers only need to cover the offsets that prefix reaches
    def span(layout, m):
        return int(layout.offsets(0, m).max()) + 1 if m <= (1 << 25) else layout.cosize
    dt = np.uint16 if w.elem_bytes == 2 else np.uint32
    src_all = None
    def run(m):
        nonlocal src_all
        s_need, d_need = span(sl, m), span(dl, m)
        if src_all is None or src_all.size < s_need:
            src_all = W.source_bits(w, elems=s_need)
        dst = np.zeros(d_need, dtype=dt)
        t0 = time.perf_counter()
        oracle.copy(src_all[:max(s_need, 1)], sl, dst, dl, 0, m, spans_checked=True)
        return time.perf_counter() - t0
    t_probe = run(probe)
    m = int(min(w.n, max(probe, probe * budget_s / max(t_probe, 1e-6))))
    if m > (1 << 22):
        m = min(m, 1 << 25)
    t = run(m) if m > probe else t_probe
    # a short sample is repeated until about ten seconds of oracle work have been timed
    passes = 1
    while t < 10.0 and passes < 16:
        t += run(m)
        passes += 1
    gbs = 2.0 * m * passes * w.elem_bytes / t / 1e9
    return {"value": round(gbs, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d passes over the first %d of %d integral coordinates of %s, %.1f s, single thread" % (passes, m, w.n, w.name, t)}


def time_gemm(torch, lc, name, dev, steps, warmup, stream, size=8192):
    """The second workload (generic GEMM, 8192^3 bf16): kernel time by HIP events on the launch stream and the
    host-clock time of lc_gemm (plan + launch + kernel).  Inputs N(0,1) from torch's seeded device generator."""
    from paper_2603_02298_amd import workloads as W
    w = W.gemm_workload(name, size, size, size, "bf16")
    g = torch.Generator(device=dev)
    g.manual_seed(W.SEED_BASE + 100)
    a = torch.randn(w.a_elems, device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    b = torch.randn(w.b_elems, device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    c = torch.zeros(w.c_elems, device=dev, dtype=torch.float32)
    la, lb, lcc = lc.Layout(w.a_layout), lc.Layout(w.b_layout), lc.Layout(w.c_layout)
    for _ in range(warmup):
        lc.lc_gemm(a.data_ptr(), la, b.data_ptr(), lb, c.data_ptr(), lcc, "bf16", stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        lc.lc_gemm(a.data_ptr(), la, b.data_ptr(), lb, c.data_ptr(), lcc, "bf16", stream)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    plan = lc.GemmPlan(w.a_layout, w.b_layout, w.c_layout, "bf16")
    ms_kernel = plan.time(a.data_ptr(), b.data_ptr(), c.data_ptr(), min(warmup, 3), steps, stream)
    desc = plan.describe()
    vendor = None
    if name in ("tn", "nt"):
        # for scale only: the vendor library behind torch.matmul on the same operands (bf16 result, no read of C)
        if name == "tn":     # A (M,K) and B (N,K) row-major: C = A B^T
            am, bm = a.view(size, size), b.view(size, size).t()
        else:                # A (M,K):(1,M) is a (K,M) row-major matrix transposed, B (N,K):(1,N) likewise
            am, bm = a.view(size, size).t(), b.view(size, size)
        for _ in range(3):
            torch.matmul(am, bm)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            torch.matmul(am, bm)
        torch.cuda.synchronize()
        vendor = (time.perf_counter() - t0) * 1e3 / steps
    del a, b, c
    torch.cuda.empty_cache()
    return w, ms_step, ms_kernel, desc, vendor


def gemm_record(w, ms_step, ms_kernel, desc):
    tf_kernel = w.flops / (ms_kernel * 1e-3) / 1e12
    traffic = None   # HBM bytes per launch from the committed counter runs (profiles/), when this workload has one
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(w.name)
    return {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "a_layout": w.a_layout, "b_layout": w.b_layout, "c_layout": w.c_layout,
            "flops": w.flops, "ms_per_step": round(ms_step, 5), "TFLOPs_whole_call": round(w.flops / (ms_step * 1e-3) / 1e12, 1),
            "roofline": {"bound": "mfma", "achieved": round(tf_kernel, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf_kernel / MFMA_PEAK_TFLOPS, 4), "traffic": traffic, "kernel_ms": round(ms_kernel, 5)},
            "plan": desc}


def gemm_cpu_baseline(name, budget_s=10.0):
    """The oracle's GEMM sum for sampled entries of C of the 8192^3 problem, single thread."""
    import numpy as np
    from oracle import pyoracle as oracle
    from paper_2603_02298_amd import workloads as W
    w = W.gemm_workload(name, 8192, 8192, 8192, "bf16")
    rng = np.random.default_rng(W.SEED_BASE + 103)
    a = rng.standard_normal(w.a_elems)
    b = rng.standard_normal(w.b_elems)
    c = np.zeros(w.c_elems)
    count, t, done = 16, 0.0, 0
    while t < budget_s and done < 4096:
        ms, ns = rng.integers(0, w.M, count), rng.integers(0, w.N, count)
        t0 = time.perf_counter()
        oracle.gemm_at(a, w.a_layout, b, w.b_layout, c, w.c_layout, ms, ns)
        t += time.perf_counter() - t0
        done += count
    return {"value": round(2.0 * done * w.K / t / 1e9, 4), "unit": "GFLOP/s", "cores": 1, "kind": "oracle",
            "sample": "%d sampled entries of C of %s (K = %d each), %.1f s, single thread" % (done, w.name, w.K, t)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-all", action="store_true", help="skip timing the other workloads (reported under all_workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path has no multi-GPU part (how it would shard is described in the design notes)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2603_02298_amd as lc
    from paper_2603_02298_amd import workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the copy only runs in the HIP kernels", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream

    if args.workload.startswith("gemm_"):
        # the second workload as the headline of this run (used for its profiles)
        gw, ms_step, ms_kernel, desc, _vendor = time_gemm(torch, lc, args.workload[5:], dev, args.steps, args.warmup, stream)
        rec = gemm_record(gw, ms_step, ms_kernel, desc)
        out = {"metric": "TFLOP/s of the layout-driven GEMM (second workload)", "value": rec["TFLOPs_whole_call"], "unit": "TFLOP/s",
               "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"], "higher_is_better": True,
               "scaling": "weak", "vs_baseline": None, "dtype": "bf16 operands, fp32 accumulation (MFMA)", "data": "synthetic, seeded N(0,1)",
               "config": {"workload": gw.name, "M": gw.M, "N": gw.N, "K": gw.K, "plan": desc}, "roofline": rec["roofline"]}
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = gemm_cpu_baseline(args.workload[5:])
        print(json.dumps(out))
        return

    w = W.workload(args.workload)
    ms_step, ms_kernel, desc, n_pairs, graph_ms = time_workload(torch, lc, w, dev, args.steps, args.warmup, stream)
    value = w.algorithmic_bytes / (ms_step * 1e-3) / 1e9
    achieved = w.algorithmic_bytes / (ms_kernel * 1e-3) / 1e9
    dram_min = dram_minimum_bytes(w)

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(w.name)

    out = {
        "metric": "effective HBM GB/s (read+write) of layout-to-layout copy",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "u32", "bf16": "u16", "f16": "u16"}[w.dtype] + " bit patterns (%s elements), int32/int64 index arithmetic" % w.dtype,
        "data": "synthetic, seeded; %d rotating buffer pairs resident in HBM" % n_pairs,
        "config": {"workload": w.name, "src_layout": w.src_layout, "dst_layout": w.dst_layout, "elements": w.n,
                   "algorithmic_bytes": w.algorithmic_bytes, "plan": desc},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "ms_per_step_in_hip_graph": None if graph_ms is None else round(graph_ms, 5),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "kernel_ms": round(ms_kernel, 5), "dram_minimum_bytes": dram_min,
                     "frac_dram_minimum": round(dram_min / (ms_kernel * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
    }
    if not args.no_all:
        allw = {}
        for name in W.WORKLOAD_NAMES + ["copy"]:
            if name == args.workload:
                continue
            wk = W.workload(name)
            st, kt, d, _, gms = time_workload(torch, lc, wk, dev, max(10, args.steps // 4), 3, stream)
            allw[wk.name] = {"ms_per_step": round(st, 5), "kernel_ms": round(kt, 5),
                             "ms_per_step_in_hip_graph": None if gms is None else round(gms, 5),
                             "GBps_algorithmic": round(wk.algorithmic_bytes / (kt * 1e-3) / 1e9, 1),
                             "frac_of_peak_dram_minimum": round(dram_minimum_bytes(wk) / (kt * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                             "plan": d}
        out["all_workloads"] = allw
        # second workload (generic GEMM on the matrix cores): reported beside the copy, not part of `value`
        gemm = {}
        for name in ("tn", "nt"):
            gw, st, kt, d, vendor_ms = time_gemm(torch, lc, name, dev, 20, 3, stream)
            gemm[gw.name] = gemm_record(gw, st, kt, d)
            if vendor_ms:
                gemm[gw.name]["vendor_library_for_scale"] = {
                    "what": "torch.matmul on the same operands in the same memory layouts: C = A B^T in bf16, no accumulation into an fp32 C",
                    "ms_per_step": round(vendor_ms, 5), "TFLOPs": round(gw.flops / (vendor_ms * 1e-3) / 1e12, 1)}
        out["gemm"] = gemm
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
