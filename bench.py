#!/usr/bin/env python3
"""Benchmark of the layout-driven tensor copy on one MI355X.

A step is one call of lc_copy through the C ABI over one synthetic batch that is already resident in HBM: the first
call of a workload plans on the host (validate, coalesce, refine, sort, vector width, tile), every later call finds
that plan in the library's plan cache, so a timed step is plan look-up + launch + kernel.  Buffers rotate so that a
step never finds its data in the last-level cache.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c1|c2|c3|c4a|c4b|copy|gemm_tn|gemm_nt|calibrate] [--no-all] [--no-extra-passes]

Prints ONE JSON line.  The headline (`value`, `config`, `roofline`, `cpu_baseline`) is the largest single-GPU
configuration, workload 5 (NCHW -> NHWC, 2^30 fp32 elements, 8 GiB moved); `workloads` carries the same record for
every BASELINE configuration, all timed over the same --steps.  `roofline.kernel_ms` is measured live with HIP events
on the launch stream; `roofline.traffic` is NOT measured in this run: it is the HBM byte count per launch from the
committed rocprofv3 counter runs of this same command (profiles/hbm_traffic.json).  `cpu_baseline` times the CPU
oracle's element loop on a bounded sample of the same workload, single thread and on all host cores.
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
    return w.dram_minimum_bytes


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


def time_workload(torch, lc, w, dev, steps, warmup, stream, extra_passes=True):
    """Times one workload: ms per step through lc_copy by host clock, ms per launch by HIP events on the launch
    stream, the plan's text, the number of rotating buffer pairs, ms per launch inside a HIP graph (short kernels
    only), the source bits of buffer 0 on the host (for the oracle's baseline) and ms per launch when one buffer pair
    is used over and over (workloads whose footprint the last-level cache holds), and the median and minimum of the
    per-launch times of one more pass with an event after every launch."""
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
    # footprints that fit the last-level cache: the same launches on ONE buffer pair (warm), beside the rotating (cold) figure
    ms_warm = plan.time(sp[:1], dp[:1], warmup=min(warmup, 3), iters=steps, stream=stream) if (n > 1 and extra_passes) else None
    each = sorted(plan.time_each(sp, dp, warmup=min(warmup, 3), iters=steps, stream=stream)) if extra_passes else [float("nan")]
    desc = plan.describe()
    graph_ms = time_in_graph(torch, plan, sp, dp, steps) if (ms_kernel < 0.05 and extra_passes) else None
    src_host = srcs[0].cpu().numpy()
    del srcs, dsts
    torch.cuda.empty_cache()
    return ms_step, ms_kernel, desc, n, graph_ms, src_host, ms_warm, (each[len(each) // 2], each[0])


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


def cpu_model():
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, src_host, budget_single_s, budget_all_s):
    """The oracle's element loop (Sec. 2.6.1) on the host over a bounded prefix [0, m) of the workload's integral
    coordinates, on the bits of source buffer 0: single thread, then the same loop cut into one range per host core
    (the destination is injective, so the ranges do not interact)."""
    import numpy as np
    from oracle import pyoracle as oracle
    sl, dl = oracle.Layout(w.src_layout), oracle.Layout(w.dst_layout)
    dt = np.uint16 if w.elem_bytes == 2 else np.uint32
    src = src_host.view(dt)
    dst = np.empty(w.dst_elems, dtype=dt)        # pages are only touched where the sample writes

    def moved(m):   # bytes by the same count as the GPU figures: reads of distinct elements + writes
        return (min(m, w.distinct_reads) + m) * w.elem_bytes

    def single(m):
        t0 = time.perf_counter()
        oracle.copy(src, sl, dst, dl, 0, m, spans_checked=True)
        return time.perf_counter() - t0

    probe = min(w.n, 1 << 20)
    t_probe = single(probe)
    rate = probe / max(t_probe, 1e-6)            # coordinates per second, one thread
    m1 = int(min(w.n, max(probe, rate * budget_single_s)))
    t1 = single(m1)
    threads = oracle.host_threads(16)
    m2 = int(min(w.n, max(probe, rate * budget_all_s * threads * 0.6)))
    t0 = time.perf_counter()
    oracle.copy_parallel(src, sl, dst, dl, threads, 0, m2, spans_checked=True)
    t2 = time.perf_counter() - t0
    return {"value": round(moved(m1) / t1 / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "the first %d of %d integral coordinates of %s, %.1f s, single thread" % (m1, w.n, w.name, t1),
            "all_cores": {"value": round(moved(m2) / t2 / 1e9, 4), "unit": "GB/s", "cores": threads,
                          "sample": "the first %d of %d integral coordinates, one range per thread, %.1f s" % (m2, w.n, t2)},
            "cpu_model": cpu_model(), "host_cores_visible": os.cpu_count()}


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
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--no-all", action="store_true", help="time the headline workload only (no `workloads` map, no GEMM)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-passes", action="store_true",
                    help="only the warm-up, the timed steps and the event-timed launches on rotating buffers (no cache-warm pass, no "
                         "per-launch pass, no graph replay): what the kernel traces under profiles/ are taken with")
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

    if args.workload == "calibrate":
        # For the counter runs only: two library kernels with traffic on ONE side that is known independently of this
        # library -- a sum over 2^28 int32 (reads 2^30 bytes, writes next to nothing) and a fill of 2^28 int32 (writes
        # 2^30 bytes, reads nothing).  rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this run gives the counters' scale.
        x = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        y = torch.empty(1 << 28, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            x.sum()
        torch.cuda.synchronize()
        for _ in range(args.steps):
            y.fill_(7)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": {"read_only": "torch.sum over 2^28 int32: 2^30 bytes read per call, %d calls" % args.steps,
                                          "write_only": "torch.Tensor.fill_ of 2^28 int32: 2^30 bytes written per call, %d calls" % args.steps}}))
        return

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

    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic_table = json.load(open(tpath))
    traffic_note = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by the same "
                    "counters on the plain copy; a committed measurement, not taken in this run")

    def record(name, headline):
        w = W.workload(name)
        ms_step, ms_kernel, desc, n_pairs, graph_ms, src_host, ms_warm, (ms_median, ms_min) = time_workload(torch, lc, w, dev, args.steps, args.warmup, stream, not args.no_extra_passes)
        sec = ms_kernel * 1e-3
        achieved = w.dram_minimum_bytes / sec / 1e9
        rec = {
            "workload": w.name, "src_layout": w.src_layout, "dst_layout": w.dst_layout, "elements": w.n, "dtype": w.dtype,
            "algorithmic_bytes": w.algorithmic_bytes, "dram_minimum_bytes": w.dram_minimum_bytes,
            "steps": args.steps, "warmup": args.warmup, "rotating_buffer_pairs": n_pairs,
            "ms_per_step": round(ms_step, 5), "value": round(w.algorithmic_bytes / (ms_step * 1e-3) / 1e9, 2), "unit": "GB/s",
            "ms_per_step_in_hip_graph": None if graph_ms is None else round(graph_ms, 5),
            # achieved / frac are on the bytes HBM has to move (for the pure permutations these are the algorithmic bytes;
            # the stride-3 gather drags whole sectors along: 2x; the broadcast's algorithmic count already reads its source once)
            "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic_table.get(w.name),
                         "traffic_source": traffic_note, "kernel_ms": round(ms_kernel, 5),
                         "kernel_ms_one_buffer_pair_cache_warm": None if ms_warm is None else round(ms_warm, 5),
                         # a second pass over the same launches with an event between every two (adds about a microsecond
                         # per launch to kernels of a few microseconds): the median and the fastest of the --steps launches
                         "kernel_ms_median_event_per_launch": None if ms_median != ms_median else round(ms_median, 5),
                         "kernel_ms_min_event_per_launch": None if ms_min != ms_min else round(ms_min, 5),
                         "bytes_priced": "dram_minimum_bytes",
                         "achieved_algorithmic": round(w.algorithmic_bytes / sec / 1e9, 2),
                         "frac_algorithmic": round(w.algorithmic_bytes / sec / 1e9 / HBM_PEAK_GBS, 4)},
            "plan": desc,
        }
        if not args.no_cpu_baseline:
            rec["cpu_baseline"] = cpu_baseline(w, src_host, 8.0 if headline else 1.5, 4.0 if headline else 1.5)
        return rec

    # The workloads with the smallest footprints are timed first, the headline (the largest) last: physical memory that
    # has gone through the 8 GiB allocations comes back to later, small allocations in scattered pieces, and the kernels of
    # 5-25 us feel where their buffers lie (+/- 1.5 % from one allocation to the next).
    others = {}
    if not args.no_all:
        footprint = lambda name: (W.workload(name).src_elems + W.workload(name).dst_elems) * W.workload(name).elem_bytes
        for name in sorted((n for n in W.WORKLOAD_NAMES + ["copy"] if n != args.workload), key=footprint):
            r = record(name, False)
            others[r["workload"]] = r
    head = record(args.workload, True)
    out = {
        "metric": "effective HBM GB/s (read+write) of layout-to-layout copy",
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "u32", "bf16": "u16", "f16": "u16"}[head["dtype"]] + " bit patterns (%s elements), int32/int64 index arithmetic" % head["dtype"],
        "data": "synthetic, seeded; %d rotating buffer pair(s) resident in HBM" % head["rotating_buffer_pairs"],
        "config": {"workload": head["workload"], "src_layout": head["src_layout"], "dst_layout": head["dst_layout"],
                   "elements": head["elements"], "algorithmic_bytes": head["algorithmic_bytes"], "plan": head["plan"]},
        "pct_of_hbm_peak": round(100.0 * head["value"] / HBM_PEAK_GBS, 2),
        "roofline": head["roofline"],
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if not args.no_all:
        allw = dict(others)
        allw[head["workload"]] = head
        out["workloads"] = dict(sorted(allw.items()))
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
    print(json.dumps(out))


if __name__ == "__main__":
    main()
