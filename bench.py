#!/usr/bin/env python3
"""Benchmark of the padded-convolution-as-SpMM path on one MI355X.

Workload: the headline shape (m, n, k, s, p) = (1024, 1024, 7, 1, 3) with a
batch of 16 vectors sharing T.  A step is one apply y = T x with T already
built and x, T resident in HBM (the method builds T once and then applies it,
paper Section 2); the build is timed in the same run and reported beside it.

Prints ONE JSON line: effective HBM GB/s of the apply (model bytes = entries *
(index + value) + row_ptr + x once + y once, divided by the time per step),
useful MAC/s, build time, the roofline of the apply kernel (HIP events on the
launch stream), a table of all named configurations and the CPU oracle timed on
this host.  Everything the headline figures rest on is timed on ONE stream,
after the device has settled (see precondition).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
FP32_VECTOR_PEAK_TFLOPS = 157.3   # MI355X published fp32 vector peak (256 CUs x 128 FMA/clk x 2.4 GHz, packed fp32)
FP32_UNPACKED_PEAK_TFLOPS = 78.6  # the same units issuing one fp32 FMA per lane: 256 CUs x 64 FMA/clk x 2.4 GHz


def cpu_baseline(w, x, K, transposed=False):
    """The oracle as it stands, timed on the host cores on the whole workload
    (one call as warm-up, then the median of repeated calls within ~20 s)."""
    import numpy as np
    import oracle
    m, n, k, s, p = w.shape
    oracle.conv(32, 32, 3, 1, 1, np.zeros(1024, np.float32), np.zeros(9, np.float32))   # load the library
    times = []
    t_all = time.perf_counter()
    while len(times) < 5 and (time.perf_counter() - t_all < 20.0 or not times):
        t0 = time.perf_counter()
        (oracle.conv_t if transposed else oracle.conv)(m, n, k, s, p, x, K, batch=w.batch)
        times.append(time.perf_counter() - t0)
    med = sorted(times)[len(times) // 2]
    nnz = oracle.nnz_closed(m, n, k, s, p)
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    out = {
        "value": nnz * w.batch / med / 1e9, "unit": "GMAC/s (useful: closed-form nnz x batch / s)",
        "seconds_per_apply": med, "cores": cores, "kind": "oracle",
        "sample": "whole workload %s (%d calls, median); explicit zero-pad + sliding window, "
                  "fp64 accumulation, OpenMP over output lines" % (w.name, len(times)),
        "cpu_model": cpu_model(),
    }
    # the same call on one thread (one call: the oracle is a correctness reference, not a tuned baseline)
    try:
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        t0 = time.perf_counter()
        (oracle.conv_t if transposed else oracle.conv)(m, n, k, s, p, x, K, batch=w.batch)
        out["one_thread_gmac_per_s"] = nnz * w.batch / (time.perf_counter() - t0) / 1e9
        gomp.omp_set_num_threads(cores)
    except OSError:
        pass
    return out


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def launch_shape(cs, shape, batch, storage=0):
    """Workgroups x threads and dynamic LDS bytes of the launch conv_spmv makes for this shape."""
    d = cs.conv_dispatch_info(*shape, batch=batch, storage=storage)
    return "%dx%d lds %d" % (d.workgroups, d.threads, d.lds_bytes)


def measured_traffic(variant, launch):
    """HBM bytes per launch of the apply kernel from the committed rocprofv3 counter summary, or
    None when there is none for this variant and launch shape, or when the source files the
    kernel is compiled from (the summary names them) have changed since the counters were taken."""
    import glob
    import hashlib
    for fn in glob.glob(os.path.join(ROOT, "profiles", "*.txt")):
        fields = {}
        with open(fn) as fh:
            for line in fh:
                if ":" in line:
                    key, _, val = line.strip().partition(":")
                    fields[key.strip()] = val.strip()
        if fields.get("traffic_kernel") != variant or fields.get("traffic_launch") != launch:
            continue
        h = hashlib.sha256()
        try:
            for name in fields.get("traffic_sources", "").split():
                with open(os.path.join(ROOT, "paper_2411_19419_amd", "csrc", name), "rb") as fh:
                    h.update(fh.read())
        except OSError:
            continue
        if fields.get("traffic_sources_sha256") == h.hexdigest():
            return int(fields["traffic_bytes_per_launch"])
    return None


def sweep_main(args):
    """Second workload: the paper's experiment (Section 4.1, Table 2) -- 123 single-channel
    layer shapes, a random-normal input and kernel per layer, total time over the list
    (the quantity of the paper's Table 1).  A step is one sweep over all 123 layers with
    the 123 matrices already built.  Three ways to run it are timed: one conv_spmv launch
    per layer on one stream, the same 123 launches replayed from a HIP graph, and all
    layers in one launch (conv_multi_apply)."""
    import numpy as np
    import torch

    import paper_2411_19419_amd as cs
    from paper_2411_19419_amd import workloads

    dev = torch.device("cuda:0")
    batch = args.batch
    layers = list(workloads.densenet121_sweep(batch=batch))
    plans = [cs.conv_csr_build(*shape, torch.from_numpy(K).to(dev)) for shape, _, K in layers]
    xs = [torch.from_numpy(x).to(dev) for _, x, _ in layers]
    ys = [torch.empty(pl.rows * batch, dtype=torch.float32, device=dev) for pl in plans]
    ys_fused = [torch.empty_like(y) for y in ys]
    multi = cs.ConvMulti(plans, xs, ys_fused, batch=batch)
    stream = torch.cuda.current_stream()
    steps, warmup = args.steps, args.warmup

    def eager():
        for pl, x, y in zip(plans, xs, ys):
            cs.conv_spmv(pl, x, y, batch=batch)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / steps

    us_eager = timed(eager)
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        eager()
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        eager()
    us_graph = timed(graph.replay)
    us_fused = timed(multi.apply)
    # the three ways agree (graph replays are checked against the eager results after real work in between)
    eager()
    torch.cuda.synchronize()
    want = [y.clone() for y in ys]
    for y in ys:
        y.zero_()
    graph.replay()
    multi.apply()
    torch.cuda.synchronize()
    worst = 0.0
    for w_, y, yf in zip(want, ys, ys_fused):
        assert torch.equal(w_, y), "graph replay differs from eager launches"
        scale = float(w_.abs().max()) or 1.0
        worst = max(worst, float((yf - w_).abs().max()) / scale)
    assert worst <= 1e-5, worst

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(steps, 100))]
    for a, b in ev:
        a.record(stream)
        multi.apply()
        b.record(stream)
    torch.cuda.synchronize()
    kern_us = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    kern_avg = sum(kern_us) / len(kern_us)
    model_bytes = sum(pl.model_bytes(batch) for pl in plans)
    nnz = sum(pl.nnz for pl in plans)
    out = {
        "metric": "DenseNet121 layer sweep (paper Table 2: 123 single-channel shapes), total time per sweep, all "
                  "layers in one launch",
        "value": us_fused, "unit": "us", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": us_fused * 1e-3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": us_fused / 9187.0, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "densenet121_sweep", "layers": len(plans), "batch": batch, "nnz_total": nnz},
        "us_per_sweep": {"one_launch_per_layer": us_eager, "hip_graph_of_123_launches": us_graph,
                         "one_launch_for_all_layers": us_fused},
        "paper_table1_us": {"CSR-T (PyTorch, GTX 1070)": 9187, "CSR-C (SciPy, i7-8700)": 1507,
                            "note": "Python proof of concept on other hardware, precision not stated: context only; "
                                    "vs_baseline is value / 9187"},
        "useful_mac_per_s": nnz * batch / (us_fused * 1e-6),
        "roofline": {"bound": "hbm", "achieved": model_bytes / (kern_avg * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": model_bytes / (kern_avg * 1e-6) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "spmm_multi_kernel", "kernel_us_avg": kern_avg, "kernel_us_min": kern_us[0],
                     "note": "8.6 MB of operands, resident in L2 / last-level cache: launch- and latency-bound, "
                             "not an HBM measurement"},
    }
    if not args.no_cpu:
        import oracle
        times = []
        for _ in range(3):
            t0 = time.perf_counter()
            for shape, x, K in layers:
                oracle.conv(*shape, x, K, batch=batch)
            times.append(time.perf_counter() - t0)
        med = sorted(times)[1]
        out["cpu_baseline"] = {"value": med * 1e6, "unit": "us per sweep", "cores": int(os.environ.get(
            "OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0)), "kind": "oracle",
            "sample": "whole sweep, 123 oracle.conv calls through ctypes (median of 3)"}
    multi.close()
    for pl in plans:
        pl.close()
    print(json.dumps(out))


def event_times_ms(fn, count, stream):
    """`count` calls of fn, each between its own pair of HIP events on `stream`: sorted durations in ms."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(count)]
    for a, b in evs:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in evs)


def precondition(fn, stream, cap_s=0.5, batch_len=50, tol=0.01):
    """Run fn until the device has settled: after an idle period the shader clock ramps for some
    tens of milliseconds (measured: 1.4 -> 2.4 GHz over the first ~250 launches of the headline
    apply, whose duration follows it, 133 -> 112 us), so launches are issued in batches of 50, each
    between its own events, until the median of a batch is within 1 % of the batch before, for at
    most half a second.  Independent of --warmup.  Returns (launches, last median in ms)."""
    t0 = time.perf_counter()
    launches, prev = 0, None
    while True:
        med = event_times_ms(fn, batch_len, stream)[batch_len // 2]
        launches += batch_len
        if prev is not None and abs(med - prev) <= tol * prev and launches >= 3 * batch_len:
            return launches, med
        if time.perf_counter() - t0 > cap_s:
            return launches, med
        prev = med


LLC_BYTES = 256 * 1024 * 1024     # Infinity Cache: a working set below this does not measure HBM


def config_entry(cs, oracle, workloads, name, dev, stream, launches=60):
    """One named workload, single stream: variant, median / min us of event-bracketed launches after
    the device has settled and the average of the same number of launches back to back, model bytes
    and rate, useful MAC/s, error against the oracle."""
    import numpy as np
    import torch
    w = workloads.WORKLOADS[name]
    m, n, k, s, p = w.shape
    x_h, K_h = workloads.make(w)
    x = torch.from_numpy(x_h).to(dev)
    plan = cs.conv_csr_build(m, n, k, s, p, torch.from_numpy(K_h).to(dev))
    y = torch.empty(plan.rows * w.batch, dtype=torch.float32, device=dev)
    fn = lambda: cs.conv_spmv(plan, x, y, batch=w.batch)
    pre, _ = precondition(fn, stream, cap_s=0.25)
    ms = event_times_ms(fn, launches, stream)
    med, mn = ms[len(ms) // 2], ms[0]
    # the same launches back to back between two events (no gap between a launch and its events)
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record(stream)
    for _ in range(launches):
        fn()
    r1.record(stream)
    torch.cuda.synchronize()
    b2b = r0.elapsed_time(r1) / launches
    ref, scale = oracle.conv(m, n, k, s, p, x_h, K_h, batch=w.batch, want_scale=True)
    got = y.cpu().numpy().astype(np.float64)
    err = np.abs(got - ref.astype(np.float64))
    live = scale > 0
    rel = err[live] / np.maximum(np.abs(ref[live]).astype(np.float64), 1e-300)
    model = plan.model_bytes(w.batch)
    out = {
        "shape": [m, n, k, s, p], "batch": w.batch, "variant": plan.variant(w.batch),
        "us_median": med * 1e3, "us_min": mn * 1e3, "us_back_to_back": b2b * 1e3,
        "frac_of_hbm_peak_back_to_back": model / (b2b * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "launches": launches, "precondition_launches": pre,
        "model_bytes": model, "model_gbs": model / (med * 1e-3) / 1e9,
        "frac_of_hbm_peak": model / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "cache_resident": bool(model < LLC_BYTES),
        "useful_mac_per_s": plan.nnz * w.batch / (med * 1e-3),
        "max_err_over_scale": float(np.max(err[live] / scale[live])) if np.any(live) else 0.0,
        "normwise_err": float(np.max(err) / max(float(np.max(np.abs(ref))), 1e-300)),
        "rel_err_vs_ref": {"median": float(np.median(rel)), "p99": float(np.quantile(rel, 0.99)), "max": float(np.max(rel))},
    }
    plan.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams of the extra 'applies in flight' measurement (0 or 1: skip it)")
    ap.add_argument("--workload", default=None,
                    help="name in workloads.WORKLOADS (default: the headline), or densenet121_sweep")
    ap.add_argument("--batch", type=int, default=1, help="batch of the densenet121_sweep workload")
    ap.add_argument("--transposed", action="store_true",
                    help="build T column-compressed and time y = T^T x (the adjoint) instead")
    ap.add_argument("--compact", action="store_true",
                    help="build T in the structure-aware storage (row descriptors + k*k table) and time y = T x from it")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-side-paths", action="store_true",
                    help="skip the brief timing of the structure-aware storage and of T^T on the same workload")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration table of the named workloads")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path is built and timed on a single MI355X "
                 "(--gpus %d is not supported)" % args.gpus)

    import numpy as np
    import torch

    import __graft_entry__ as entry
    if not os.path.exists(entry.LIB):
        entry.build_library()
    import paper_2411_19419_amd as cs
    from paper_2411_19419_amd import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.workload == "densenet121_sweep":
        return sweep_main(args)
    dev = torch.device("cuda:0")
    w = workloads.WORKLOADS[args.workload or workloads.HEADLINE]
    m, n, k, s, p = w.shape
    x_h, K_h = workloads.make(w)
    if args.transposed:      # the operand of T^T has the size of the convolution's output
        mo_, no_ = cs.conv_out_shape(m, n, k, s, p)
        x_h = workloads.make_input(mo_, no_, w.batch, w.x_dist, w.seed + 100)
    x = torch.from_numpy(x_h).to(dev)
    K = torch.from_numpy(K_h).to(dev)
    stream = torch.cuda.current_stream()

    # ---- build (row_ptr + fill kernels; allocation of the CSR arrays excluded from the event time)
    if args.compact and args.transposed:
        sys.exit("--compact stores T; it has no transposed variant")
    build_py = cs.conv_compact_build if args.compact else (cs.conv_csc_build if args.transposed else cs.conv_csr_build)
    plan = build_py(m, n, k, s, p, K)
    torch.cuda.synchronize()
    build_ms = []
    lib = cs.binding._load()
    import ctypes
    for _ in range(5):
        h = ctypes.c_void_p()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        if args.compact:
            st = lib.conv_compact_build(m, n, k, s, p, K.data_ptr(), plan.row_desc.data_ptr(), plan.ktab.data_ptr(),
                                        ctypes.c_void_p(stream.cuda_stream), ctypes.byref(h))
        else:
            build_fn = lib.conv_csc_build if args.transposed else lib.conv_csr_build
            st = build_fn(m, n, k, s, p, K.data_ptr(), plan.row_ptr.data_ptr(), plan.col_idx.data_ptr(),
                          plan.vals.data_ptr(), ctypes.c_void_p(stream.cuda_stream), ctypes.byref(h))
        e1.record(stream)
        torch.cuda.synchronize()
        assert st == 0
        lib.conv_plan_destroy(h)
        build_ms.append(e0.elapsed_time(e1))
    build_med = sorted(build_ms)[len(build_ms) // 2]

    y = torch.empty(plan.rows * w.batch, dtype=torch.float32, device=dev)
    apply_once = lambda: cs.conv_spmv(plan, x, y, batch=w.batch)

    # ---- the device settles first (clock ramp after idle), whatever --warmup says
    pre_launches, pre_median = precondition(apply_once, stream)

    # ---- W warm-up steps, then exactly K steps on ONE stream between two synchronisations.  Two HIP
    # events on that stream bracket the K launches: elapsed / K is the kernel's average launch
    # duration over the timed region, the figure of the roofline.
    for _ in range(args.warmup):
        apply_once()
    torch.cuda.synchronize()
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    r0.record(stream)
    for _ in range(args.steps):
        apply_once()
    r1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    region_avg = r0.elapsed_time(r1) / args.steps

    # ---- single launches, each between its own pair of events (includes the gap between two
    # launches, a few microseconds): median and minimum
    kern_ms = event_times_ms(apply_once, max(min(args.steps, 100), 20), stream)
    kern_avg = sum(kern_ms) / len(kern_ms)

    # ---- extra: the same applies issued in turn on several streams (independent batches through one
    # T, each stream with its own y).  The applies in flight then share T through the L2 and the
    # Infinity Cache, so this is a throughput of a stream of batches, NOT an HBM bandwidth figure.
    overlapped = None
    if args.streams > 1:
        side = [torch.cuda.Stream() for _ in range(args.streams)]
        ys = [torch.empty_like(y) for _ in range(args.streams)]

        def run_steps(count):
            for q in side:
                q.wait_stream(stream)
            for i in range(count):
                j = i % len(side)
                cs.conv_spmv(plan, x, ys[j], batch=w.batch, stream=side[j])
            for q in side:
                stream.wait_stream(q)

        run_steps(max(args.warmup, 3 * args.streams))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(args.steps)
        torch.cuda.synchronize()
        ov_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        overlapped = {"streams": args.streams, "ms_per_apply": ov_ms,
                      "model_bytes_over_time_gbs": plan.model_bytes(w.batch) / (ov_ms * 1e-3) / 1e9,
                      "note": "applies in flight on several streams share T in the L2 / Infinity Cache: "
                              "throughput of a stream of batches, not an HBM bandwidth measurement"}
        del ys

    # ---- a plain copy that moves the same number of bytes (half read, half written): the
    # streaming ceiling of this machine, and the kernel of known size that calibrates the
    # FETCH_SIZE / WRITE_SIZE counters in the rocprofv3 runs (torch.mul by 1.0 into `out`
    # is one elementwise kernel that reads src once and writes dst once)
    model_bytes = plan.model_bytes(w.batch)
    src = torch.empty(model_bytes // 8, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for _ in range(20):
        torch.mul(src, 1.0, out=dst)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 2 * src.numel() * 4 * 20 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    copy_bytes_each_way = src.numel() * 4
    del src, dst

    launch = launch_shape(cs, w.shape, w.batch, storage=2 if args.compact else (1 if args.transposed else 0))
    gbs = model_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = model_bytes / (region_avg * 1e-3) / 1e9
    out = {
        "metric": ("structure-aware storage of T: effective GB/s (descriptor-format model bytes / time per apply)"
                   if args.compact else
                   "SpMM effective HBM GB/s at 1024^2, k=7, batch 16 (model bytes / time per apply)"
                   if w.name == workloads.HEADLINE else "SpMV/SpMM effective GB/s (model bytes / time per apply)"),
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "m": m, "n": n, "k": k, "s": s, "p": p, "batch": w.batch,
                   "nnz": plan.nnz, "rows": plan.rows, "cols": plan.cols,
                   "apply_variant": plan.variant(w.batch), "streams": 1,
                   "matrix": "T (row descriptors + k*k table)" if args.compact
                   else ("T^T (CSC of T)" if args.transposed else "T (CSR)")},
        "timing": "one stream; %d launches until the device had settled (median of 50 within 1 %% of the 50 before, "
                  "at most 0.5 s), %d warm-up, %d timed between two synchronisations" % (pre_launches, args.warmup, args.steps),
        "precondition_launches": pre_launches, "precondition_last_median_ms": pre_median,
        "pct_of_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
        "useful_mac_per_s": plan.nnz * w.batch / (ms_per_step * 1e-3),
        "model_bytes": model_bytes,
        "error_criterion": "per output |y - ref| <= 1e-5 * sum_e |vals[e]| |x[col_idx[e]]| (componentwise backward "
                           "error of the dot product) and max|y - ref| <= 1e-5 * max|ref|; the plain per-output "
                           "relative error is reported per configuration as rel_err_vs_ref",
        "build_ms": build_med,
        "build_over_apply": build_med / ms_per_step,
        "copy_gbs_same_bytes": copy_gbs,
        "value_over_copy": gbs / copy_gbs,
        "copy_bytes_each_way": copy_bytes_each_way,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(plan.variant(w.batch), launch),
                     "kernel": plan.variant(w.batch), "launch": launch, "kernel_ms_avg": region_avg,
                     "timing": "two HIP events on the launch stream around the %d timed launches, elapsed / %d"
                               % (args.steps, args.steps),
                     "single_launch_ms_avg": kern_avg, "single_launch_ms_median": kern_ms[len(kern_ms) // 2],
                     "single_launch_ms_min": kern_ms[0],
                     "frac_from_single_launch_median": model_bytes / (kern_ms[len(kern_ms) // 2] * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if overlapped is not None:
        out["applies_in_flight_on_several_streams"] = overlapped
    if args.compact:
        # 8 bytes per row instead of 8 per entry: the multiply-adds, not the bytes, bound this kernel
        tflops = 2.0 * plan.nnz * w.batch / (region_avg * 1e-3) / 1e12
        out["roofline"].update({"bound": "alu", "achieved": tflops, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tflops / FP32_VECTOR_PEAK_TFLOPS,
                                "frac_of_unpacked_fp32_peak": tflops / FP32_UNPACKED_PEAK_TFLOPS,
                                "hbm_frac": achieved / HBM_PEAK_GBS})
    if not (args.compact or args.transposed) and not args.no_side_paths:
        # the widened paths on the same workload, briefly (outside the timed region above): HIP-event
        # average of single launches after a warm-up; their own runs are --compact and --transposed
        side = {}
        for tag, build in (("compact_storage", cs.conv_compact_build), ("transposed_csc", cs.conv_csc_build)):
            pl = build(m, n, k, s, p, K)
            xin = x if tag == "compact_storage" else torch.empty(pl.cols * w.batch, dtype=torch.float32,
                                                                  device=dev).normal_()
            yo = torch.empty(pl.rows * w.batch, dtype=torch.float32, device=dev)
            for _ in range(100):
                cs.conv_spmv(pl, xin, yo, batch=w.batch)
            torch.cuda.synchronize()
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
            for a, b in pairs:
                a.record(stream)
                cs.conv_spmv(pl, xin, yo, batch=w.batch)
                b.record(stream)
            torch.cuda.synchronize()
            avg = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)
            side[tag] = {"kernel": pl.variant(w.batch), "kernel_ms_avg": avg, "model_bytes": pl.model_bytes(w.batch),
                         "model_gbs": pl.model_bytes(w.batch) / (avg * 1e-3) / 1e9,
                         "useful_tflops": 2.0 * pl.nnz * w.batch / (avg * 1e-3) / 1e12}
            if tag == "transposed_csc":
                # y = T x from the same column-compressed arrays (a scatter: zero fill + sums per tile)
                for _ in range(10):
                    cs.conv_spmv_from_csc(pl, x, y, batch=w.batch)
                torch.cuda.synchronize()
                for a, b in pairs:
                    a.record(stream)
                    cs.conv_spmv_from_csc(pl, x, y, batch=w.batch)
                    b.record(stream)
                torch.cuda.synchronize()
                avg = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)
                side["product_from_csc"] = {"ms_avg": avg, "useful_tflops": 2.0 * pl.nnz * w.batch / (avg * 1e-3) / 1e12}
            pl.close()
        # a layer-like sum over input channels (56 x 56, k = 3, 64 channels, this batch) from both storages
        cm, cn, ck, cs_, cp, cc = 56, 56, 3, 1, 1, 64
        Kc = torch.empty(cc * ck * ck, dtype=torch.float32, device=dev).normal_()
        xc = torch.empty(cc * cm * cn * w.batch, dtype=torch.float32, device=dev).normal_()
        # ... and a sum over 3 channels at this workload's own shape (CSR: the marching kernel walks the
        # channels inside one launch when the shape takes it)
        K3 = torch.empty(3 * k * k, dtype=torch.float32, device=dev).normal_()
        x3 = torch.empty(3 * m * n * w.batch, dtype=torch.float32, device=dev).normal_()
        for tag, pl, (cm, cn, ck, cs_, cp, cc), xc in (
                ("channel_sum_csr", cs.conv_csr_build_channels(cm, cn, ck, cs_, cp, Kc, cc), (cm, cn, ck, cs_, cp, cc), xc),
                ("channel_sum_compact", cs.conv_compact_build(cm, cn, ck, cs_, cp, Kc, channels=cc), (cm, cn, ck, cs_, cp, cc), xc),
                ("channel_sum_csr_3_at_shape", cs.conv_csr_build_channels(m, n, k, s, p, K3, 3), (m, n, k, s, p, 3), x3),
                ("channel_sum_compact_3_at_shape", cs.conv_compact_build(m, n, k, s, p, K3, channels=3), (m, n, k, s, p, 3), x3)):
            yc = torch.empty(pl.rows * w.batch, dtype=torch.float32, device=dev)
            for _ in range(20):
                cs.conv_spmv(pl, xc, yc, batch=w.batch)
            torch.cuda.synchronize()
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
            for a, b in pairs:
                a.record(stream)
                cs.conv_spmv(pl, xc, yc, batch=w.batch)
                b.record(stream)
            torch.cuda.synchronize()
            avg = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)
            side[tag] = {"shape": [cm, cn, ck, cs_, cp], "channels": cc, "kernel": pl.variant(w.batch), "ms_avg": avg,
                         "useful_tflops": 2.0 * pl.nnz * cc * w.batch / (avg * 1e-3) / 1e12}
            pl.close()
        out["side_paths"] = side
    plan.close()
    del plan, y
    if not (args.compact or args.transposed or args.no_configs) and w.name == workloads.HEADLINE:
        # every named configuration, single stream, each against the oracle
        import oracle
        oracle.build()
        names = {"1": "small_32_k3", "2": "strided_256_k5_b64", "3a": "headline_1024_k7_b1",
                 "3b": "headline_1024_k7_b16", "4": "cnn_224_k3_b256", "5a": "padheavy_512_k9_s3",
                 "5b": "padheavy_4096_k11_s4_b4"}
        out["configs"] = {tag: dict(config_entry(cs, oracle, workloads, nm, dev, stream), workload=nm)
                          for tag, nm in names.items()}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, x_h, K_h, args.transposed)
        out["gpu_over_cpu"] = out["useful_mac_per_s"] / 1e9 / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
