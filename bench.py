#!/usr/bin/env python3
"""Benchmark of the fused Harris coarsity kernel on one MI355X.

A step is one pass of the whole pipeline (grayscale, Sobel pair, products, 3x3 sums,
coarsity: one kernel launch) over one synthetic 3x1536x2560 float32 image that is
already resident in device memory.  Successive steps use different input/result
buffers, rotating over more than 1 GiB, so that no step finds its image in the
256 MB last-level cache left there by an earlier step.

Prints one JSON line: throughput in Mpixels/s (input pixels), the roofline object
for the kernel (algorithmic bytes / launch duration against 8 TB/s of HBM) and the
CPU oracle timed on this host as a baseline.

Clocks.  After an idle period the GPU's clocks need about 10 ms of work to settle (the
first several hundred launches of this size run some 5 % slower than the rest).  Whatever
--warmup says, the timed region therefore starts only after at least SETTLE_MS of untimed
back-to-back launches (their number is reported as config.settle_launches), so that a run
of 20 timed steps measures the same steady state as one of 3000.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # published MI355X HBM3E bandwidth
SETTLE_MS = 20.0               # untimed launches before the timed region, in GPU time

# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (summaries under profiles/), valid only
# for the kernel sources they were taken with: (sha256 of the csrc files without comments, {workload: bytes}).
TRAFFIC_SOURCES_SHA256 = "afb62ddae48fa5f0140fe70a49733a13eb522ec8c8da10fe2dfd692c10a8c2e7"
TRAFFIC_BYTES = {"noise_f32_1536x2560": 65109553, "rects_f32_64x1080x1920": 2138767251,
                 "blobs_f32_2832x4256": 196600535, "noise_u8_8192x8192": 474898329}


def kernel_sources_sha256():
    """Hash of the kernel sources without comments and blank lines: what the compiler sees."""
    import hashlib
    import re
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2212_12035_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        text = "\n".join(line.rstrip() for line in text.splitlines() if line.strip())
        h.update(name.encode() + b"\0" + text.encode())
    return h.hexdigest()
WORKLOAD = "noise_f32_1536x2560"
K_COARSITY = 0.04


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: ~40 ms of back-to-back launches in the timed region.  The clocks are settled by
    # time (SETTLE_MS), not by the warm-up count.
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default=WORKLOAD, help="one of harris_inputs.WORKLOADS (default: the headline one)")
    ap.add_argument("--rotate-bytes", type=float, default=float(1 << 30), help="distinct buffer bytes to rotate over")
    ap.add_argument("--schedule", type=int, default=0, help="0 auto, 1 bands, 2 tiles")
    ap.add_argument("--px", type=int, default=0)
    ap.add_argument("--rows", type=int, default=0)
    ap.add_argument("--prefetch", type=int, default=0)
    ap.add_argument("--waves-per-block", type=int, default=0)
    ap.add_argument("--lds-kb", type=int, default=0)
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-groupings", action="store_true", help="skip timing the unfused kernel groupings")
    ap.add_argument("--probes", action="store_true", help="also time pure read and pure write streams of the launch's bytes")
    ap.add_argument("--warm-cache", action="store_true", help="reuse one buffer pair (cache-resident; not the roofline number)")
    ap.add_argument("--out-dtype", choices=("f32", "f16", "bf16", "u8"), default="f32",
                    help="type the result is stored in (the arithmetic stays float32; u8: codes rint(v + 128) clamped); "
                         "not the headline configuration")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (--gpus must be 1)")

    import numpy as np
    import torch
    import harris_inputs
    import paper_2212_12035_amd as pkg

    if not os.path.exists(pkg.library_path()):
        from paper_2212_12035_amd import build as product_build
        product_build.build_library()
    lib = pkg.load_library()

    gen, seed, B, H, W, dt = harris_inputs.WORKLOADS[args.workload]
    is_u8 = dt == "u8"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    host = harris_inputs.make(args.workload)
    n, m = H - 4, W - 4
    in_bytes = B * 3 * H * W * (1 if is_u8 else 4)
    out_torch = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "u8": torch.uint8}[args.out_dtype]
    out_code = {"f32": pkg.HARRIS_OUT_F32, "f16": pkg.HARRIS_OUT_F16, "bf16": pkg.HARRIS_OUT_BF16, "u8": pkg.HARRIS_OUT_U8}[args.out_dtype]
    out_bytes = B * n * m * {"f32": 4, "f16": 2, "bf16": 2, "u8": 1}[args.out_dtype]
    Q_SCALE, Q_OFFSET = 1.0, 128.0
    algo_bytes = in_bytes + out_bytes                      # each input element read once, each result written once
    pixels = B * H * W

    # Rotating buffer pairs.  Pair 0 holds the seeded image; pair i holds the same image
    # rolled down by i rows (same statistics, different addresses).
    n_pairs = 1 if args.warm_cache else max(2, int(-(-args.rotate_bytes // algo_bytes)))
    free_b, _ = torch.cuda.mem_get_info(dev)
    n_pairs = max(1, min(n_pairs, int(0.8 * free_b // algo_bytes)))
    base = torch.from_numpy(host).to(dev)
    ins = [base] + [torch.roll(base, shifts=i, dims=2) for i in range(1, n_pairs)]
    outs = [torch.empty((B, n, m), dtype=out_torch, device=dev) for _ in range(n_pairs)]

    explicit_tuning = any((args.schedule, args.px, args.rows, args.prefetch, args.waves_per_block, args.flags, args.lds_kb))
    tuning = pkg.HarrisTuning(args.schedule, args.px, args.rows, args.prefetch, args.waves_per_block, args.flags, args.lds_kb)
    shape, n_blocks = pkg.harris_plan_typed(pkg.HARRIS_U8 if is_u8 else pkg.HARRIS_F32, out_code, B, H, W, tuning=tuning)
    stream = torch.cuda.current_stream(dev)
    sptr = ctypes.c_void_p(stream.cuda_stream)
    dtype_code = pkg.HARRIS_U8 if is_u8 else pkg.HARRIS_F32
    calls = [(ctypes.c_void_p(i.data_ptr()), ctypes.c_void_p(o.data_ptr())) for i, o in zip(ins, outs)]
    tref = ctypes.byref(tuning)
    fn = lib.harris_coarsity_typed

    def step(i):
        a, o = calls[i % n_pairs]
        if args.out_dtype == "u8":
            rc = lib.harris_coarsity_quantized(a, dtype_code, B, H, W, None, K_COARSITY, 1.0, 0, Q_SCALE, Q_OFFSET, o, tref, sptr)
        else:
            rc = fn(a, dtype_code, B, H, W, None, K_COARSITY, 1.0, 0, o, out_code, tref, sptr)
        if rc != 0:
            raise RuntimeError(pkg.harris_strerror(rc))

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize(dev)

    # Settle the clocks by time: a short probe gives the launch duration, then as many untimed
    # back-to-back launches as fill SETTLE_MS, in one go (no gaps in which the clocks could fall
    # again), and the timed region follows the synchronisation at once.
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s0.record(stream)
    for i in range(40):
        step(i)
    s1.record(stream)
    torch.cuda.synchronize(dev)
    settle_launches = 40 + max(0, int(SETTLE_MS / max(s0.elapsed_time(s1) / 40, 1e-4)) + 1)
    for i in range(settle_launches - 40):
        step(i)

    # Timed region: exactly `steps` launches, wall clock between synchronisations, and a
    # pair of HIP events on the launch stream for the GPU-side duration.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize(dev)
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall_ms / args.steps
    launch_us = gpu_ms * 1e3 / args.steps                 # average per launch over the timed region

    # The kernel's own duration, for the roofline: an event pair around further launches issued
    # right behind a few untimed ones, with no synchronisation in between.  The pair of the timed
    # region above starts on an idle queue, so it also contains the host's latency until the first
    # launch arrives (some 5 to 10 us, which is 4 % of 20 steps and nothing of 3000); here the
    # queue is busy when the first event is reached, and what the pair brackets is kernels back to
    # back: the figure that rocprofv3's kernel trace gives for the same launches.
    KERNEL_LEAD_IN = 12
    n_kernel = max(args.steps, 200)
    k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(KERNEL_LEAD_IN):
        step(i)
    k0.record(stream)
    for i in range(n_kernel):
        step(KERNEL_LEAD_IN + i)
    k1.record(stream)
    torch.cuda.synchronize(dev)
    kernel_us = k0.elapsed_time(k1) * 1e3 / n_kernel

    # Single-launch durations (event pair around each launch), for information.
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 60))]
    for i, (a, b) in enumerate(pairs):
        a.record(stream); step(i); b.record(stream)
    torch.cuda.synchronize(dev)
    singles = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
    single_med_us = singles[len(singles) // 2]

    # The thesis's kernel groupings (unfused baselines) on the same rotating buffers, for comparison.
    groupings = None
    if not args.no_groupings and args.out_dtype == "f32":
        groupings = {}
        ws_bytes = pkg.harris_grouped_workspace_bytes(1, B, H, W)
        ws = torch.empty(max(1, ws_bytes // 4), dtype=torch.float32, device=dev)
        reps = max(10, min(100, args.steps // 8))
        for g in (1, 2, 3):
            def gstep(i, g=g):
                a, o = calls[i % n_pairs]
                rc = lib.harris_coarsity_grouped(a, dtype_code, B, H, W, K_COARSITY, 1.0, 0, g, ctypes.c_void_p(ws.data_ptr()),
                                                 ws_bytes, o, sptr)
                if rc != 0:
                    raise RuntimeError(pkg.harris_strerror(rc))
            for i in range(3):
                gstep(i)
            torch.cuda.synchronize(dev)
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record(stream)
            for i in range(reps):
                gstep(i)
            g1.record(stream)
            torch.cuda.synchronize(dev)
            groupings["grouping_%d_us" % g] = round(g0.elapsed_time(g1) * 1e3 / reps, 2)
        groupings["grouping_4_fused_us"] = round(kernel_us, 2)
        del ws
        step(0)                                   # pair 0 holds the fused kernel's result again
        torch.cuda.synchronize(dev)

    # What a kernel that only moves these bytes reaches on this GPU: the library's streaming-copy
    # probe (three planes in, one float per result pixel out) on the same rotating buffers.
    probe = None
    if args.out_dtype == "f32":
        probe_bytes = B * n * m * (3 * (1 if is_u8 else 4) + 4)
        reps = max(20, min(400, args.steps // 4))
        def pstep(i):
            a, o = calls[i % n_pairs]
            rc = lib.harris_probe_copy(a, dtype_code, B, H, W, o, sptr)
            if rc != 0:
                raise RuntimeError(pkg.harris_strerror(rc))
        for i in range(max(12, reps // 4)):     # untimed, and no synchronisation before the pair: a busy queue, as for the Harris figure
            pstep(i)
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record(stream)
        for i in range(reps):
            pstep(i)
        p1.record(stream)
        torch.cuda.synchronize(dev)
        probe_us = p0.elapsed_time(p1) * 1e3 / reps
        probe = {"us": round(probe_us, 3), "bytes": probe_bytes, "GB/s": round(probe_bytes / (probe_us * 1e-6) / 1e9, 1),
                 "what": "harris_probe_copy: reads 3 planes, writes 1 float per result pixel, nothing else"}
        step(0)                                   # pair 0 holds the fused kernel's result again
        torch.cuda.synchronize(dev)

    # Pure streams of the launch's algorithmic bytes, reads alone and writes alone, on rotating
    # buffers of their own: with the copy probe they bound what this many bytes, cold, can reach.
    streams = None
    if args.probes:
        sbytes = algo_bytes - algo_bytes % 16
        bufs = [torch.randint(0, 256, (sbytes,), dtype=torch.uint8, device=dev) for _ in range(n_pairs)]
        sink = torch.zeros(64, dtype=torch.uint8, device=dev)
        streams = {"bytes": sbytes}
        reps = max(20, min(400, args.steps // 4))
        for kind, name in ((pkg.HARRIS_PROBE_READ, "read"), (pkg.HARRIS_PROBE_WRITE, "write")):
            def sstep(i, kind=kind):
                b = bufs[i % n_pairs]
                rc = lib.harris_probe_stream(kind, ctypes.c_void_p(b.data_ptr()), ctypes.c_void_p(sink.data_ptr() if kind == pkg.HARRIS_PROBE_READ else b.data_ptr()), sbytes, sptr)
                if rc != 0:
                    raise RuntimeError(pkg.harris_strerror(rc))
            for i in range(max(12, reps // 4)):
                sstep(i)
            q0, q1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            q0.record(stream)
            for i in range(reps):
                sstep(i)
            q1.record(stream)
            torch.cuda.synchronize(dev)
            us = q0.elapsed_time(q1) * 1e3 / reps
            streams[name + "_us"] = round(us, 3)
            streams[name + "_GB/s"] = round(sbytes / (us * 1e-6) / 1e9, 1)
        del bufs
        # What a kernel launch costs the GPU by itself: launches that touch no memory, replayed from
        # a captured graph so that the host's launch rate does not bound their period.
        def idle():
            rc = lib.harris_probe_stream(pkg.HARRIS_PROBE_NONE, None, None, 0, ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream))
            if rc != 0:
                raise RuntimeError(pkg.harris_strerror(rc))
        side = torch.cuda.Stream(dev)
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            idle()                                # the kernel is loaded before the capture
        side.synchronize()
        graph, nodes, replays = torch.cuda.CUDAGraph(), 500, 8
        with torch.cuda.graph(graph, stream=side):
            for _ in range(nodes):
                idle()
        graph.replay()
        torch.cuda.synchronize(dev)
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record(stream)
        for _ in range(replays):
            graph.replay()
        g1.record(stream)
        torch.cuda.synchronize(dev)
        streams["idle_launch_us"] = round(g0.elapsed_time(g1) * 1e3 / (nodes * replays), 3)
        streams["idle_launch_what"] = "harris_probe_stream(HARRIS_PROBE_NONE): a launch that touches no memory, %d of them in a graph, %d replays" % (nodes, replays)

    # Correctness of what was timed: pair 0 against the oracle (also the CPU baseline).
    got = outs[0].float().cpu().numpy()
    cpu = None
    max_err = bound = rounding = None
    if not args.no_cpu_baseline:
        from oracle import harris_oracle
        nt = harris_oracle.hardware_threads()
        sample = host if B == 1 else host[:1]
        spx = sample.shape[0] * H * W
        harris_oracle.harris(sample, K_COARSITY, nthreads=nt)            # page in
        reps_all, reps_one = 25, 5
        ta = []
        for _ in range(reps_all):
            s = time.perf_counter(); want = harris_oracle.harris(sample, K_COARSITY, nthreads=nt); ta.append(time.perf_counter() - s)
        to = []
        for _ in range(reps_one):
            s = time.perf_counter(); harris_oracle.harris(sample, K_COARSITY, nthreads=1); to.append(time.perf_counter() - s)
        ta.sort(); to.sort()
        bound = 1e-4 * float(np.abs(want).max()) + 1e-6
        if args.out_dtype == "u8":                 # codes against the oracle's codes: the bar in codes, plus one
            want = harris_oracle.quantize_u8(want, Q_SCALE, Q_OFFSET).astype(np.float32)
            bound = float(np.ceil(bound * abs(Q_SCALE))) + 1.0
        elif args.out_dtype != "f32":              # plus one spacing of the 16-bit format at the largest value
            bound += float(np.abs(want).max()) * (2.0 ** -10 if args.out_dtype == "f16" else 2.0 ** -7)
        max_err = float(np.abs(got[:sample.shape[0]] - want).max())
        if args.out_dtype == "f32":
            # Beside the bar, a diagnostic at rounding level: the distance to the float64 referee in
            # units of float32 eps times the largest trace^2 (every term of the coarsity is bounded
            # by trace^2; a correct float32 implementation stays within a few units).
            ref64 = harris_oracle.harris(sample, K_COARSITY, precision="f64", nthreads=nt)
            unit = float(np.finfo(np.float32).eps) * harris_oracle.max_trace_squared(sample)
            rounding = {"gpu_vs_f64_in_eps_trace2": round(float(np.abs(got[:sample.shape[0]] - ref64).max()) / unit, 3),
                        "oracle_f32_vs_f64_in_eps_trace2": round(float(np.abs(want - ref64).max()) / unit, 3), "limit": 64.0}
        cpu = {"value": round(spx / ta[len(ta) // 2] / 1e6, 2), "unit": "Mpixels/s", "cores": nt, "kind": "oracle",
               "sample": "%d image(s) of %s: median of %d runs on %d threads (and of %d runs on one thread), about %.0f s of CPU work" % (sample.shape[0], args.workload, reps_all, nt, reps_one, sum(ta) * nt + sum(to)),
               "value_1_thread": round(spx / to[len(to) // 2] / 1e6, 2)}

    achieved = algo_bytes / (kernel_us * 1e-6) / 1e9
    achieved_wall = algo_bytes / (ms_per_step * 1e-3) / 1e9
    achieved_region = algo_bytes / (launch_us * 1e-6) / 1e9
    result = {
        "metric": "harris_mpixels_per_s",
        "value": round(pixels / (ms_per_step * 1e-3) / 1e6, 1),
        "unit": "Mpixels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8" if is_u8 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "H": H, "W": W, "input": dt, "arithmetic": "f32", "k": K_COARSITY,
                   "result": args.out_dtype, "buffer_pairs": n_pairs, "cache": "warm" if args.warm_cache else "cold (rotating buffers)",
                   "settle_launches": settle_launches, "settle_ms": SETTLE_MS,
                   "launch": shape, "workgroups": n_blocks},
        # achieved/frac: algorithmic bytes over the kernel's average duration (event pair around
        # kernel_launches back-to-back launches on a busy queue).  The same bytes over the two clocks
        # of the timed region of `steps` launches are given beside it: its own event pair (which
        # starts on an idle queue) and the wall clock between the synchronisations (`value`'s clock).
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "clock": "HIP event pair on the launch stream around kernel_launches launches behind %d untimed ones, no synchronisation in between" % KERNEL_LEAD_IN,
                     "kernel_launches": n_kernel, "kernel_us_avg": round(kernel_us, 3),
                     "achieved_timed_region_events": round(achieved_region, 1), "frac_timed_region_events": round(achieved_region / HBM_PEAK_GBS, 4),
                     "achieved_wall": round(achieved_wall, 1), "frac_wall": round(achieved_wall / HBM_PEAK_GBS, 4),
                     "traffic": TRAFFIC_BYTES.get(args.workload) if kernel_sources_sha256() == TRAFFIC_SOURCES_SHA256 and not explicit_tuning and args.out_dtype == "f32" else None,
                     "algorithmic_bytes_per_launch": algo_bytes,
                     "launch_us_avg_over_timed_region": round(launch_us, 3),
                     "launch_us_single_median": round(single_med_us, 3),
                     "frac_of_copy_probe": round(achieved / probe["GB/s"], 4) if probe else None},
        "copy_probe": probe,
        "stream_probes": streams,
        "cpu_baseline": cpu,
        "kernel_groupings": groupings,
        "max_abs_err_vs_oracle": max_err, "err_bound": bound, "rounding": rounding,
    }
    print(json.dumps(result))
    if max_err is not None and not max_err <= bound:
        sys.exit("bench: GPU result differs from the oracle by %g (bound %g)" % (max_err, bound))
    if rounding is not None and not rounding["gpu_vs_f64_in_eps_trace2"] <= rounding["limit"]:
        sys.exit("bench: GPU result is %g eps*trace^2 from the float64 referee (limit %g)" % (rounding["gpu_vs_f64_in_eps_trace2"], rounding["limit"]))


if __name__ == "__main__":
    main()
