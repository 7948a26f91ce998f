"""Launch-shape sweep: the planner's choice against every candidate shape, size by size.

    python -m paper_2212_12035_amd.sweep [--dtype f32|u8] [--sizes BxHxW,BxHxW,...] [--rounds N] [--steps K]

For each problem size the library's default launch shape (harris_plan) is timed against the
candidate tile shapes it could have taken instead -- one tile per CU in every wavefront/row
split that covers the image, with the barrier and with ready flags, and many small tiles with
their LDS reservations -- on buffers that rotate over more than 1 GiB, in interleaved rounds.
One line per size: the default's shape and time, the fastest candidate and its time, and how
much faster that is.  This is the measurement the planner's thresholds come from; run it again
to re-tune them for another GPU.  It needs the built library and a ROCm device, nothing else.
"""
from __future__ import annotations

import argparse
import ctypes
import statistics
import sys

F32_SIZES = "1x480x640,4x480x640,1x600x800,1x720x1280,2x720x1280,1x768x1024,1x900x1600,1x960x1280,1x1000x1000,1x1024x1024," \
            "1x1024x1280,1x1050x1400,1x1080x1920,2x1080x1920,3x1080x1920,1x1200x1600,1x1440x2560,1x1536x2560,1x2048x2048,1x2160x3840,2x1536x2560"
U8_SIZES = "1x768x1024,1x960x1280,1x1024x1024,1x1080x1920,2x1080x1920,1x1200x1600,1x1440x2560,1x1536x2560,1x2048x2048,1x2160x3840," \
           "2x1536x2560,1x2048x4096,4x1080x1920,1x3000x4000,1x4096x4096,1x4320x7680"


def candidates(pkg, dtype, B, H, W):
    """(name, HarrisTuning) pairs: the default first."""
    T = pkg.HarrisTuning
    n, m = H - 4, W - 4
    out = [("default", T())]
    keep = pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS
    for rows, waves, lds in ((4, 4, 0), (4, 4, 36), (5, 4, 36), (5, 4, 48), (5, 5, 48), (5, 5, 64), (6, 5, 64), (6, 4, 48), (6, 4, 64), (8, 4, 64)):
        out.append(("many %dx%d lds%d" % (waves, rows, lds), T(pkg.HARRIS_SCHEDULE_TILES, 4, rows, 0, waves, keep, lds)))
    n_strips = -(-m // 240)
    if B * n_strips <= 256:
        need = -(-n // (256 // (B * n_strips))) + 4              # input rows of one tile per CU
        for rows in (4, 5, 6, 8, 9, 10):
            waves = max(2, -(-need // rows))
            if waves <= 16:
                out.append(("one/CU %dx%d barrier" % (waves, rows), T(pkg.HARRIS_SCHEDULE_TILES, 4, rows, 0, waves, pkg.HARRIS_TUNE_STREAM_LOADS, 0)))
                if dtype == pkg.HARRIS_F32:
                    out.append(("one/CU %dx%d flags" % (waves, rows), T(pkg.HARRIS_SCHEDULE_TILES, 4, rows, 0, waves, pkg.HARRIS_TUNE_FLAG_HANDOFF, 0)))
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--dtype", choices=("f32", "u8"), default="f32")
    ap.add_argument("--sizes", default=None, help="comma-separated BxHxW (default: a built-in list)")
    ap.add_argument("--rounds", type=int, default=5)
    ap.add_argument("--steps", type=int, default=120)
    ap.add_argument("--all", action="store_true", help="also print every candidate's time, fastest first")
    args = ap.parse_args()

    import torch
    import paper_2212_12035_amd as pkg
    lib = pkg.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream(dev)
    sptr = ctypes.c_void_p(stream.cuda_stream)
    dtype = pkg.HARRIS_U8 if args.dtype == "u8" else pkg.HARRIS_F32
    elem = 1 if args.dtype == "u8" else 4
    sizes = [tuple(int(v) for v in s.split("x")) for s in (args.sizes or (U8_SIZES if args.dtype == "u8" else F32_SIZES)).split(",")]
    worst = 1.0
    print("# %s input; times in us per launch, median of %d interleaved rounds of %d launches, rotating buffers" % (args.dtype, args.rounds, args.steps))
    print("# %-14s %-34s %8s   %-24s %8s  %s" % ("size", "default shape", "default", "fastest candidate", "fastest", "default/fastest"))
    for B, H, W in sizes:
        n, m = H - 4, W - 4
        algo = B * (3 * H * W * elem + 4 * n * m)
        pairs = max(2, min(64, -(-(1 << 30) // algo)))
        if args.dtype == "u8":
            ins = [torch.randint(0, 256, (B, 3, H, W), dtype=torch.uint8, device=dev) for _ in range(pairs)]
        else:
            ins = [torch.rand((B, 3, H, W), device=dev) for _ in range(pairs)]
        outs = [torch.empty((B, n, m), device=dev) for _ in range(pairs)]
        turn = [0]

        def burst(tuning, k):
            ref = ctypes.byref(tuning)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(k):
                i = turn[0] % pairs
                turn[0] += 1
                rc = lib.harris_coarsity_ex(ins[i].data_ptr(), dtype, B, H, W, 0.04, 1.0, 0, outs[i].data_ptr(), ref, sptr)
                if rc != 0:
                    raise RuntimeError(pkg.harris_strerror(rc))
            e1.record(stream)
            torch.cuda.synchronize(dev)
            return e0.elapsed_time(e1) * 1e3 / k

        cands = []
        for name, t in candidates(pkg, dtype, B, H, W):
            try:
                pkg.harris_plan(dtype, B, H, W, tuning=t)
                cands.append((name, t))
            except pkg.HarrisError:
                pass                                             # a shape the library has no kernel for
        for _ in range(3):                                       # settle the clocks
            burst(cands[0][1], max(200, int(4e9 // algo)))
        times = {name: [] for name, _ in cands}
        for r in range(args.rounds):
            for name, t in (cands if r % 2 == 0 else cands[::-1]):
                times[name].append(burst(t, args.steps))
        med = {name: statistics.median(v) for name, v in times.items()}
        best = min(med, key=med.get)
        shape = pkg.harris_plan(dtype, B, H, W)[0]
        desc = "%dx%d flags=%d lds=%d" % (shape["waves_per_block"], shape["rows"], shape["flags"], shape["lds_kb"])
        ratio = med["default"] / med[best]
        worst = max(worst, ratio)
        print("%-16s %-34s %8.2f   %-24s %8.2f  %.3f" % ("%dx%dx%d" % (B, H, W), desc, med["default"], best, med[best], ratio), flush=True)
        if args.all:
            print("#    " + "  ".join("%s %.2f" % kv for kv in sorted(med.items(), key=lambda kv: kv[1])), flush=True)
        del ins, outs
    print("# largest default/fastest: %.3f" % worst)
    return 0


if __name__ == "__main__":
    sys.exit(main())
