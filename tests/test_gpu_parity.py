"""GPU parity: libharris (through its C interface) against the CPU oracle, element by
element on the same seeded inputs.

Bar (float32): max|gpu - oracle| <= 1e-4 * max|oracle| + 1e-6, over the whole result
and, for batches, per image.  Both sides compute in float32; they differ in summation
order, in the separated form of the 3x3 kernels and in fused multiply-adds.
"""
import os
import sys

import numpy as np
import pytest

import harris_inputs as hi

pytestmark = pytest.mark.gpu

K = 0.04
S12 = float(np.float32(1.0) / np.float32(12.0))


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need a GPU"
    import paper_2212_12035_amd as pkg
    if not os.path.exists(pkg.library_path()):
        from paper_2212_12035_amd import build
        build.build_library()
    pkg.load_library()                      # fails loudly if the HIP library is missing
    return pkg


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_gpu(pkg, rgb, **kw):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(rgb)).cuda()
    out = pkg.harris_coarsity_ex(t, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


ROUNDING_LIMIT = 64.0       # in units of float32 eps * max trace^2; a correct kernel measures 0.3 to 2


def rounding_distance(oracle, got, rgb, k=K, scale=1.0, window=0, nthreads=4):
    """max|gpu - float64 referee| in units of float32 eps times the largest trace^2.

    The parity bar is far above float32 rounding (observed errors are a few thousandths of
    it), so a wrong rounding path or a small lost term could hide below it.  Every term of the
    coarsity is bounded by trace^2: a correct float32 evaluation, in any order and with or
    without fused multiply-adds, stays within a few eps * trace^2 of the exact result."""
    ref = oracle.harris(rgb, k, scale, window, precision="f64", nthreads=nthreads)
    unit = float(np.finfo(np.float32).eps) * oracle.max_trace_squared(rgb, scale, window)
    if ref.size == 0 or unit == 0.0:
        return 0.0
    return float(np.abs(got.astype(np.float64) - ref).max()) / unit


def check(got, want, per_image=True, referee=None):
    """The bar; with referee=(oracle, rgb, k, scale, window) also the rounding-level diagnostic."""
    assert got.shape == want.shape and got.dtype == np.float32
    assert np.all(np.isfinite(got))
    if want.size == 0:
        return 0.0
    bound = 1e-4 * float(np.abs(want).max()) + 1e-6
    err = float(np.abs(got - want).max())
    assert err <= bound, "max|gpu-oracle| = %g > %g" % (err, bound)
    if referee is not None:
        dist = rounding_distance(referee[0], got, *referee[1:])
        say("   distance to the float64 referee: %.3g eps*trace^2" % dist)
        assert dist <= ROUNDING_LIMIT, "max|gpu-f64| = %g eps*trace^2 > %g" % (dist, ROUNDING_LIMIT)
    if per_image and want.ndim == 3 and want.shape[0] > 1:
        for b in range(want.shape[0]):
            bb = 1e-4 * float(np.abs(want[b]).max()) + 1e-6
            eb = float(np.abs(got[b] - want[b]).max())
            assert eb <= bb, "image %d: max|gpu-oracle| = %g > %g" % (b, eb, bb)
    return err / bound


# ---------------------------------------------------------------- the C entry points as they are

def test_tiny_config_default_entry(gpu, oracle):
    import torch
    rgb = hi.make("tiny_f32_64x96")
    say("case tiny_f32_64x96 harris_coarsity")
    out = gpu.harris_coarsity(torch.from_numpy(rgb).cuda(), K)
    torch.cuda.synchronize()
    check(out.cpu().numpy(), oracle.harris(rgb, K))


def test_u8_default_entry(gpu, oracle):
    import torch
    rgb = hi.make("noise_u8_8192x8192", H=96, W=160)
    say("case u8 96x160 harris_coarsity_u8")
    out = gpu.harris_coarsity_u8(torch.from_numpy(rgb).cuda(), K)
    torch.cuda.synchronize()
    check(out.cpu().numpy(), oracle.harris(rgb, K))


def test_result_buffer_is_fully_overwritten_and_nothing_else(gpu, oracle):
    import torch
    rgb = hi.white_noise_f32(40, 2, 37, 264)
    B, _, H, W = rgb.shape
    n = B * (H - 4) * (W - 4)
    say("case guard bands around out, 2x3x37x264")
    big = torch.full((n + 512,), float("nan"), device="cuda")
    out = big[256:256 + n].view(B, H - 4, W - 4)
    gpu.harris_coarsity(torch.from_numpy(rgb).cuda(), K, out=out)
    torch.cuda.synchronize()
    host = big.cpu().numpy()
    assert np.all(np.isnan(host[:256])) and np.all(np.isnan(host[256 + n:]))
    check(host[256:256 + n].reshape(B, H - 4, W - 4), oracle.harris(rgb, K))


# ---------------------------------------------------------------- launch shapes: several tiles, ragged tails

SHAPES = [
    # (H, W): W picks the widest path; sizes span several strips/bands with ragged ends
    (23, 520), (41, 1028), (70, 256), (9, 260), (33, 98), (30, 131), (5, 5), (5, 1040), (64, 8), (12, 12),
]


@pytest.mark.parametrize("H,W", SHAPES)
def test_f32_shapes_default_plan(gpu, oracle, H, W):
    rgb = hi.white_noise_f32(100 + H + W, 2, H, W)
    say("case f32 2x3x%dx%d default plan %s" % (H, W, gpu.harris_plan(0, 2, H, W)))
    check(run_gpu(gpu, rgb, k=K), oracle.harris(rgb, K), referee=(oracle, rgb))


@pytest.mark.parametrize("px", [1, 2, 4])
@pytest.mark.parametrize("prefetch", [3])
def test_f32_every_kernel_instance(gpu, oracle, px, prefetch):
    H, W = 45, 8 * 67            # 536 columns: 2-3 strips at px 4/8, 5 at px 2, 9 at px 1
    rgb = hi.white_noise_f32(7, 2, H, W)
    want = oracle.harris(rgb, K)
    for rows, wpb, flags in ((7, 4, 0), (10, 1, 1 | 4), (64, 2, 2 | 8), (1, 4, 3)):
        tune = dict(schedule=1, px=px, rows=rows, prefetch=prefetch, waves_per_block=wpb, flags=flags)
        say("case f32 2x3x%dx%d %s" % (H, W, tune))
        check(run_gpu(gpu, rgb, k=K, tuning=tune), want)


@pytest.mark.parametrize("px,rows", [(1, 4), (2, 4), (4, 4), (4, 8)])
def test_tile_schedule_every_kernel_instance(gpu, oracle, px, rows):
    H, W = 75, 8 * 67
    for rgb in (hi.white_noise_f32(17, 2, H, W), hi.white_noise_u8(18, 2, H, W)):
        want = oracle.harris(rgb, K)
        for waves, flags in ((2, 0), (3, 2 | 4), (8, 8), (16, 0)):
            tune = dict(schedule=2, px=px, rows=rows, waves_per_block=waves, flags=flags)
            say("case tiles %s 2x3x%dx%d %s" % (rgb.dtype, H, W, tune))
            check(run_gpu(gpu, rgb, k=K, tuning=tune), want)


@pytest.mark.parametrize("rows", [5, 6, 9, 10])
def test_tile_schedule_other_heights(gpu, oracle, rows):
    H, W = 131, 4 * 130
    rgb = hi.white_noise_f32(19, 2, H, W)
    want = oracle.harris(rgb, K)
    for waves in (2, 7, 12):
        tune = dict(schedule=2, px=4, rows=rows, waves_per_block=waves)
        say("case tiles f32 2x3x%dx%d %s" % (H, W, tune))
        check(run_gpu(gpu, rgb, k=K, tuning=tune), want)
    u8 = hi.white_noise_u8(20, 1, 50, 256)
    check(run_gpu(gpu, u8, k=K, window=1, tuning=dict(schedule=2, px=4, rows=rows, waves_per_block=3)), oracle.harris(u8, K, 1.0, 1))


@pytest.mark.parametrize("rows", [4, 5, 6, 8, 9, 10])
def test_tile_schedule_shared_rows_kept_in_cache(gpu, oracle, rows):
    # Non-temporal loads except for the rows two tiles share: its own kernel instances (float32
    # and 8-bit, both windows), including tiles of two wavefronts, where the first and the last
    # wavefront are neighbours, and tile heights below 8, where the two groups of rows overlap.
    H, W = 97, 4 * 131
    flags = gpu.HARRIS_TUNE_STREAM_LOADS | gpu.HARRIS_TUNE_KEEP_SHARED_ROWS
    for rgb in (hi.white_noise_f32(23, 2, H, W), hi.white_noise_u8(24, 2, H, W)):
        for window in (0, 1):
            want = oracle.harris(rgb, K, 1.0, window)
            for waves in (2, 3, 5):
                tune = dict(schedule=2, px=4, rows=rows, waves_per_block=waves, flags=flags)
                say("case tiles keep-shared %s window=%d %s" % (rgb.dtype, window, tune))
                check(run_gpu(gpu, rgb, k=K, window=window, tuning=tune), want)


@pytest.mark.parametrize("rows", [4, 5, 6, 8, 9, 10])
def test_tile_schedule_ready_flags_instead_of_the_barrier(gpu, oracle, rows):
    # The hand-off by ready flags has kernel instances of its own (float32 input): both
    # windows, from 2 to 16 wavefronts per tile, several tiles down the image and a ragged last
    # one, every result type; plus a workgroup count far above what is resident at once.
    import torch
    flags = gpu.HARRIS_TUNE_FLAG_HANDOFF
    H, W = 151, 4 * 131
    with pytest.raises(gpu.HarrisError) as e:                      # no such kernels for 8-bit input
        run_gpu(gpu, hi.white_noise_u8(28, 2, H, W), k=K, tuning=dict(schedule=2, px=4, rows=rows, waves_per_block=3, flags=flags))
    assert e.value.status == -3
    for rgb in (hi.white_noise_f32(27, 2, H, W),):
        for window in (0, 1):
            want = oracle.harris(rgb, K, 1.0, window)
            for waves in (2, 3, 9, 16):
                tune = dict(schedule=2, px=4, rows=rows, waves_per_block=waves, flags=flags)
                say("case tiles ready flags %s window=%d %s" % (rgb.dtype, window, tune))
                check(run_gpu(gpu, rgb, k=K, window=window, tuning=tune), want)
    rgb = hi.rectangles_f32(29, 3, 90, 520)
    want = oracle.harris(rgb, K)
    src = torch.from_numpy(rgb).cuda()
    for tdt, fmt in ((torch.float16, "f16"), (torch.bfloat16, "bf16")):
        out = torch.empty((3, 86, 516), dtype=tdt, device="cuda")
        gpu.harris_coarsity_typed(src, out, K, tuning=dict(schedule=2, rows=rows, waves_per_block=4, flags=flags))
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
        assert np.all(np.abs(got.astype(np.float64) - _as_f32(oracle.round_to_16bit(want, fmt), fmt)) <= 1e-4 * float(np.abs(want).max()) + 1e-6 + _ulp16(want, fmt))
    big = hi.white_noise_f32(30, 1, 2200, 1000)                 # thousands of small tiles with flags
    check(run_gpu(gpu, big, k=K, tuning=dict(schedule=2, rows=rows, waves_per_block=2, flags=flags)), oracle.harris(big, K, nthreads=8))


def test_repeated_launches_give_identical_results(gpu):
    # The hand-over through LDS (barrier or ready flags) must not depend on timing: 300 launches of
    # the same image, alternating with launches on other data, bit-identical results.
    import torch
    rgb = torch.from_numpy(hi.make("noise_f32_1536x2560")).cuda()
    other = torch.rand_like(rgb)
    scratch = torch.empty((1, 1532, 2556), device="cuda")
    for tune in (None, dict(flags=gpu.HARRIS_TUNE_STREAM_LOADS), dict(schedule=2, rows=4, waves_per_block=4),
                 dict(schedule=2, rows=5, waves_per_block=16, flags=gpu.HARRIS_TUNE_FLAG_HANDOFF)):
        say("case repeat 300 launches, tuning %s" % (tune,))
        first = gpu.harris_coarsity_ex(rgb, K, tuning=tune).clone()
        out = torch.empty_like(first)
        for i in range(300):
            gpu.harris_coarsity_ex(rgb, K, tuning=tune, out=out)
            if i % 3 == 0:
                gpu.harris_coarsity_ex(other, K, tuning=tune, out=scratch)
            if i % 50 == 49:
                torch.cuda.synchronize()
                assert torch.equal(out, first)
        torch.cuda.synchronize()
        assert torch.equal(out, first)


def test_tile_schedule_shapes(gpu, oracle):
    for H, W in SHAPES:
        rgb = hi.white_noise_f32(200 + H + W, 2, H, W)
        say("case tiles f32 2x3x%dx%d" % (H, W))
        check(run_gpu(gpu, rgb, k=K, tuning=dict(schedule=2)), oracle.harris(rgb, K))


def test_lds_reservation_changes_nothing_but_the_residency(gpu, oracle):
    # Reserving more LDS than a tile needs only bounds the workgroups resident on a CU: the
    # results are the same bit for bit, for every reservation the planner uses and the extremes.
    import torch
    rgb = hi.rectangles_f32(230, 3, 150, 1000)
    want = oracle.harris(rgb, K)
    src = torch.from_numpy(rgb).cuda()
    for rows, waves in ((4, 4), (5, 4), (5, 5), (6, 5), (6, 4), (8, 9)):
        base = None
        for lds_kb in (0, 28, 36, 48, 64):
            say("case tile %dx%d with %d KB of LDS reserved" % (waves, rows, lds_kb))
            out = gpu.harris_coarsity_ex(src, K, tuning=dict(schedule=2, px=4, rows=rows, waves_per_block=waves, lds_kb=lds_kb))
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            check(got, want)
            base = got if base is None else base
            assert np.array_equal(got, base)
    for bad in (dict(lds_kb=65), dict(lds_kb=-1), dict(schedule=1, lds_kb=16)):
        with pytest.raises(gpu.HarrisError) as e:
            gpu.harris_coarsity_ex(src, K, tuning=bad)
        assert e.value.status == -3


@pytest.mark.parametrize("px", [1, 2, 4])
@pytest.mark.parametrize("prefetch", [3])
def test_u8_every_kernel_instance(gpu, oracle, px, prefetch):
    H, W = 39, 8 * 65
    rgb = hi.white_noise_u8(8, 2, H, W)
    want = oracle.harris(rgb, K)
    for rows, wpb, flags in ((5, 4, 0), (13, 1, 3)):
        tune = dict(schedule=1, px=px, rows=rows, prefetch=prefetch, waves_per_block=wpb, flags=flags)
        say("case u8 2x3x%dx%d %s" % (H, W, tune))
        check(run_gpu(gpu, rgb, k=K, tuning=tune), want)


@pytest.mark.parametrize("batch,H,W", [(1, 4100, 8), (1, 5, 20000), (300, 9, 9), (2, 6, 1025), (1, 2049, 12), (70000 // 1000, 5, 8)])
def test_extreme_aspect_ratios_and_many_small_images(gpu, oracle, batch, H, W):
    rgb = hi.white_noise_f32(300 + H + W, batch, H, W)
    want = oracle.harris(rgb, K, nthreads=4)
    for tune in (None, dict(schedule=1), dict(schedule=2, rows=8, waves_per_block=16), dict(schedule=1, rows=64, prefetch=3, waves_per_block=4)):
        say("case extreme %dx3x%dx%d %s" % (batch, H, W, tune))
        check(run_gpu(gpu, rgb, k=K, tuning=tune), want)


def test_misaligned_base_pointers(gpu, oracle):
    import torch
    H, W = 21, 300
    rgb = hi.white_noise_f32(9, 1, H, W)
    want = oracle.harris(rgb, K)
    flat = torch.zeros(rgb.size + 8, device="cuda")
    for off in (1, 2, 3):                       # input 4-, 8-, 4-byte aligned only
        say("case f32 input offset by %d floats" % off)
        flat[off:off + rgb.size] = torch.from_numpy(rgb.reshape(-1)).cuda()
        t = flat[off:off + rgb.size].view(1, 3, H, W)
        out = gpu.harris_coarsity(t, K)
        torch.cuda.synchronize()
        check(out.cpu().numpy(), want)
    oflat = torch.zeros(want.size + 8, device="cuda")
    src = torch.from_numpy(rgb).cuda()
    for off in (1, 2):
        say("case f32 result offset by %d floats" % off)
        o = oflat[off:off + want.size].view(1, H - 4, W - 4)
        gpu.harris_coarsity(src, K, out=o)
        torch.cuda.synchronize()
        check(o.cpu().numpy(), want)
    u8 = hi.white_noise_u8(10, 1, H, W)
    uflat = torch.zeros(u8.size + 8, dtype=torch.uint8, device="cuda")
    for off in (1, 2):
        say("case u8 input offset by %d bytes" % off)
        uflat[off:off + u8.size] = torch.from_numpy(u8.reshape(-1)).cuda()
        out = gpu.harris_coarsity_u8(uflat[off:off + u8.size].view(1, 3, H, W), K)
        torch.cuda.synchronize()
        check(out.cpu().numpy(), oracle.harris(u8, K))


def test_misaligned_base_pointers_on_the_narrow_paths(gpu, oracle):
    # The kernels with 1 and 2 pixels per lane, asked for explicitly, in both schedules.
    import torch
    H, W = 21, 300
    rgb = hi.white_noise_f32(11, 1, H, W)
    want = oracle.harris(rgb, K)
    flat = torch.zeros(rgb.size + 8, device="cuda")
    for off, px in ((1, 1), (2, 2), (2, 1), (3, 1)):
        flat[off:off + rgb.size] = torch.from_numpy(rgb.reshape(-1)).cuda()
        t = flat[off:off + rgb.size].view(1, 3, H, W)
        for schedule in (1, 2):
            say("case f32 input offset by %d floats, px %d, schedule %d" % (off, px, schedule))
            out = gpu.harris_coarsity_ex(t, K, tuning=dict(schedule=schedule, px=px))
            torch.cuda.synchronize()
            check(out.cpu().numpy(), want)
    u8 = hi.white_noise_u8(12, 1, H, W)
    want8 = oracle.harris(u8, K)
    uflat = torch.zeros(u8.size + 8, dtype=torch.uint8, device="cuda")
    for off, px in ((1, 1), (2, 2), (3, 1)):
        uflat[off:off + u8.size] = torch.from_numpy(u8.reshape(-1)).cuda()
        for schedule in (1, 2):
            say("case u8 input offset by %d bytes, px %d, schedule %d" % (off, px, schedule))
            out = gpu.harris_coarsity_ex(uflat[off:off + u8.size].view(1, 3, H, W), K, tuning=dict(schedule=schedule, px=px))
            torch.cuda.synchronize()
            check(out.cpu().numpy(), want8)


@pytest.mark.parametrize("W", [97, 98, 99, 261, 515, 1026])
def test_any_width_and_row_alignment_with_16_byte_lanes(gpu, oracle, W):
    # The tile kernel keeps four pixels per lane when rows are not naturally aligned: float32
    # rows on any 4-byte boundary (vector accesses need no more; the lane that straddles the
    # end of a row loads zeros beyond it and stores nothing there), 8-bit rows on any byte
    # (loaded as the aligned words that hold them, then shifted).  Input and result are views
    # inside larger buffers: guard bands show that nothing else is written, and whatever a
    # straddling access did would stay inside an allocation.
    import torch
    B, H = 2, 37
    n, m = H - 4, W - 4
    G = 1024
    rgb = hi.white_noise_f32(90 + W, B, H, W)
    want = oracle.harris(rgb, K)
    wantb = oracle.harris(rgb, K, window=1)
    u8 = hi.white_noise_u8(91 + W, B, H, W)
    want8 = oracle.harris(u8, K)
    obuf = torch.empty(G + B * n * m + 3 + G, device="cuda")

    def run(src, off_out, expect, **kw):
        obuf.fill_(float("nan"))
        out = obuf[G + off_out:G + off_out + B * n * m].view(B, n, m)
        gpu.harris_coarsity_ex(src, K, out=out, **kw)
        torch.cuda.synchronize()
        check(out.cpu().numpy(), expect)
        rest = obuf.clone()
        rest[G + off_out:G + off_out + B * n * m] = float("nan")
        assert bool(torch.isnan(rest).all())                     # guard bands untouched

    ibuf = torch.full((G + rgb.size + 3 + G,), 0.5, device="cuda")
    for off_in, off_out in ((0, 0), (1, 3), (2, 1), (3, 2)):
        src = ibuf[G + off_in:G + off_in + rgb.size].view(B, 3, H, W)
        src.copy_(torch.from_numpy(rgb))
        shape, _ = gpu.harris_plan(gpu.HARRIS_F32, B, H, W, rgb_align=4, out_align=4)
        assert shape["px"] == 4 and shape["schedule"] == gpu.HARRIS_SCHEDULE_TILES
        say("case f32 W=%d input offset %d result offset %d floats, default plan" % (W, off_in, off_out))
        run(src, off_out, want)
        if off_in != 1:
            continue
        for rows, waves, flags in ((4, 4, 0), (5, 2, gpu.HARRIS_TUNE_STREAM_LOADS | gpu.HARRIS_TUNE_KEEP_SHARED_ROWS), (6, 3, gpu.HARRIS_TUNE_CACHED_LOADS),
                                   (8, 2, gpu.HARRIS_TUNE_FLAG_HANDOFF), (9, 2, 0), (10, 2, gpu.HARRIS_TUNE_FLAG_HANDOFF)):
            say("case f32 W=%d tile %dx%d flags %d" % (W, waves, rows, flags))
            run(src, off_out, want, tuning=dict(schedule=2, px=4, rows=rows, waves_per_block=waves, flags=flags))
        say("case f32 W=%d binomial window" % W)
        run(src, off_out, wantb, window=1)
        with pytest.raises(gpu.HarrisError):                     # moved strip borders need naturally aligned lanes
            gpu.harris_coarsity_ex(src, K, tuning=dict(flags=gpu.HARRIS_TUNE_ALIGNED_STORES))
        with pytest.raises(gpu.HarrisError):                     # and so does the band schedule with px = 4
            gpu.harris_coarsity_ex(src, K, tuning=dict(schedule=1, px=4))

    ubuf = torch.full((G + u8.size + 3 + G,), 200, dtype=torch.uint8, device="cuda")
    for off_in in (0, 1, 2, 3):
        src = ubuf[G + off_in:G + off_in + u8.size].view(B, 3, H, W)
        src.copy_(torch.from_numpy(u8))
        say("case u8 W=%d input offset %d bytes, default plan" % (W, off_in))
        run(src, off_in, want8)
        for rows, waves, flags in ((4, 3, gpu.HARRIS_TUNE_STREAM_LOADS | gpu.HARRIS_TUNE_KEEP_SHARED_ROWS), (8, 2, gpu.HARRIS_TUNE_CACHED_LOADS), (8, 3, gpu.HARRIS_TUNE_STREAM_LOADS)):
            say("case u8 W=%d input offset %d tile %dx%d flags %d" % (W, off_in, waves, rows, flags))
            run(src, off_in, want8, tuning=dict(schedule=2, px=4, rows=rows, waves_per_block=waves, flags=flags))
    src = ubuf[G + 1:G + 1 + u8.size].view(B, 3, H, W)
    src.copy_(torch.from_numpy(u8))
    say("case u8 W=%d binomial window" % W)
    run(src, 0, oracle.harris(u8, K, window=1), window=1)
    for bad in (dict(schedule=2, px=4, rows=5), dict(schedule=2, px=4, rows=8, flags=gpu.HARRIS_TUNE_FLAG_HANDOFF)):
        with pytest.raises(gpu.HarrisError):                     # shifted rows: kernels for 4 and 8 rows, barrier only
            gpu.harris_coarsity_ex(src, K, tuning=bad)
    # 16-bit results on 4-byte boundaries keep the wide lanes too (8-byte stores)
    if W % 2 == 0:
        f32src = ibuf[G + 1:G + 1 + rgb.size].view(B, 3, H, W)
        f32src.copy_(torch.from_numpy(rgb))
        hbuf = torch.full((G + B * n * m + 2 + G,), float("nan"), dtype=torch.float16, device="cuda")
        for off_out in (0, 2):
            say("case f16 result W=%d offset %d" % (W, off_out))
            hbuf.fill_(float("nan"))
            out16 = hbuf[G + off_out:G + off_out + B * n * m].view(B, n, m)
            assert gpu.harris_plan_typed(gpu.HARRIS_F32, gpu.HARRIS_OUT_F16, B, H, W, rgb_align=4, out_align=4)[0]["px"] == 4
            gpu.harris_coarsity_typed(f32src, out16, K)
            out32 = torch.empty((B, n, m), device="cuda")
            gpu.harris_coarsity_typed(f32src, out32, K)
            torch.cuda.synchronize()
            bits = out16.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            check(out32.cpu().numpy(), want)
            assert np.array_equal(bits, oracle.round_to_16bit(out32.cpu().numpy(), "f16"))
            rest = hbuf.clone()
            rest[G + off_out:G + off_out + B * n * m] = float("nan")
            assert bool(torch.isnan(rest).all())


@pytest.mark.parametrize("W", [744, 1000, 488])
def test_strip_borders_on_64_byte_boundaries(gpu, oracle, W):
    # With px = 4 the tile kernel moves the border between two strips, row by row, to the
    # next 64-byte boundary of the result row's address.  Where that lies depends on the
    # base address and the row pitch modulo 16 floats: go through every phase of the base
    # (offsets of 0, 4, 8, 12 floats from a 64-byte boundary), with dense rows (pitch W-4,
    # every row another phase) and padded rows, three to five strips (W = 488: 484 = 2 x 240 + 4
    # columns need a third one) and guard bands all around; the same with fixed borders and
    # with 8-bit input.
    import torch
    H = 29
    n, m = H - 4, W - 4
    rgb = hi.white_noise_f32(60 + W, 2, H, W)
    want = oracle.harris(rgb, K)
    src = torch.from_numpy(rgb).cuda()
    u8 = hi.white_noise_u8(61 + W, 2, H, W)
    want8 = oracle.harris(u8, K)
    src8 = torch.from_numpy(u8).cuda()
    for pitch in (m, m + 4, m + 12, ((m + 15) // 16) * 16):
        for off in (0, 4, 8, 12):
            flat = torch.full((2 * n * pitch + 64,), float("nan"), device="cuda")
            assert flat.data_ptr() % 64 == 0
            view = flat[16 + off:16 + off + 2 * n * pitch].view(2, n, pitch)[:, :, :m]
            for flags in (gpu.HARRIS_TUNE_ALIGNED_STORES, gpu.HARRIS_TUNE_PLAIN_STORES):
                for rows, waves in ((4, 4), (8, 3), (5, 2)):
                    say("case borders W=%d pitch=%d offset=%d flags=%d tile %dx%d" % (W, pitch, off, flags, waves, rows))
                    flat.fill_(float("nan"))
                    gpu.harris_coarsity_pitched(src, view, K, tuning=dict(schedule=2, px=4, rows=rows, waves_per_block=waves, flags=flags))
                    torch.cuda.synchronize()
                    check(view.cpu().numpy(), want)
                    rest = flat.clone()
                    rest[16 + off:16 + off + 2 * n * pitch].view(2, n, pitch)[:, :, :m] = float("nan")
                    assert bool(torch.isnan(rest).all())             # padding and guard bands untouched
            say("case borders u8 W=%d pitch=%d offset=%d" % (W, pitch, off))
            gpu.harris_coarsity_pitched(src8, view, K, tuning=dict(flags=gpu.HARRIS_TUNE_ALIGNED_STORES))
            torch.cuda.synchronize()
            check(view.cpu().numpy(), want8)


# ---------------------------------------------------------------- operator variants

@pytest.mark.parametrize("scale", [1.0, S12])
@pytest.mark.parametrize("window", [0, 1])
@pytest.mark.parametrize("k", [0.04, 0.06, 0.0])
def test_operator_variants(gpu, oracle, scale, window, k):
    rgb = hi.rectangles_f32(31, 2, 90, 260)
    say("case variants scale=%g window=%d k=%g" % (scale, window, k))
    check(run_gpu(gpu, rgb, k=k, sobel_scale=scale, window=window), oracle.harris(rgb, k, scale, window), referee=(oracle, rgb, k, scale, window))


def test_reduced_workloads_all_recipes(gpu, oracle):
    for name, kw in [("noise_f32_1536x2560", dict(H=192, W=320)),
                     ("blobs_f32_2832x4256", dict(H=354, W=532, sigma_lo=3, sigma_hi=25)),
                     ("rects_f32_64x1080x1920", dict(batch=5, H=135, W=240)),
                     ("noise_u8_8192x8192", dict(H=256, W=512))]:
        rgb = hi.make(name, **kw)
        say("case reduced %s %s" % (name, rgb.shape))
        check(run_gpu(gpu, rgb, k=K), oracle.harris(rgb, K, nthreads=4), referee=(oracle, rgb))


# ---------------------------------------------------------------- pitched layouts: padded rows, regions of interest

def test_region_of_interest_and_padded_result(gpu, oracle):
    import torch
    big = hi.rectangles_f32(51, 2, 120, 340)
    dev = torch.from_numpy(big).cuda()
    for (y0, x0, H, W) in ((8, 16, 90, 260), (3, 5, 77, 131), (0, 2, 120, 338), (40, 64, 5, 5)):
        roi = dev[:, :, y0:y0 + H, x0:x0 + W]                       # a view: pitches of the big image
        padded = torch.full((2, H - 4 + 3, W - 4 + 7), float("nan"), device="cuda")
        out = padded[:, 1:1 + H - 4, 4:4 + W - 4]                   # a view into a larger result buffer
        say("case roi y0=%d x0=%d %dx%d" % (y0, x0, H, W))
        gpu.harris_coarsity_pitched(roi, out, K)
        torch.cuda.synchronize()
        check(out.cpu().numpy(), oracle.harris(np.ascontiguousarray(big[:, :, y0:y0 + H, x0:x0 + W]), K))
        rest = padded.clone(); rest[:, 1:1 + H - 4, 4:4 + W - 4] = float("nan")
        assert bool(torch.isnan(rest).all())                         # nothing written outside the view


def test_padded_rows_and_separate_planes(gpu, oracle):
    import torch
    H, W, pitch = 50, 250, 256                                       # rows rounded up to 256 elements
    rgb = hi.white_noise_u8(52, 3, H, W)
    store = torch.zeros((3, 3, H + 2, pitch), dtype=torch.uint8, device="cuda")
    view = store[:, :, 1:1 + H, :W]
    view.copy_(torch.from_numpy(rgb).cuda())
    out = torch.empty((3, H - 4, pitch), device="cuda")[:, :, :W - 4]
    say("case padded u8 rows")
    for tune in (None, dict(schedule=1), dict(schedule=2, rows=8, waves_per_block=3)):
        gpu.harris_coarsity_pitched(view, out, K, S12, 1, tuning=tune)
        torch.cuda.synchronize()
        check(out.cpu().numpy(), oracle.harris(rgb, K, S12, 1))
    f32 = hi.white_noise_f32(53, 2, 41, 260)
    store = torch.zeros((2, 3, 41, 264), device="cuda")              # 16-byte multiple pitch: widest lanes stay usable
    store[:, :, :, :260].copy_(torch.from_numpy(f32).cuda())
    res = torch.empty((2, 37, 256), device="cuda")
    gpu.harris_coarsity_pitched(store[:, :, :, :260], res, K)
    torch.cuda.synchronize()
    check(res.cpu().numpy(), oracle.harris(f32, K))


# ---------------------------------------------------------------- 16-bit results

def _as_f32(bits, fmt):
    if fmt == "f16":
        return bits.view(np.float16).astype(np.float32)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _ulp16(x, fmt):
    # spacing of the 16-bit format at |x| (11 or 8 significant bits), at least the subnormal spacing
    frac_bits, min_exp = (10, -14) if fmt == "f16" else (7, -126)
    e = np.floor(np.log2(np.maximum(np.abs(x).astype(np.float64), 2.0 ** min_exp)))
    return 2.0 ** (e - frac_bits)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_16_bit_results(gpu, oracle, fmt):
    # Two checks.  (1) The 16-bit result is the float32 result of the same kernel rounded to
    # nearest-even, bit for bit (the rounding is the oracle's, applied to the GPU's own float32
    # output: the same launch shape gives the same float32 values).  (2) Against the oracle's
    # float32 result rounded the same way: the float32 bar plus one spacing of the 16-bit
    # format (two float32 values within the bar may fall on either side of a rounding border).
    import torch
    tdt = torch.float16 if fmt == "f16" else torch.bfloat16
    for rgb, scale in ((hi.rectangles_f32(71, 2, 61, 520), 1.0), (hi.white_noise_u8(72, 1, 45, 264), 1.0),
                       (hi.white_noise_f32(73, 1, 37, 98), S12), (hi.white_noise_f32(74, 2, 22, 131), 1.0)):
        B, _, H, W = rgb.shape
        want32 = oracle.harris(rgb, K, scale)
        want16 = _as_f32(oracle.round_to_16bit(want32, fmt), fmt)
        src = torch.from_numpy(rgb).cuda()
        for tune in (None, dict(schedule=2, rows=8 if W % 2 == 0 else 4, waves_per_block=3), dict(schedule=2, rows=5 if W % 4 == 0 else 4, waves_per_block=2, flags=gpu.HARRIS_TUNE_PLAIN_STORES)):
            say("case %s result %s %s tuning %s" % (fmt, rgb.dtype, rgb.shape, tune))
            out16 = torch.full((B, H - 4, W - 4), float("nan"), dtype=tdt, device="cuda")
            gpu.harris_coarsity_typed(src, out16, K, scale, tuning=tune)
            out32 = torch.empty((B, H - 4, W - 4), dtype=torch.float32, device="cuda")
            # the same lane width as the 16-bit launch (rows of odd width get one pixel per lane there)
            gpu.harris_coarsity_typed(src, out32, K, scale, tuning=tune if W % 2 == 0 else dict(tune or {}, px=1))
            torch.cuda.synchronize()
            bits = out16.view(torch.int16).cpu().numpy().view(np.uint16)
            got32 = out32.cpu().numpy()
            check(got32, want32)
            assert np.array_equal(bits, oracle.round_to_16bit(got32, fmt))
            got16 = _as_f32(bits, fmt)
            bound = 1e-4 * float(np.abs(want32).max()) + 1e-6
            assert np.all(np.abs(got16.astype(np.float64) - want16) <= bound + _ulp16(want32, fmt))


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("W", [97, 131])
def test_16_bit_results_of_odd_width_in_padded_rows(gpu, oracle, fmt, W):
    # An odd number of 16-bit results per row, rows padded to an even pitch and a buffer on a
    # 4-byte boundary: every row starts on a 4-byte boundary, and the 32-bit word that holds a
    # row's last column also holds the first padding element.  That column must be written and
    # the padding must not (a store of whole words would do one or the other wrong).
    import torch
    tdt = torch.float16 if fmt == "f16" else torch.bfloat16
    B, H = 2, 41
    n, m = H - 4, W - 4
    pitch = m + 1
    rgb = hi.rectangles_f32(140 + W, B, H, W, n_rect=10)
    want32 = oracle.harris(rgb, K)
    src = torch.from_numpy(rgb).cuda()
    for off in (0, 2, 6):
        for tune in (None, dict(schedule=2, rows=4, waves_per_block=3)):
            say("case %s results, W=%d, row pitch %d, offset %d elements, tuning %s" % (fmt, W, pitch, off, tune))
            flat = torch.full((64 + B * n * pitch + 64,), float("nan"), dtype=tdt, device="cuda")
            view = flat[64 + off:64 + off + B * n * pitch].view(B, n, pitch)[:, :, :m]
            assert view.data_ptr() % 4 == 0 and (pitch * 2) % 4 == 0
            gpu.harris_coarsity_typed(src, view, K, tuning=tune)
            out32 = torch.empty((B, n, m), device="cuda")
            gpu.harris_coarsity_typed(src, out32, K, tuning=dict(tune or {}, px=1))   # the lane width such rows get
            torch.cuda.synchronize()
            got32 = out32.cpu().numpy()
            check(got32, want32)
            bits = view.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(bits, oracle.round_to_16bit(got32, fmt))       # every column written, the last one too
            rest = flat.clone()
            rest[64 + off:64 + off + B * n * pitch].view(B, n, pitch)[:, :, :m] = float("nan")
            assert bool(torch.isnan(rest).all())                                 # padding and guard bands untouched
    # 8-bit input takes the same path
    u8 = hi.white_noise_u8(141 + W, B, H, W)
    flat = torch.full((64 + B * n * pitch + 64,), float("nan"), dtype=tdt, device="cuda")
    view = flat[64:64 + B * n * pitch].view(B, n, pitch)[:, :, :m]
    gpu.harris_coarsity_typed(torch.from_numpy(u8).cuda(), view, K)
    out32 = torch.empty((B, n, m), device="cuda")
    gpu.harris_coarsity_typed(torch.from_numpy(u8).cuda(), out32, K, tuning=dict(px=1))
    torch.cuda.synchronize()
    check(out32.cpu().numpy(), oracle.harris(u8, K))
    assert np.array_equal(view.contiguous().view(torch.int16).cpu().numpy().view(np.uint16), oracle.round_to_16bit(out32.cpu().numpy(), fmt))
    rest = flat.clone()
    rest[64:64 + B * n * pitch].view(B, n, pitch)[:, :, :m] = float("nan")
    assert bool(torch.isnan(rest).all())


def test_16_bit_results_layouts_and_overflow(gpu, oracle):
    import torch
    # every 8-byte phase of the result address with moved strip borders (64 bytes = 32 columns),
    # dense and padded rows, several strips, guard bands
    H, W = 23, 1000
    n, m = H - 4, W - 4
    rgb = hi.white_noise_f32(75, 2, H, W)
    src = torch.from_numpy(rgb).cuda()
    want = oracle.round_to_16bit(oracle.harris(rgb, K), "f16")
    for pitch in (m, m + 4, m + 20):
        for off in (0, 4, 12, 28):
            flat = torch.full((2 * n * pitch + 128,), float("nan"), dtype=torch.float16, device="cuda")
            view = flat[32 + off:32 + off + 2 * n * pitch].view(2, n, pitch)[:, :, :m]
            say("case f16 borders pitch=%d offset=%d" % (pitch, off))
            gpu.harris_coarsity_typed(src, view, K, tuning=dict(flags=gpu.HARRIS_TUNE_ALIGNED_STORES))
            torch.cuda.synchronize()
            got = view.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            diff = np.abs(_as_f32(got, "f16").astype(np.float64) - _as_f32(want, "f16"))
            assert np.all(diff <= 1e-4 * float(_as_f32(want, "f16").max()) + 1e-6 + _ulp16(_as_f32(want, "f16"), "f16"))
            rest = flat.clone()
            rest[32 + off:32 + off + 2 * n * pitch].view(2, n, pitch)[:, :, :m] = float("nan")
            assert bool(torch.isnan(rest).all())
    # binary16 overflows to infinity from 65520 on: an image scaled by 8 gives results 4096 times larger
    big = (hi.rectangles_f32(76, 1, 40, 260) * 8.0).astype(np.float32)
    want32 = oracle.harris(big, K)
    assert np.abs(want32).max() > 65520
    out = torch.empty((1, 36, 256), dtype=torch.float16, device="cuda")
    gpu.harris_coarsity_typed(torch.from_numpy(big).cuda(), out, K)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    wantb = oracle.round_to_16bit(want32, "f16")
    clear = np.abs(np.abs(want32) - 65520) > 1e-4 * np.abs(want32).max()       # away from the overflow border
    assert np.array_equal(np.isinf(_as_f32(got, "f16"))[clear], np.isinf(_as_f32(wantb, "f16"))[clear])
    assert np.isinf(_as_f32(got, "f16")).any()
    # infinities and NaN survive the conversion to either format: a NaN and an infinite sample
    # in the image spoil the results around them, the rest stays finite
    huge = big.copy()
    huge[0, 1, 10, 20] = np.nan
    huge[0, 0, 30, 200] = np.inf
    src = torch.from_numpy(huge).cuda()
    out32 = torch.empty((1, 36, 256), device="cuda")
    gpu.harris_coarsity_typed(src, out32, K)
    got32 = out32.cpu().numpy()
    assert np.isnan(got32).any() and np.isfinite(got32).any()
    for fmt, tdt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        say("case %s of infinities and NaN" % fmt)
        out16 = torch.empty((1, 36, 256), dtype=tdt, device="cuda")
        gpu.harris_coarsity_typed(src, out16, K)
        torch.cuda.synchronize()
        g = _as_f32(out16.view(torch.int16).cpu().numpy().view(np.uint16), fmt)
        w = _as_f32(oracle.round_to_16bit(got32, fmt), fmt)
        assert np.array_equal(np.isnan(g), np.isnan(w)) and np.array_equal(g[~np.isnan(w)], w[~np.isnan(w)])
    # the band schedule has no 16-bit results
    with pytest.raises(gpu.HarrisError) as e:
        gpu.harris_coarsity_typed(torch.from_numpy(big).cuda(), out, K, tuning=dict(schedule=1))
    assert e.value.status == -3


def test_8_bit_codes(gpu, oracle):
    # (1) The codes equal the oracle's quantisation of the kernel's own float32 result bit for
    # bit.  (2) Against the oracle's codes of the oracle's float32 result: two float32 values
    # within the bar give codes at most ceil(bar * |scale|) + 1 apart.  Several lane widths,
    # tile shapes, padded rows, every phase of the row address, guard bands, clamping at both ends.
    import torch
    for rgb, scale, q_scale, q_offset in ((hi.rectangles_f32(81, 2, 45, 520), 1.0, 0.5, 128.0), (hi.white_noise_u8(82, 1, 33, 264), 1.0, 2.0, 100.0),
                                          (hi.white_noise_f32(83, 1, 37, 98), 1.0, -1.0, 64.0), (hi.white_noise_f32(84, 2, 22, 131), S12, 30000.0, 10.0)):
        B, _, H, W = rgb.shape
        n, m = H - 4, W - 4
        want32 = oracle.harris(rgb, K, scale)
        want8 = oracle.quantize_u8(want32, q_scale, q_offset).astype(int)
        src = torch.from_numpy(rgb).cuda()
        slack = int(np.ceil((1e-4 * float(np.abs(want32).max()) + 1e-6) * abs(q_scale))) + 1
        for pitch, off, tune in ((m, 0, None), (m + 4, 4, dict(schedule=2, rows=8 if W % 4 == 0 else 4, waves_per_block=3)), (m + 9, 1, None),
                                 (m, 8, dict(flags=gpu.HARRIS_TUNE_ALIGNED_STORES) if W % 4 == 0 else None)):
            say("case 8-bit codes %s %s pitch=%d offset=%d tuning %s" % (rgb.dtype, rgb.shape, pitch, off, tune))
            flat = torch.full((B * n * pitch + 32,), 77, dtype=torch.uint8, device="cuda")
            view = flat[off:off + B * n * pitch].view(B, n, pitch)[:, :, :m]
            gpu.harris_coarsity_quantized(src, view, q_scale, q_offset, K, scale, tuning=tune)
            f32 = torch.empty((B, n, m), device="cuda")
            gpu.harris_coarsity_typed(src, f32, K, scale)
            torch.cuda.synchronize()
            got = view.cpu().numpy()
            assert np.array_equal(got, oracle.quantize_u8(f32.cpu().numpy(), q_scale, q_offset))
            assert np.all(np.abs(got.astype(int) - want8) <= slack)
            assert got.min() == 0 or got.max() == 255 or q_scale == 0.5       # the chosen scales reach the clamp
            rest = flat.clone()
            rest[off:off + B * n * pitch].view(B, n, pitch)[:, :, :m] = 77
            assert bool((rest == 77).all())
    # Rounding itself: with a scale of 0 every code is the rounded, clamped offset (ties go to
    # the even code, anything outside [0, 255] to the nearer end), and a NaN result gives 0.
    rgb = hi.white_noise_f32(85, 1, 20, 264)
    rgb[0, 2, 9, 100] = np.nan
    src = torch.from_numpy(rgb).cuda()
    codes = torch.empty((1, 16, 260), dtype=torch.uint8, device="cuda")
    f32 = torch.empty((1, 16, 260), device="cuda")
    gpu.harris_coarsity_typed(src, f32, K)
    for q_offset, code in ((0.5, 0), (1.5, 2), (2.5, 2), (3.5, 4), (254.5, 254), (255.5, 255), (0.49999997, 0), (0.50000006, 1), (1.4999999, 1),
                           (127.5, 128), (128.5, 128), (-0.5, 0), (-7.0, 0), (255.49998, 255), (300.0, 255), (1e30, 255), (-1e30, 0), (77.0, 77)):
        say("case 8-bit code of %r" % q_offset)
        gpu.harris_coarsity_quantized(src, codes, 0.0, q_offset)
        torch.cuda.synchronize()
        got = codes.cpu().numpy()
        assert np.array_equal(got, oracle.quantize_u8(f32.cpu().numpy(), 0.0, q_offset))
        nan = np.isnan(f32.cpu().numpy())
        assert nan.any() and np.all(got[nan] == 0) and np.all(got[~nan] == code)
    with pytest.raises(gpu.HarrisError):
        gpu.harris_coarsity_quantized(src, codes, 1.0, 0.0, tuning=dict(schedule=1))


# ---------------------------------------------------------------- seeded random shapes, layouts and launch shapes

def test_random_shapes_layouts_and_launch_shapes(gpu, oracle):
    # 60 seeded cases over everything a caller can vary at once: batch, height, width (any
    # residue modulo 4), input and result type, Sobel scale, window, k, row padding and base
    # offsets of both arrays (so every lane width and every phase of a moved strip border
    # occurs), and a launch shape drawn from the valid ones.  Guard bands and padding must stay
    # untouched.
    import torch
    rng = np.random.default_rng(20221212)
    for case in range(60):
        B = int(rng.integers(1, 4)); H = int(rng.integers(5, 70)); W = int(rng.choice([rng.integers(5, 40), rng.integers(40, 300), rng.integers(300, 800)]))
        if rng.random() < 0.5:
            W = max(8, W // 4 * 4)                                   # half of the cases on the 16-byte path
        u8 = bool(rng.random() < 0.35)
        fmt = str(rng.choice(["f32", "f32", "f16", "bf16"]))
        scale = float(rng.choice([1.0, S12])); window = int(rng.integers(0, 2)); k = float(rng.choice([0.04, 0.06, 0.15]))
        n, m = H - 4, W - 4
        in_pitch = W + int(rng.choice([0, 0, 4, 7, 12])); in_off = int(rng.choice([0, 0, 4, 1, 16]))
        out_pitch = m + int(rng.choice([0, 0, 4, 5, 8, 28])); out_off = int(rng.choice([0, 0, 4, 2, 8, 12, 20]))
        rgb = hi.white_noise_u8(1000 + case, B, H, W) if u8 else hi.rectangles_f32(1000 + case, B, H, W, n_rect=12)
        store = torch.zeros(B * 3 * H * in_pitch + 64, dtype=torch.uint8 if u8 else torch.float32, device="cuda")
        src = store[in_off:in_off + B * 3 * H * in_pitch].view(B, 3, H, in_pitch)[:, :, :, :W]
        src.copy_(torch.from_numpy(rgb).cuda())
        tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[fmt]
        flat = torch.full((B * n * out_pitch + 64,), float("nan"), dtype=tdt, device="cuda")
        view = flat[out_off:out_off + B * n * out_pitch].view(B, n, out_pitch)[:, :, :m]
        tune = None
        r = rng.random()
        if r < 0.3:
            tune = dict(schedule=2, rows=int(rng.choice([4, 8])), waves_per_block=int(rng.integers(2, 9)))
        elif r < 0.45 and fmt == "f32":
            tune = dict(schedule=1, rows=int(rng.integers(1, 40)), prefetch=3 + 0 * int(rng.choice([2, 3, 6])), waves_per_block=int(rng.choice([1, 2, 4])))
        say("case random %d: %s %dx3x%dx%d -> %s scale=%g window=%d k=%g pitches %d/%d offsets %d/%d tuning %s"
            % (case, "u8" if u8 else "f32", B, H, W, fmt, scale, window, k, in_pitch, out_pitch, in_off, out_off, tune))
        try:
            gpu.harris_coarsity_typed(src, view, k, scale, window, tuning=tune)
        except gpu.HarrisError as e:                             # 8 rows per wavefront exist with four pixels per lane only
            assert e.status == -3 and tune is not None and tune.get("rows") == 8
            tune = dict(tune, rows=4)
            say("   (this layout runs with narrower lanes: 4 rows per wavefront)")
            gpu.harris_coarsity_typed(src, view, k, scale, window, tuning=tune)
        torch.cuda.synchronize()
        want = oracle.harris(rgb, k, scale, window)
        got = view.float().cpu().numpy()
        bound = 1e-4 * float(np.abs(want).max()) + 1e-6
        if fmt == "f32":
            check(got, want)
        else:
            want16 = _as_f32(oracle.round_to_16bit(want, fmt), fmt)
            assert np.all(np.abs(got.astype(np.float64) - want16) <= bound + _ulp16(want, fmt))
        rest = flat.clone()
        rest[out_off:out_off + B * n * out_pitch].view(B, n, out_pitch)[:, :, :m] = float("nan")
        assert bool(torch.isnan(rest).all())


def test_random_tile_shapes_policies_and_reservations(gpu, oracle):
    # 80 seeded cases on larger images (several tiles down and across, ragged last ones) with a
    # tile shape drawn from everything the library has kernels for: 4 to 10 rows per wavefront, 2 to
    # 16 wavefronts, each load policy, the barrier or the ready flags, any LDS reservation; shapes
    # the library rejects fall back to its own plan.  Float32 and 8-bit input, float32 and 16-bit
    # results, padded rows and offset bases; guard bands and padding must stay untouched.
    import torch
    rng = np.random.default_rng(20221213)
    for case in range(80):
        B = int(rng.integers(1, 4)); H = int(rng.choice([rng.integers(30, 200), rng.integers(200, 500)]))
        W = int(rng.choice([rng.integers(40, 300), rng.integers(300, 1300)]))
        if rng.random() < 0.5:
            W = max(8, W // 4 * 4)
        u8 = bool(rng.random() < 0.4)
        fmt = str(rng.choice(["f32", "f32", "f16", "bf16"]))
        scale = float(rng.choice([1.0, S12])); window = int(rng.integers(0, 2)); k = float(rng.choice([0.04, 0.06]))
        n, m = H - 4, W - 4
        in_pitch = W + int(rng.choice([0, 0, 4, 7, 1, 33])); in_off = int(rng.choice([0, 0, 4, 1, 3]))
        out_pitch = m + int(rng.choice([0, 0, 4, 5, 1, 3])); out_off = int(rng.choice([0, 0, 4, 2, 1, 3]))
        rgb = hi.white_noise_u8(3000 + case, B, H, W) if u8 else hi.rectangles_f32(3000 + case, B, H, W, n_rect=12)
        store = torch.zeros(B * 3 * H * in_pitch + 64, dtype=torch.uint8 if u8 else torch.float32, device="cuda")
        src = store[in_off:in_off + B * 3 * H * in_pitch].view(B, 3, H, in_pitch)[:, :, :, :W]
        src.copy_(torch.from_numpy(rgb).cuda())
        tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[fmt]
        flat = torch.full((B * n * out_pitch + 64,), float("nan"), dtype=tdt, device="cuda")
        view = flat[out_off:out_off + B * n * out_pitch].view(B, n, out_pitch)[:, :, :m]
        flags = 0
        if rng.random() < 0.5:
            flags |= gpu.HARRIS_TUNE_STREAM_LOADS
        if rng.random() < 0.3:
            flags |= gpu.HARRIS_TUNE_STREAM_LOADS | gpu.HARRIS_TUNE_KEEP_SHARED_ROWS
        if rng.random() < 0.3 and not u8:
            flags |= gpu.HARRIS_TUNE_FLAG_HANDOFF
        tune = dict(schedule=2, rows=int(rng.choice([4, 5, 6, 8, 9, 10])), waves_per_block=int(rng.integers(2, 17)), flags=flags,
                    lds_kb=int(rng.choice([0, 0, 28, 36, 48, 64])))
        say("case random tiles %d: %s %dx3x%dx%d -> %s scale=%g window=%d k=%g pitches %d/%d offsets %d/%d tuning %s"
            % (case, "u8" if u8 else "f32", B, H, W, fmt, scale, window, k, in_pitch, out_pitch, in_off, out_off, tune))
        try:
            gpu.harris_coarsity_typed(src, view, k, scale, window, tuning=tune)
        except gpu.HarrisError as e:
            assert e.status == -3
            say("   (no kernel for this shape and layout: the library's own plan instead)")
            gpu.harris_coarsity_typed(src, view, k, scale, window)
        torch.cuda.synchronize()
        want = oracle.harris(rgb, k, scale, window)
        got = view.float().cpu().numpy()
        bound = 1e-4 * float(np.abs(want).max()) + 1e-6
        if fmt == "f32":
            check(got, want)
        else:
            want16 = _as_f32(oracle.round_to_16bit(want, fmt), fmt)
            with np.errstate(invalid="ignore"):                      # a value beyond binary16's range is infinite on both sides
                assert np.all((np.abs(got.astype(np.float64) - want16) <= bound + _ulp16(want, fmt)) | (np.isinf(want16) & (got == want16)))
        rest = flat.clone()
        rest[out_off:out_off + B * n * out_pitch].view(B, n, out_pitch)[:, :, :m] = float("nan")
        assert bool(torch.isnan(rest).all())


# ---------------------------------------------------------------- the streaming-copy probe (measurement aid)

def test_copy_probe_moves_what_it_says(gpu):
    # Not the Harris operator: out[b][i] = R[i] + G[i] + B[i] over the first (H-4)*(W-4) elements of
    # the flat planes.  Exact in float32 for these inputs (sums of three small integers or of
    # multiples of 2^-10), several chunks per wavefront and a ragged last chunk.
    import torch
    for B, H, W, u8 in ((2, 36, 260, False), (1, 12, 8, False), (3, 40, 1028, True), (1, 68, 132, True)):
        rng = np.random.default_rng(H * W)
        if u8:
            rgb = rng.integers(0, 256, size=(B, 3, H, W), dtype=np.uint8)
        else:
            rgb = (rng.integers(0, 1024, size=(B, 3, H, W)) / 1024.0).astype(np.float32)
        n = (H - 4) * (W - 4)
        flat = rgb.reshape(B, 3, H * W).astype(np.float32)
        want = (flat[:, 0, :n] + flat[:, 1, :n] + flat[:, 2, :n]).reshape(B, H - 4, W - 4)
        say("case copy probe %s %dx3x%dx%d" % ("u8" if u8 else "f32", B, H, W))
        out = torch.full((B, H - 4, W - 4), float("nan"), device="cuda")
        gpu.harris_probe_copy(torch.from_numpy(rgb).cuda(), out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("B,H,W,u8", [(8, 1080, 1920, False), (16, 1080, 1920, False), (1, 8192, 4096, True), (1, 8192, 8192, True)])
def test_copy_probe_at_the_sizes_where_its_store_policy_changes(gpu, B, H, W, u8):
    # Above 128 MB and above 400 MB the probe stores with other cache policies (kernels of their own).
    import torch
    say("case copy probe %s %dx3x%dx%d" % ("u8" if u8 else "f32", B, H, W))
    gen = torch.Generator(device="cuda").manual_seed(H + W + B)
    if u8:
        rgb = torch.randint(0, 256, (B, 3, H, W), dtype=torch.uint8, device="cuda", generator=gen)
    else:
        rgb = torch.randint(0, 1024, (B, 3, H, W), device="cuda", generator=gen).float() / 1024.0
    n = (H - 4) * (W - 4)
    flat = rgb.reshape(B, 3, H * W)[:, :, :n].float()
    want = (flat[:, 0] + flat[:, 1] + flat[:, 2]).reshape(B, H - 4, W - 4)       # exact in float32 for these values
    out = torch.full((B, H - 4, W - 4), float("nan"), device="cuda")
    gpu.harris_probe_copy(rgb, out)
    torch.cuda.synchronize()
    assert torch.equal(out, want)


def test_stream_probes_touch_what_they_say(gpu):
    # Measurement aids: the writing probe fills exactly `bytes` bytes (every fourth word of its
    # pattern is the bits of 1.0f), the reading probe writes nothing, not even its sink.
    import torch
    for nbytes in (16, 1024, 4096 + 64, 5 * 4096 * 4 + 1040):
        say("case stream probes, %d bytes" % nbytes)
        buf = torch.full((nbytes // 4 + 64,), -7, dtype=torch.int32, device="cuda")
        gpu.harris_probe_stream(gpu.HARRIS_PROBE_WRITE, None, buf, nbytes)
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert np.all(host[3:nbytes // 4:4] == 0x3f800000) and np.all(host[2:nbytes // 4:4] == 0) and np.all(host[nbytes // 4:] == -7)
        assert np.array_equal(host[0:nbytes // 4:4] % 64, (np.arange(nbytes // 16) % 64))     # the lane that wrote each 16 bytes
        sink = torch.full((16,), -7, dtype=torch.int32, device="cuda")
        gpu.harris_probe_stream(gpu.HARRIS_PROBE_READ, buf, sink, nbytes)
        torch.cuda.synchronize()
        assert bool((sink == -7).all()) and np.array_equal(buf.cpu().numpy(), host)
    say("case idle launch, eager and in a graph")
    guard = torch.full((1024,), -7, dtype=torch.int32, device="cuda")
    gpu.harris_probe_stream(gpu.HARRIS_PROBE_NONE, None, None, 0)          # no pointers: it touches no memory
    gpu.harris_probe_stream(gpu.HARRIS_PROBE_NONE, guard, guard, 4096)      # and ignores those it gets
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(50):
            gpu.harris_probe_stream(gpu.HARRIS_PROBE_NONE, None, None, 0)
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    assert bool((guard == -7).all())


# ---------------------------------------------------------------- unfused kernel groupings (baselines)

@pytest.mark.parametrize("grouping", [1, 2, 3, 4])
def test_kernel_groupings_match_the_oracle(gpu, oracle, grouping):
    import torch
    for rgb, scale, window, k in ((hi.rectangles_f32(41, 3, 70, 150), 1.0, 0, K), (hi.white_noise_u8(42, 2, 33, 67), S12, 1, 0.06),
                                  (hi.white_noise_f32(43, 1, 5, 5), 1.0, 0, K)):
        say("case grouping %d %s %s scale=%g window=%d" % (grouping, rgb.dtype, rgb.shape, scale, window))
        out = gpu.harris_coarsity_grouped(torch.from_numpy(rgb).cuda(), k, scale, window, grouping)
        torch.cuda.synchronize()
        check(out.cpu().numpy(), oracle.harris(rgb, k, scale, window))


def test_groupings_agree_with_the_fused_kernel_at_full_size(gpu):
    import torch
    rgb = torch.from_numpy(hi.make("noise_f32_1536x2560")).cuda()
    say("case groupings vs fused, full 1536x2560")
    fused = gpu.harris_coarsity(rgb, K)
    ws = torch.empty(gpu.harris_grouped_workspace_bytes(1, 1, 1536, 2560) // 4, device="cuda")
    for grouping in (1, 2, 3):
        other = gpu.harris_coarsity_grouped(rgb, K, grouping=grouping, workspace=ws)
        torch.cuda.synchronize()
        scale = float(fused.abs().max())
        assert float((other - fused).abs().max()) <= 1e-4 * scale + 1e-6


# ---------------------------------------------------------------- degenerate inputs and closed forms on the GPU

def test_constant_image_gives_exact_zero(gpu):
    rgb = np.empty((1, 3, 40, 300), np.float32)
    rgb[0, 0], rgb[0, 1], rgb[0, 2] = 0.8125, 0.3, 0.61
    say("case constant image")
    assert np.all(run_gpu(gpu, rgb, k=K) == 0.0)
    u8 = np.full((1, 3, 17, 64), 201, np.uint8)
    assert np.all(run_gpu(gpu, u8, k=K) == 0.0)


def test_horizontal_ramp_closed_form(gpu):
    a = 2.0 ** -8
    y, x = np.mgrid[0:20, 0:280]
    g = (a * x + 0.125).astype(np.float32)
    rgb = np.ascontiguousarray(np.broadcast_to(g[None, None], (1, 3, 20, 280)))
    say("case ramp")
    out = run_gpu(gpu, rgb, k=K)
    expect = -float(np.float32(K)) * (9.0 * (8 * a) ** 2) ** 2
    # gray is rounded to f32 before the differences: a few 1e-5 relative on Ix^4
    assert np.abs(out - expect).max() <= 1e-4 * abs(expect)


def test_empty_results(gpu):
    import torch
    say("case empty results")
    assert tuple(gpu.harris_coarsity(torch.zeros(0, 3, 16, 16, device="cuda")).shape) == (0, 12, 12)
    assert tuple(gpu.harris_coarsity(torch.zeros(2, 3, 4, 16, device="cuda")).shape) == (2, 0, 12)
    assert tuple(gpu.harris_coarsity_u8(torch.zeros(2, 3, 16, 4, dtype=torch.uint8, device="cuda")).shape) == (2, 12, 0)
    with pytest.raises(gpu.HarrisError):
        gpu.harris_coarsity(torch.zeros(1, 3, 3, 16, device="cuda"))


def test_runs_on_a_side_stream(gpu, oracle):
    import torch
    rgb = hi.white_noise_f32(77, 1, 64, 512)
    say("case side stream")
    s = torch.cuda.Stream()
    t = torch.from_numpy(rgb).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = gpu.harris_coarsity(t, K)
    s.synchronize()
    check(out.cpu().numpy(), oracle.harris(rgb, K))


def test_concurrent_calls_from_host_threads_on_their_own_streams(gpu, oracle):
    # The library keeps no state between calls: four host threads, each with a stream, inputs and
    # results of its own (default stream priority), launch different problems at the same time,
    # so that kernels of several calls share the GPU; every result is checked against the oracle.
    import threading
    import torch
    jobs = [(hi.white_noise_f32(500, 2, 300, 1000), None),
            (hi.white_noise_u8(501, 1, 400, 1203), None),
            (hi.rectangles_f32(502, 1, 700, 1500, n_rect=20), dict(schedule=2, px=4, rows=8, waves_per_block=9, flags=gpu.HARRIS_TUNE_FLAG_HANDOFF)),
            (hi.white_noise_f32(503, 3, 90, 517), dict(schedule=1, rows=16, prefetch=3, waves_per_block=2))]
    srcs = [torch.from_numpy(rgb).cuda() for rgb, _ in jobs]
    outs = [torch.empty((rgb.shape[0], rgb.shape[2] - 4, rgb.shape[3] - 4), device="cuda") for rgb, _ in jobs]
    streams = [torch.cuda.Stream() for _ in jobs]
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            with torch.cuda.stream(streams[i]):
                for _ in range(40):
                    gpu.harris_coarsity_ex(srcs[i], K, tuning=jobs[i][1], out=outs[i])
            streams[i].synchronize()
        except Exception as e:                                   # reported by the main thread
            errors.append((i, e))

    say("case four host threads, four streams, 40 launches each")
    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(jobs))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for (rgb, _), out in zip(jobs, outs):
        check(out.cpu().numpy(), oracle.harris(rgb, K))


def test_captured_in_a_graph_and_replayed(gpu, oracle):
    # The library allocates nothing and never synchronises, so its launches can be captured.
    # A graph of three launches (barrier hand-over, ready flags with 64 KB of LDS reserved, 8-bit
    # input through the shifted loads) is replayed several times with fresh inputs and eager work in between; every
    # replay is checked against the oracle and against the eager launch, bit for bit.
    import torch
    H, W = 150, 1000
    a = torch.empty((1, 3, H, W), device="cuda")
    b = torch.empty((1, 3, H, W - 1), dtype=torch.uint8, device="cuda")
    out_a = torch.empty((1, H - 4, W - 4), device="cuda")
    out_f = torch.empty((1, H - 4, W - 4), device="cuda")
    out_b = torch.empty((1, H - 4, W - 5), device="cuda")
    flags_tuning = dict(schedule=2, px=4, rows=8, waves_per_block=5, flags=gpu.HARRIS_TUNE_FLAG_HANDOFF, lds_kb=64)
    a.copy_(torch.from_numpy(hi.white_noise_f32(400, 1, H, W)))
    b.copy_(torch.from_numpy(hi.white_noise_u8(401, 1, H, W - 1)))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                # one eager pass on the capture stream first
        gpu.harris_coarsity_ex(a, K, out=out_a)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.harris_coarsity_ex(a, K, out=out_a)
        gpu.harris_coarsity_ex(a, K, out=out_f, tuning=flags_tuning)
        gpu.harris_coarsity_ex(b, K, out=out_b)
    for replay in range(4):
        say("case graph replay %d" % replay)
        rgb = hi.white_noise_f32(410 + replay, 1, H, W)
        u8 = hi.white_noise_u8(420 + replay, 1, H, W - 1)
        a.copy_(torch.from_numpy(rgb))
        b.copy_(torch.from_numpy(u8))
        for o in (out_a, out_f, out_b):
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_a, got_f, got_b = out_a.cpu().numpy(), out_f.cpu().numpy(), out_b.cpu().numpy()
        check(got_a, oracle.harris(rgb, K))
        check(got_f, oracle.harris(rgb, K))
        check(got_b, oracle.harris(u8, K))
        eager_a = gpu.harris_coarsity_ex(a, K)                   # eager work between the replays
        eager_f = gpu.harris_coarsity_ex(a, K, tuning=flags_tuning)
        eager_b = gpu.harris_coarsity_ex(b, K)
        torch.cuda.synchronize()
        assert np.array_equal(got_a, eager_a.cpu().numpy()) and np.array_equal(got_f, eager_f.cpu().numpy()) and np.array_equal(got_b, eager_b.cpu().numpy())


# ---------------------------------------------------------------- full sizes, in the launch shape the benchmark times

@pytest.mark.parametrize("name", ["noise_f32_1536x2560", "blobs_f32_2832x4256", "noise_u8_8192x8192"])
def test_full_size_single_images(gpu, oracle, name):
    rgb = hi.make(name)
    say("case full %s %s plan %s" % (name, rgb.shape, gpu.harris_plan(1 if rgb.dtype == np.uint8 else 0, *rgb.shape[:1], *rgb.shape[2:])))
    got = run_gpu(gpu, rgb, k=K)
    want = oracle.harris(rgb, K, nthreads=oracle.hardware_threads())
    say("   ratio to bound: %.3g" % check(got, want, referee=(oracle, rgb, K, 1.0, 0, oracle.hardware_threads())))


@pytest.mark.parametrize("name", ["noise_f32_1536x2560", "blobs_f32_2832x4256"])
def test_full_size_psnr_of_the_thesis_operator(gpu, oracle, name):
    # The thesis's own consistency check (section 4.4): mean squared error and PSNR against a
    # reference output, "always above 170 dB", on its two image sizes, for the operator exactly
    # as its listings define it (Sobel matrices scaled by 1/12).  The reference here is the
    # float64 oracle; the peak is taken as 1, the range of the input image (the thesis does not
    # say which peak it uses).
    rgb = hi.make(name)
    say("case psnr %s" % name)
    got = run_gpu(gpu, rgb, k=K, sobel_scale=S12).astype(np.float64)
    want = oracle.harris(rgb, K, S12, precision="f64", nthreads=oracle.hardware_threads())
    mse = float(np.mean((got - want) ** 2))
    psnr = 10.0 * np.log10(1.0 / mse) if mse > 0 else float("inf")
    say("   mse %.3g  psnr %.1f dB" % (mse, psnr))
    assert psnr > 170.0


def test_full_size_batch_of_64(gpu, oracle):
    import torch
    name = "rects_f32_64x1080x1920"
    rgb = hi.make(name)
    say("case full %s %s plan %s" % (name, rgb.shape, gpu.harris_plan(0, 64, 1080, 1920)))
    got = run_gpu(gpu, rgb, k=K)
    nt = oracle.hardware_threads()
    worst = 0.0
    for b in range(rgb.shape[0]):            # the oracle one image at a time: bounded memory
        want = oracle.harris(rgb[b], K, nthreads=nt)
        worst = max(worst, check(got[b], want, referee=(oracle, rgb[b], K, 1.0, 0, nt) if b % 16 == 0 else None))
        assert want.max() > 0                # rectangles have corners: positive responses exist
        if b % 16 == 15:
            say("   image %d done" % b)
    say("   worst ratio to bound: %.3g" % worst)
