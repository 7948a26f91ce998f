"""The entry point that allocates nothing: harris_coarsity_grouped_static against
harris_coarsity_grouped (same kernels, the caller's workspace) and against the oracle.

Collected last on purpose (the file name sorts behind the other test files)."""
import ctypes
import os
import sys

import numpy as np
import pytest

import harris_inputs as hi

pytestmark = pytest.mark.gpu

K = 0.04


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need a GPU"
    import paper_2212_12035_amd as pkg
    if not os.path.exists(pkg.library_path()):
        from paper_2212_12035_amd import build
        build.build_library()
    pkg.load_library()
    return pkg


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_static_scratch_matches_the_callers_workspace_on_two_calls_in_a_row(gpu, oracle):
    # Two calls in a row through the C interface, the second on a smaller image, so that the
    # array still holds the first call's intermediates beyond what the second one overwrites.
    # The kernels and the layout of the intermediates are those of harris_coarsity_grouped:
    # the results must be the same bit for bit, and within the bar of the oracle.
    import torch
    lib = gpu.load_library()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    big = hi.rectangles_f32(501, 2, 300, 700)
    small = hi.white_noise_u8(502, 1, 61, 133)
    for grouping in (1, 2, 3):
        for rgb, scale, window in ((big, 1.0, 0), (small, 1.0 / 12.0, 1)):
            B, _, H, W = rgb.shape
            dtype = gpu.HARRIS_U8 if rgb.dtype == np.uint8 else gpu.HARRIS_F32
            say("case static scratch: grouping %d, %s %s" % (grouping, rgb.dtype, rgb.shape))
            src = torch.from_numpy(rgb).cuda()
            got = torch.full((B, H - 4, W - 4), float("nan"), device="cuda")
            rc = lib.harris_coarsity_grouped_static(ctypes.c_void_p(src.data_ptr()), dtype, B, H, W, K, scale, window, grouping,
                                                    ctypes.c_void_p(got.data_ptr()), stream)
            assert rc == 0, gpu.harris_strerror(rc)
            need = gpu.harris_grouped_workspace_bytes(grouping, B, H, W)
            ws = torch.empty(need // 4, device="cuda")
            ref = torch.full((B, H - 4, W - 4), float("nan"), device="cuda")
            rc = lib.harris_coarsity_grouped(ctypes.c_void_p(src.data_ptr()), dtype, B, H, W, K, scale, window, grouping,
                                             ctypes.c_void_p(ws.data_ptr()), need, ctypes.c_void_p(ref.data_ptr()), stream)
            assert rc == 0, gpu.harris_strerror(rc)
            torch.cuda.synchronize()
            g, r = got.cpu().numpy(), ref.cpu().numpy()
            assert np.array_equal(g, r)
            want = oracle.harris(rgb, K, scale, window, nthreads=4)
            assert float(np.abs(g - want).max()) <= 1e-4 * float(np.abs(want).max()) + 1e-6


def test_static_scratch_at_its_limit_and_beyond(gpu, oracle):
    import torch
    say("case static scratch: one 1536x2560 image, grouping 2 (62.8 of 64 MiB), then grouping 1 refused")
    rgb = hi.make("noise_f32_1536x2560")
    src = torch.from_numpy(rgb).cuda()
    out = torch.empty((1, 1532, 2556), device="cuda")
    gpu.harris_coarsity_grouped_static(src, out, K, grouping=2)
    fused = gpu.harris_coarsity(src, K)
    torch.cuda.synchronize()
    assert float((out - fused).abs().max()) <= 1e-4 * float(fused.abs().max()) + 1e-6
    with pytest.raises(gpu.HarrisError) as e:
        gpu.harris_coarsity_grouped_static(src, out, K, grouping=1)
    assert e.value.status == -5
    gpu.harris_coarsity_grouped_static(src, out, K, grouping=4)            # the fused kernel: no intermediates, any size
    torch.cuda.synchronize()
    assert torch.equal(out, fused)
