"""Pins for the CPU oracle: facts fixed by the thesis's definition and by mathematics,
none of which is computed by the oracle itself (and none by the GPU path).

The thesis prints no worked numeric example for Harris (its only printed check is
a PSNR above 170 dB against Halide's output, section 4.4), so the pins are closed
forms, hand expansions, library routines and exact invariants.
"""
import os

import numpy as np
import pytest
import scipy.ndimage
import scipy.signal

import harris_inputs as hi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
K = 0.04
KF = float(np.float32(0.04))          # the value the f32 interface actually carries
S12 = float(np.float32(1.0) / np.float32(12.0))


def gray_to_rgb(g):
    """An RGB image whose three channels all equal g (gray = (0.299+0.587+0.114) g)."""
    return np.ascontiguousarray(np.broadcast_to(g.astype(np.float32)[None], (3,) + g.shape))


def rel(a, b):
    return np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)).max() / max(np.abs(b).max(), 1e-300)


# ---------------------------------------------------------------- shapes / degenerate sizes

def test_output_is_four_smaller(oracle):
    # Section 4.2.2: input 3.(n+4).(m+4) -> output n.m ; one 3x3 stage maps 8x8 to 6x6.
    rgb = hi.white_noise_f32(11, 2, 9, 13)
    assert oracle.harris(rgb).shape == (2, 5, 9)
    assert oracle.sum3x3(np.zeros((8, 8), np.float32)).shape == (6, 6)
    assert oracle.harris(hi.white_noise_f32(1, 1, 4, 9)).shape == (1, 0, 5)
    assert oracle.harris(hi.white_noise_f32(1, 1, 7, 4)).shape == (1, 3, 0)


# ---------------------------------------------------------------- P1 constant images

@pytest.mark.parametrize("scale", [1.0, S12])
@pytest.mark.parametrize("window", [0, 1])
def test_constant_image_is_exactly_zero(oracle, scale, window):
    rgb = np.empty((1, 3, 12, 17), np.float32)
    rgb[0, 0], rgb[0, 1], rgb[0, 2] = 0.8125, 0.3, 0.61
    for prec in ("f32", "f64"):
        out = oracle.harris(rgb, K, scale, window, precision=prec)
        assert out.shape == (1, 8, 13)
        assert np.all(out == 0.0)
    u8 = np.empty((1, 3, 9, 9), np.uint8)
    u8[0, 0], u8[0, 1], u8[0, 2] = 200, 17, 99
    assert np.all(oracle.harris(u8, K, scale, window) == 0.0)


# ---------------------------------------------------------------- P2 ramps (closed forms)

def test_sobel_on_ramps_stage_level(oracle):
    # gray = a*x + b*y + c  =>  Sx = 8a, Sy = 8b exactly (dyadic a, b, c).
    a, b, c = 2.0 ** -6, 3 * 2.0 ** -7, 0.25
    y, x = np.mgrid[0:10, 0:14]
    g = (a * x + b * y + c).astype(np.float32)
    assert np.all(oracle.sobel(g, "x") == np.float32(8 * a))
    assert np.all(oracle.sobel(g, "y") == np.float32(8 * b))
    # the thesis's 1/12 scale: 8a/12 up to rounding of the weights
    assert rel(oracle.sobel(g.astype(np.float64), "x", 1.0 / 12), np.full((8, 12), 8 * a / 12)) < 1e-14


@pytest.mark.parametrize("axis", ["horizontal", "vertical"])
def test_pure_ramp_closed_form(oracle, axis):
    # Horizontal ramp: Iy = 0, Ix = 8a, Sxx = 9*Ix^2, det = 0, out = -k*(9*Ix^2)^2.
    a = 2.0 ** -8
    H, W = 11, 15
    y, x = np.mgrid[0:H, 0:W]
    g = (a * (x if axis == "horizontal" else y) + 0.125)
    expect = -KF * (9.0 * (8 * a) ** 2) ** 2
    o64 = oracle.harris(gray_to_rgb(g), KF, precision="f64")
    o32 = oracle.harris(gray_to_rgb(g), KF, precision="f32")
    assert o64.shape == (H - 4, W - 4)
    # end to end through RGB: gray = (0.299f+0.587f+0.114f)*g, one ulp of f32 from g
    assert rel(o64, np.full_like(o64, expect)) < 1e-6
    assert rel(o32, np.full_like(o64, expect)) < 1e-5
    # entered after grayscale the f64 result is exact to double rounding
    gx = oracle.sobel(g, "x"); gy = oracle.sobel(g, "y")
    sxx, sxy, syy = (oracle.sum3x3(oracle.mul(p, q)) for p, q in ((gx, gx), (gx, gy), (gy, gy)))
    assert np.all((syy if axis == "horizontal" else sxx) == 0) and np.all(sxy == 0)
    assert rel(oracle.coarsity(sxx, sxy, syy, KF), np.full((H - 4, W - 4), expect)) < 1e-15


def test_affine_image_closed_form(oracle):
    # gray = a*x + b*y + c: Ix = 8a, Iy = 8b, S** = 9*64*{a^2, ab, b^2}, det = 0,
    # out = -k * (576 (a^2 + b^2))^2.  With a != b this separates Sx from Sy and
    # catches a missing transpose or a sign error in the cross term.
    a, b = 0.01, -0.023
    y, x = np.mgrid[0:9, 0:12]
    g = a * x + b * y + 0.4
    gx, gy = oracle.sobel(g, "x"), oracle.sobel(g, "y")
    assert rel(gx, np.full_like(gx, 8 * a)) < 1e-12 and rel(gy, np.full_like(gy, 8 * b)) < 1e-12
    sxy = oracle.sum3x3(oracle.mul(gx, gy))
    assert rel(sxy, np.full_like(sxy, 576 * a * b)) < 1e-12          # negative: sign kept
    out = oracle.harris(gray_to_rgb(g), KF, precision="f64")
    assert rel(out, np.full_like(out, -KF * (576 * (a * a + b * b)) ** 2)) < 2e-5


# ---------------------------------------------------------------- P9 step edge, corner

def test_vertical_step_edge_closed_form(oracle):
    # gray = 0 left of column c, d right of it: Ix = 4d on the two columns next to the
    # edge, Iy = 0.  A 3x3 window holding both columns has Sxx = 6*16 d^2, one column
    # 3*16 d^2, none 0; det = 0 so out = -k*Sxx^2 <= 0 (an edge is never a corner).
    d, c, H, W = 0.5, 7, 9, 16
    g = np.zeros((H, W)); g[:, c:] = d
    out = oracle.harris(gray_to_rgb(g), KF, precision="f64")
    # output column x covers Sobel centres x+1..x+3 ; edge columns are c-1 and c
    expect = np.zeros(W - 4)
    for xo in range(W - 4):
        n_edge_cols = len({c - 1, c} & {xo + 1, xo + 2, xo + 3})
        expect[xo] = -KF * (3 * n_edge_cols * 16 * d * d) ** 2
    assert rel(out, np.broadcast_to(expect, out.shape)) < 1e-6
    assert np.all(out <= 0)


def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def test_hand_computed_corner_example(oracle):
    gold = _read_golden("quadrant_corner_5x5.txt")
    g = np.zeros((5, 5)); g[2:, 2:] = 1.0
    gx, gy = oracle.sobel(g, "x"), oracle.sobel(g, "y")
    assert np.array_equal(np.abs(gx), [[1, 1, 0], [3, 3, 0], [4, 4, 0]])
    assert np.array_equal(np.abs(gy), [[1, 3, 4], [1, 3, 4], [0, 0, 0]])
    assert oracle.sum3x3(oracle.mul(gx, gx))[0, 0] == gold["Sxx"]
    assert oracle.sum3x3(oracle.mul(gy, gy))[0, 0] == gold["Syy"]
    assert oracle.sum3x3(oracle.mul(gx, gy))[0, 0] == gold["Sxy"]
    o1 = oracle.harris(gray_to_rgb(g), KF, 1.0, precision="f64")
    o12 = oracle.harris(gray_to_rgb(g), KF, S12, precision="f64")
    assert o1.shape == (1, 1)
    assert abs(o1[0, 0] - gold["out_scale1"]) < 2e-6 * gold["out_scale1"]
    assert abs(o12[0, 0] - gold["out_scale12"]) < 2e-6 * gold["out_scale12"]
    assert abs(oracle.harris(gray_to_rgb(g), KF, 1.0)[0, 0] - gold["out_scale1"]) < 1e-5 * gold["out_scale1"]


def test_corner_is_positive_maximum_edges_negative(oracle):
    g = np.zeros((24, 24)); g[12:, 12:] = 0.75
    out = oracle.harris(gray_to_rgb(g), KF, precision="f64")
    yy, xx = np.unravel_index(np.argmax(out), out.shape)
    assert out.max() > 0 and abs(yy + 2 - 12) <= 1 and abs(xx + 2 - 12) <= 1
    assert out[18, 9] < 0 and out[9, 18] < 0 and out[2, 2] == 0     # on the two edges; flat area


# ---------------------------------------------------------------- P3 brute force, hand expansion

def _harris_by_hand(rgb, k, s, binomial=False):
    """Every output pixel from the 5x5 input patch by literal expansion, python floats."""
    _, H, W = rgb.shape
    g = [[float(np.float32(0.299)) * float(rgb[0, y, x])
          + float(np.float32(0.587)) * float(rgb[1, y, x])
          + float(np.float32(0.114)) * float(rgb[2, y, x]) for x in range(W)] for y in range(H)]
    out = [[0.0] * (W - 4) for _ in range(H - 4)]
    for y in range(H - 4):
        for x in range(W - 4):
            sxx = sxy = syy = 0.0
            for dy in range(3):
                for dx in range(3):
                    cy, cx = y + dy + 1, x + dx + 1          # Sobel centre in input coordinates
                    ix = s * (-g[cy - 1][cx - 1] + g[cy - 1][cx + 1]
                              - 2 * g[cy][cx - 1] + 2 * g[cy][cx + 1]
                              - g[cy + 1][cx - 1] + g[cy + 1][cx + 1])
                    iy = s * (-g[cy - 1][cx - 1] - 2 * g[cy - 1][cx] - g[cy - 1][cx + 1]
                              + g[cy + 1][cx - 1] + 2 * g[cy + 1][cx] + g[cy + 1][cx + 1])
                    wgt = (2 - abs(dy - 1)) * (2 - abs(dx - 1)) if binomial else 1
                    sxx += wgt * ix * ix
                    sxy += wgt * ix * iy
                    syy += wgt * iy * iy
            out[y][x] = (sxx * syy - sxy * sxy) - k * (sxx + syy) * (sxx + syy)
    return np.array(out)


@pytest.mark.parametrize("scale", [1.0, S12])
@pytest.mark.parametrize("window", [0, 1])
def test_brute_force_6x6(oracle, scale, window):
    rgb = hi.white_noise_f32(123, 1, 6, 6)[0]
    hand = _harris_by_hand(rgb, KF, scale, binomial=bool(window))
    assert hand.shape == (2, 2)
    assert rel(oracle.harris(rgb, KF, scale, window, precision="f64"), hand) < 1e-12
    assert rel(oracle.harris(rgb, KF, scale, window, precision="f32"), hand) < 1e-5


def test_brute_force_ragged_and_u8(oracle):
    rgb = hi.white_noise_f32(5, 1, 7, 9)[0]
    assert rel(oracle.harris(rgb, 0.06, 1.0, precision="f64"), _harris_by_hand(rgb, float(np.float32(0.06)), 1.0)) < 1e-12
    u8 = hi.white_noise_u8(6, 1, 6, 8)[0]
    asfloat = (u8.astype(np.float32) / np.float32(255.0))
    assert rel(oracle.harris(u8, KF, precision="f64"), _harris_by_hand(asfloat.astype(np.float64), KF, 1.0)) < 1e-6
    # the 8-bit entry is exactly the float entry applied to u/255 rounded to f32
    assert np.array_equal(oracle.harris(u8, KF), oracle.harris(asfloat, KF))


# ---------------------------------------------------------------- library cross-checks per stage

def test_stages_against_library_routines(oracle):
    rgb = hi.white_noise_f32(77, 1, 21, 33)[0].astype(np.float64)
    w = np.array([np.float32(0.299), np.float32(0.587), np.float32(0.114)], np.float64)
    g = oracle.gray(rgb)
    assert rel(g, np.tensordot(w, rgb, axes=(0, 0))) < 1e-15
    kx = np.array([[-1, 0, 1], [-2, 0, 2], [-1, 0, 1]], np.float64)
    gx, gy = oracle.sobel(g, "x"), oracle.sobel(g, "y")
    assert rel(gx, scipy.signal.correlate2d(g, kx, mode="valid")) < 1e-13
    assert rel(gy, scipy.signal.correlate2d(g, kx.T, mode="valid")) < 1e-13
    # textbook Sobel from the imaging library (derivative along one axis, [1,2,1] along the other)
    assert rel(gx, scipy.ndimage.sobel(g, axis=1)[1:-1, 1:-1]) < 1e-13
    assert rel(gy, scipy.ndimage.sobel(g, axis=0)[1:-1, 1:-1]) < 1e-13
    p = oracle.mul(gx, gy)
    assert np.array_equal(p, gx * gy)
    assert rel(oracle.sum3x3(p), scipy.signal.correlate2d(p, np.ones((3, 3)), mode="valid")) < 1e-13
    assert rel(oracle.sum3x3(p), 9 * scipy.ndimage.uniform_filter(p, 3)[1:-1, 1:-1]) < 1e-12
    wts = np.arange(1.0, 10.0).reshape(3, 3)            # asymmetric: catches a flipped or transposed window
    assert rel(oracle.conv3x3(g, wts), scipy.signal.correlate2d(g, wts, mode="valid")) < 1e-13


def test_whole_pipeline_against_library_composition(oracle):
    rgb = hi.rectangles_f32(9, 1, 48, 64)[0]
    w = np.array([np.float32(0.299), np.float32(0.587), np.float32(0.114)], np.float64)
    g = np.tensordot(w, rgb.astype(np.float64), axes=(0, 0))
    ix = scipy.ndimage.sobel(g, axis=1)[1:-1, 1:-1]
    iy = scipy.ndimage.sobel(g, axis=0)[1:-1, 1:-1]
    box = lambda a: scipy.signal.correlate2d(a, np.ones((3, 3)), mode="valid")
    sxx, sxy, syy = box(ix * ix), box(ix * iy), box(iy * iy)
    lib = sxx * syy - sxy * sxy - KF * (sxx + syy) ** 2
    assert rel(oracle.harris(rgb, KF, precision="f64"), lib) < 1e-12
    assert rel(oracle.harris(rgb, KF, precision="f32"), lib) < 1e-5
    binom = np.outer([1, 2, 1], [1, 2, 1]).astype(np.float64)
    bw = lambda a: scipy.signal.correlate2d(a, binom, mode="valid")
    sxx, sxy, syy = bw(ix * ix), bw(ix * iy), bw(iy * iy)
    lib = sxx * syy - sxy * sxy - KF * (sxx + syy) ** 2
    assert rel(oracle.harris(rgb, KF, 1.0, 1, precision="f64"), lib) < 1e-12


def test_sobel_pair_equals_conv3x3_with_the_rise_matrices(oracle):
    # Listing "High-level stencil operators in Rise": Sx = conv3x3([-1 0 1; -2 0 2; -1 0 1]/12),
    # Sy = conv3x3 of its transpose; the oracle's Sobel stage uses the Halide term order.
    g = hi.uniform_f32(31, 0, 17 * 22).reshape(17, 22).astype(np.float64)
    kx = np.array([[-1, 0, 1], [-2, 0, 2], [-1, 0, 1]], np.float64)
    for s in (1.0, 1.0 / 12):
        assert rel(oracle.sobel(g, "x", s), oracle.conv3x3(g, kx * s)) < 1e-13
        assert rel(oracle.sobel(g, "y", s), oracle.conv3x3(g, kx.T * s)) < 1e-13


def test_unweighted_sum_equals_conv_with_ones_bitwise(oracle):
    p = hi.uniform_f32(3, 0, 20 * 31).reshape(20, 31)
    assert np.array_equal(oracle.sum3x3(p), oracle.conv3x3(p, np.ones((3, 3), np.float32)))


# ---------------------------------------------------------------- P8 separable identities

def test_separable_identities(oracle):
    g = hi.uniform_f32(4, 0, 19 * 23).reshape(19, 23).astype(np.float64)
    smooth = g[:-2] + 2 * g[1:-1] + g[2:]            # [1,2,1] down the columns
    diff = g[2:] - g[:-2]                            # [-1,0,1] down the columns
    assert rel(oracle.sobel(g, "x"), smooth[:, 2:] - smooth[:, :-2]) < 1e-13
    assert rel(oracle.sobel(g, "y"), diff[:, :-2] + 2 * diff[:, 1:-1] + diff[:, 2:]) < 1e-13
    v = g[:-2] + g[1:-1] + g[2:]
    assert rel(oracle.sum3x3(g), v[:, :-2] + v[:, 1:-1] + v[:, 2:]) < 1e-13


# ---------------------------------------------------------------- symmetries and invariants

def test_transpose_symmetry(oracle):
    rgb = hi.white_noise_f32(21, 1, 37, 53)
    t = np.ascontiguousarray(rgb.transpose(0, 1, 3, 2))
    a64 = oracle.harris(rgb, KF, precision="f64"); b64 = oracle.harris(t, KF, precision="f64")
    assert rel(b64.transpose(0, 2, 1), a64) < 1e-12
    assert rel(oracle.harris(t, KF).transpose(0, 2, 1), oracle.harris(rgb, KF)) < 1e-5


def test_flip_symmetry(oracle):
    rgb = hi.white_noise_f32(22, 1, 30, 41)
    a = oracle.harris(rgb, KF, precision="f64")
    for ax in (2, 3, (2, 3)):
        f = np.ascontiguousarray(np.flip(rgb, ax))
        oax = tuple(i - 1 for i in (ax if isinstance(ax, tuple) else (ax,)))
        assert rel(np.flip(oracle.harris(f, KF, precision="f64"), oax), a) < 1e-12


def test_power_of_two_homogeneity_is_bit_exact(oracle):
    # harris(2^p * RGB) = 2^(4p) * harris(RGB): scaling by a power of two commutes with
    # every rounding, so the f32 results must agree bit for bit.
    rgb = hi.white_noise_f32(23, 1, 25, 36)
    base = oracle.harris(rgb, KF)
    for p in (-3, 2):
        scaled = oracle.harris(rgb * np.float32(2.0 ** p), KF)
        assert np.array_equal(scaled, base * np.float32(2.0 ** (4 * p)))


def test_offset_invariance(oracle):
    rgb = hi.smooth_blobs_f32(24, 1, 40, 56, sigma_lo=3, sigma_hi=12, noise_sigma=0.0) * np.float32(0.5)
    a = oracle.harris(rgb, KF, precision="f64")
    b = oracle.harris(rgb + np.float32(0.25), KF, precision="f64")
    assert rel(b, a) < 1e-4


def test_scale_relation_between_sobel_variants(oracle):
    rgb = hi.white_noise_f32(25, 1, 32, 48)
    a = oracle.harris(rgb, KF, 1.0, precision="f64")
    b = oracle.harris(rgb, KF, S12, precision="f64")
    assert rel(b * 20736.0, a) < 1e-6            # 12^4; S12 is 1/12 rounded to f32
    assert rel(oracle.harris(rgb, KF, S12) * 20736.0, a) < 1e-5


def test_kappa_enters_linearly(oracle):
    rgb = hi.white_noise_f32(26, 1, 16, 20)
    o0 = oracle.harris(rgb, 0.0, precision="f64")
    o1 = oracle.harris(rgb, 0.0625, precision="f64")
    o2 = oracle.harris(rgb, 0.125, precision="f64")
    assert rel(o2 - o0, 2 * (o1 - o0)) < 1e-12 and np.all(o1 <= o0)   # -k*trace^2 <= 0


# ---------------------------------------------------------------- precision, batching, threads

@pytest.mark.parametrize("name,kw", [
    ("tiny_f32_64x96", {}),
    ("noise_f32_1536x2560", dict(H=96, W=160)),
    ("blobs_f32_2832x4256", dict(H=177, W=266, sigma_lo=2, sigma_hi=13)),
    ("rects_f32_64x1080x1920", dict(batch=2, H=135, W=240)),
    ("noise_u8_8192x8192", dict(H=128, W=128)),
])
def test_f32_oracle_against_f64_referee(oracle, name, kw):
    rgb = hi.make(name, **kw)
    o32 = oracle.harris(rgb, KF, precision="f32")
    o64 = oracle.harris(rgb, KF, precision="f64")
    assert rel(o32, o64) < 1e-5


def test_batch_and_threads_do_not_change_results(oracle):
    rgb = hi.rectangles_f32(8, 3, 33, 47)
    whole = oracle.harris(rgb, KF, nthreads=1)
    for b in range(3):
        assert np.array_equal(whole[b], oracle.harris(rgb[b], KF))
    assert np.array_equal(whole, oracle.harris(rgb, KF, nthreads=5))
    assert np.array_equal(oracle.harris(rgb, KF, precision="f64", nthreads=4), oracle.harris(rgb, KF, precision="f64"))


# ---------------------------------------------------------------- rounding to 16-bit results

def test_rounding_to_binary16_and_bfloat16(oracle):
    # The oracle's rounding (written from the IEEE definition in double arithmetic) against two
    # library conversions that share nothing with it: numpy's float32 -> float16 and torch's
    # float32 -> bfloat16, both round-to-nearest-even.
    import torch
    f16 = lambda a: oracle.round_to_16bit(a, "f16")
    bf16 = lambda a: oracle.round_to_16bit(a, "bf16")
    rng = np.random.default_rng(7)
    x = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32).view(np.float32)
    x = x[~np.isnan(x)]                                       # every binade, both signs, subnormals, infinities
    with np.errstate(over="ignore"):
        assert np.array_equal(f16(x), x.astype(np.float16).view(np.uint16))
    assert np.array_equal(bf16(x), torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    # every tie of binary16: the midpoint of two neighbouring values goes to the one with an even fraction
    h = np.arange(0, 0x7c00, dtype=np.uint16)                 # all finite non-negative binary16 values
    lo = h[:-1].view(np.float16).astype(np.float64); hi_ = h[1:].view(np.float16).astype(np.float64)
    mid = ((lo + hi_) / 2).astype(np.float32)                 # exact in float32
    assert np.array_equal(mid.astype(np.float64), (lo + hi_) / 2)
    want = np.where(h[:-1] % 2 == 0, h[:-1], h[1:])
    assert np.array_equal(f16(mid), want) and np.array_equal(f16(-mid), want | 0x8000)
    # hand-picked values
    cases16 = [(1.0, 0x3c00), (-2.0, 0xc000), (65504.0, 0x7bff), (65519.996, 0x7bff), (65520.0, 0x7c00), (1e9, 0x7c00),
               (2.0 ** -24, 0x0001), (2.0 ** -25, 0x0000), (2.0 ** -25 * 1.0000002, 0x0001), (2.0 ** -14, 0x0400),
               (0.0, 0x0000), (-0.0, 0x8000), (float("inf"), 0x7c00), (float("-inf"), 0xfc00), (1.0 + 2.0 ** -11, 0x3c00),
               (1.0 + 3 * 2.0 ** -11, 0x3c02)]
    for v, bits in cases16:
        assert int(f16(np.array([v], dtype=np.float32))[0]) == bits, (v, hex(bits))
    cases_b = [(1.0, 0x3f80), (1.0 + 2.0 ** -8, 0x3f80), (1.0 + 3 * 2.0 ** -8, 0x3f82), (-1.5, 0xbfc0), (3.3895314e38, 0x7f7f),
               (3.4e38, 0x7f80), (0.0, 0x0000), (-0.0, 0x8000), (float("inf"), 0x7f80), (2.0 ** -133, 0x0001), (2.0 ** -134, 0x0000)]
    for v, bits in cases_b:
        assert int(bf16(np.array([v], dtype=np.float32))[0]) == bits, (v, hex(bits))
    nan = np.array([np.nan], dtype=np.float32)
    assert (int(f16(nan)[0]) & 0x7c00) == 0x7c00 and (int(f16(nan)[0]) & 0x03ff) != 0
    assert (int(bf16(nan)[0]) & 0x7f80) == 0x7f80 and (int(bf16(nan)[0]) & 0x007f) != 0


def test_quantisation_to_8_bit_codes(oracle):
    # Exact cases: v * scale + offset is representable, so the code is fixed by the definition:
    # ties go to the even integer, the range is clamped, NaN gives 0.
    q = lambda v, s, o: oracle.quantize_u8(np.array(v, dtype=np.float32), s, o).tolist()
    assert q([0.0, 0.25, 0.5, 0.75, 1.0, 1.25, 1.5, 2.5, 3.5, 254.5, 255.5, 300.0, -0.5, -3.0], 1.0, 0.0) == [0, 0, 0, 1, 1, 1, 2, 2, 4, 254, 255, 255, 0, 0]
    assert q([0.0, 1.0, -1.0, 63.75, -64.0, 1e30, -1e30], 2.0, 128.0) == [128, 130, 126, 255, 0, 255, 0]
    assert q([float("nan"), float("inf"), float("-inf")], 1.0, 0.0) == [0, 255, 0]
    # random values against the same formula in float64 (exact product, one rounding of the sum):
    # equal except where the sum lies within 1e-4 of a rounding border
    rng = np.random.default_rng(3)
    v = (rng.standard_normal(200000) * 60).astype(np.float32)
    for s, o in ((1.0, 128.0), (0.37, 17.5), (-2.0, 100.0)):
        t = v.astype(np.float64) * np.float64(np.float32(s)) + np.float64(np.float32(o))
        want = np.clip(np.rint(t), 0, 255).astype(np.uint8)
        got = oracle.quantize_u8(v, s, o)
        near_border = np.abs(t - np.floor(t) - 0.5) < 1e-4
        assert np.array_equal(got[~near_border], want[~near_border]) and np.all(np.abs(got.astype(int) - want.astype(int)) <= 1)
    # the multiply-add is rounded once: 4097 * 4097 = 16785409 is not a float32 (it would round to
    # 16785408), so with offset -16785400 the fused result is 9 and a separately rounded one 8
    assert float(np.float32(-16785400.0)) == -16785400.0
    assert oracle.quantize_u8(np.array([4097.0], dtype=np.float32), 4097.0, -16785400.0)[0] == 9


# ---------------------------------------------------------------- input generators (host logic)

def test_generators_are_deterministic_and_in_range():
    a = hi.make("tiny_f32_64x96"); b = hi.make("tiny_f32_64x96")
    assert a.dtype == np.float32 and a.shape == (1, 3, 64, 96) and np.array_equal(a, b)
    assert 0.0 <= a.min() and a.max() < 1.0 and abs(a.mean() - 0.5) < 0.02
    # counter-based: a later slice of a stream equals the same indices generated directly
    assert np.array_equal(hi.uniform_f32(9, 3, 100, start=50), hi.uniform_f32(9, 3, 150)[50:])
    assert not np.array_equal(hi.uniform_f32(9, 3, 64), hi.uniform_f32(9, 4, 64))
    n = hi.normal_f32(5, 0, 200000, 0.05)
    assert abs(n.mean()) < 1e-3 and abs(n.std() - 0.05) < 1e-3
    u = hi.make("noise_u8_8192x8192", H=64, W=64)
    assert u.dtype == np.uint8 and u.shape == (1, 3, 64, 64) and u.min() == 0 and u.max() == 255
    r = hi.make("rects_f32_64x1080x1920", batch=2, H=90, W=160)
    assert r.shape == (2, 3, 90, 160) and r.min() >= 0 and r.max() <= 1 and not np.array_equal(r[0], r[1])
    s = hi.make("blobs_f32_2832x4256", H=64, W=96, sigma_lo=2, sigma_hi=10)
    assert s.shape == (1, 3, 64, 96) and s.min() >= 0 and s.max() <= 1
