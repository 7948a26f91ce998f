"""Seeded synthetic RGB images for the Harris coarsity pipeline.

This module only *makes inputs*.  It holds none of the Harris arithmetic and is
the one piece of code that both the CPU oracle's tests and the GPU path's tests
and benchmark import, so that both sides see byte-identical images.

The thesis measures on two photographs (a 1536x2560 one from the Halide
repository and a 4256x2832 one from the PolyMage repository, section 4.4
"Experimental Setup").  Neither is available offline, so the images made here
stand in for them: same shapes, same planar float32 layout, same [0, 1] value
range; plus three further workloads (a tiny one, a batch with real corners, and
a large uint8 one).

Random numbers come from a counter-based generator written out here
(SplitMix64, Steele/Lea/Flood 2014: a Weyl sequence with increment
0x9E3779B97F4A7C15 followed by the 64-bit finaliser), so that the value of the
i-th sample of a stream depends only on (seed, stream, i), not on a library's
RNG state or version.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22  # samples generated per numpy pass (bounds temporary memory)


def _mix64(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function on an array of uint64 states."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_base(seed: int, stream: int) -> np.uint64:
    """Starting state of one (seed, stream) sequence."""
    s = np.array([(int(seed) * 0x100000001B3 + int(stream) * 0xD1342543DE82EF95 + 0x632BE59BD9B4E019)
                  & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    return _mix64(s)[0]


def raw_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """`count` 64-bit outputs of stream (seed, stream), beginning at index `start`."""
    with np.errstate(over="ignore"):
        base = _stream_base(seed, stream)
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix64(base + idx * _GOLDEN)


def uniform_f32(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """Uniform float32 in [0, 1): the top 24 bits of each output over 2**24 (exact in f32)."""
    out = np.empty(count, dtype=np.float32)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        z = raw_u64(seed, stream, start + lo, n)
        out[lo:lo + n] = (z >> np.uint64(40)).astype(np.float32) * np.float32(1.0 / (1 << 24))
    return out


def uniform_u8(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """Uniform integers 0..255: the top byte of each output."""
    out = np.empty(count, dtype=np.uint8)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        z = raw_u64(seed, stream, start + lo, n)
        out[lo:lo + n] = (z >> np.uint64(56)).astype(np.uint8)
    return out


def normal_f32(seed: int, stream: int, count: int, sigma: float, start: int = 0) -> np.ndarray:
    """N(0, sigma**2) samples by the Box-Muller transform, one sample per output word.

    The high 24 bits give u1 in (0, 1], the next 24 bits give u2 in [0, 1);
    sample = sigma * sqrt(-2 ln u1) * cos(2 pi u2).
    """
    out = np.empty(count, dtype=np.float32)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        z = raw_u64(seed, stream, start + lo, n)
        u1 = ((z >> np.uint64(40)).astype(np.float64) + 1.0) * (1.0 / (1 << 24))
        u2 = ((z >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) * (1.0 / (1 << 24))
        out[lo:lo + n] = (sigma * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    return out


# ----------------------------------------------------------------------------
# The five workloads.  Every function takes the shape as arguments so that tests
# can make reduced-size images with the same recipe; defaults are the full sizes.
# All results are C-contiguous, planar: [batch][3][H][W].
# ----------------------------------------------------------------------------

def white_noise_f32(seed: int, batch: int, H: int, W: int) -> np.ndarray:
    """i.i.d. uniform [0, 1) float32 in every channel."""
    return uniform_f32(seed, 0, batch * 3 * H * W).reshape(batch, 3, H, W)


def white_noise_u8(seed: int, batch: int, H: int, W: int) -> np.ndarray:
    """i.i.d. uniform integers 0..255 in every channel."""
    return uniform_u8(seed, 0, batch * 3 * H * W).reshape(batch, 3, H, W)


def smooth_blobs_f32(seed: int, batch: int, H: int, W: int, n_blobs: int = 32,
                     sigma_lo: float = 20.0, sigma_hi: float = 200.0,
                     noise_sigma: float = 0.02) -> np.ndarray:
    """Smooth, photo-like content: a sum of isotropic 2-D Gaussian blobs plus weak noise.

    Per image and blob: centre uniform over the image, sigma uniform in
    [sigma_lo, sigma_hi] pixels, one amplitude per colour channel uniform in
    [0, 1).  A Gaussian blob is an outer product of a column profile and a row
    profile, so each channel is assembled as one small matrix product.
    Gaussian noise N(0, noise_sigma**2) is added per sample and the result is
    clipped to [0, 1].
    """
    out = np.empty((batch, 3, H, W), dtype=np.float32)
    ys = np.arange(H, dtype=np.float64)[:, None]
    xs = np.arange(W, dtype=np.float64)[None, :]
    for b in range(batch):
        p = uniform_f32(seed, 1, 6 * n_blobs, start=b * 6 * n_blobs).astype(np.float64).reshape(n_blobs, 6)
        cy = p[:, 0] * H
        cx = p[:, 1] * W
        sg = sigma_lo + p[:, 2] * (sigma_hi - sigma_lo)
        amp = p[:, 3:6]
        ey = np.exp(-0.5 * ((ys - cy[None, :]) / sg[None, :]) ** 2)          # H x n_blobs
        ex = np.exp(-0.5 * ((xs - cx[:, None]) / sg[:, None]) ** 2)          # n_blobs x W
        for c in range(3):
            img = (ey * amp[None, :, c]) @ ex
            noise = normal_f32(seed, 2, H * W, noise_sigma, start=(b * 3 + c) * H * W).reshape(H, W)
            out[b, c] = np.clip(img.astype(np.float32) + noise, 0.0, 1.0)
    return out


def rectangles_f32(seed: int, batch: int, H: int, W: int, n_rect: int = 200,
                   noise_sigma: float = 0.05) -> np.ndarray:
    """Piecewise-constant content with real corners: overlapping filled rectangles.

    Per image: a uniform random background colour, then n_rect axis-aligned
    rectangles painted in order (later ones cover earlier ones), each with width
    uniform in [8, max(9, W/4)), height uniform in [8, max(9, H/4)), top-left
    corner uniform over the image (clipped at the borders) and a uniform random
    colour; then N(0, noise_sigma**2) noise per sample, clipped to [0, 1].
    """
    out = np.empty((batch, 3, H, W), dtype=np.float32)
    per = 3 + 7 * n_rect
    for b in range(batch):
        p = uniform_f32(seed, 1, per, start=b * per)
        img = out[b]
        img[:] = p[0:3, None, None]
        q = p[3:].reshape(n_rect, 7)
        for r in range(n_rect):
            w = 8 + int(q[r, 0] * (max(9, W // 4) - 8))
            h = 8 + int(q[r, 1] * (max(9, H // 4) - 8))
            x0 = int(q[r, 2] * W)
            y0 = int(q[r, 3] * H)
            img[:, y0:min(H, y0 + h), x0:min(W, x0 + w)] = q[r, 4:7, None, None]
        for c in range(3):
            noise = normal_f32(seed, 2, H * W, noise_sigma, start=(b * 3 + c) * H * W).reshape(H, W)
            img[c] = np.clip(img[c] + noise, 0.0, 1.0)
    return out


#: name -> (generator, seed, batch, H, W, dtype string); index = position in the workload list.
WORKLOADS = {
    "tiny_f32_64x96":        (white_noise_f32, 0, 1, 64, 96, "f32"),
    "noise_f32_1536x2560":   (white_noise_f32, 1, 1, 1536, 2560, "f32"),
    "blobs_f32_2832x4256":   (smooth_blobs_f32, 2, 1, 2832, 4256, "f32"),
    "rects_f32_64x1080x1920": (rectangles_f32, 3, 64, 1080, 1920, "f32"),
    "noise_u8_8192x8192":    (white_noise_u8, 4, 1, 8192, 8192, "u8"),
}


def make(name: str, batch: int | None = None, H: int | None = None, W: int | None = None, **recipe) -> np.ndarray:
    """Build workload `name`; batch/H/W override the full size (same recipe, same seed).

    Further keyword arguments go to the generator (e.g. a narrower sigma range
    for a reduced-size blob image, so that it does not saturate).
    """
    gen, seed, b0, h0, w0, _ = WORKLOADS[name]
    return gen(seed, batch or b0, H or h0, W or w0, **recipe)
