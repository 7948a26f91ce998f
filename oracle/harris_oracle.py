"""ctypes front end of the CPU oracle (oracle/harris_ref.cpp): test infrastructure only.

Argument marshalling and nothing else: every number comes out of the C++ file.
The shared object is compiled here with g++ when it is missing or older than
its source (two seconds), so CPU-only test runs need no separate build step.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "harris_ref.cpp")
_LIB = os.path.join(_HERE, "libharris_ref.so")
# -ffp-contract=off: no fused multiply-add, so the f32 instantiation rounds after
# every operation exactly as written.
_CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread"]

_lib = None


def build(force: bool = False) -> str:
    """Compile oracle/harris_ref.cpp into oracle/libharris_ref.so; return its path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["g++", *_CXXFLAGS, _SRC, "-o", tmp], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        ci, cf, cd = ctypes.c_int, ctypes.c_float, ctypes.c_double
        for name, inp, outp in (("harris_ref_f32", _f32p, _f32p), ("harris_ref_u8_f32", _u8p, _f32p),
                                ("harris_ref_f64", _f32p, _f64p), ("harris_ref_u8_f64", _u8p, _f64p)):
            fn = getattr(lib, name)
            fn.argtypes = [inp, ci, ci, ci, cf, cf, ci, outp, ci]
            fn.restype = ci
        for sfx, p, real in (("f32", _f32p, cf), ("f64", _f64p, cd)):
            getattr(lib, "harris_ref_gray_" + sfx).argtypes = [p, ci, ci, p]
            getattr(lib, "harris_ref_conv3x3_" + sfx).argtypes = [p, ci, ci, p, p]
            getattr(lib, "harris_ref_sobel_" + sfx).argtypes = [p, ci, ci, real, ci, p]
            getattr(lib, "harris_ref_mul_" + sfx).argtypes = [p, p, ci, ci, p]
            getattr(lib, "harris_ref_sum3x3_" + sfx).argtypes = [p, ci, ci, p]
            getattr(lib, "harris_ref_coarsity_" + sfx).argtypes = [p, p, p, ci, ci, real, p]
            for stage in ("gray", "conv3x3", "sobel", "mul", "sum3x3", "coarsity"):
                getattr(lib, "harris_ref_%s_%s" % (stage, sfx)).restype = None
        for name in ("harris_ref_round_binary16", "harris_ref_round_bfloat16"):
            getattr(lib, name).argtypes = [_f32p, ctypes.c_longlong, ctypes.POINTER(ctypes.c_uint16)]
            getattr(lib, name).restype = None
        lib.harris_ref_quantize_u8.argtypes = [_f32p, ctypes.c_longlong, cf, cf, _u8p]
        lib.harris_ref_quantize_u8.restype = None
        lib.harris_ref_hardware_threads.restype = ci
        _lib = lib
    return _lib


def hardware_threads() -> int:
    return int(_load().harris_ref_hardware_threads())


def _ptr(a: np.ndarray):
    return a.ctypes.data_as({np.dtype(np.float32): _f32p, np.dtype(np.float64): _f64p,
                             np.dtype(np.uint8): _u8p}[a.dtype])


def _sfx(dtype) -> str:
    return {np.dtype(np.float32): "f32", np.dtype(np.float64): "f64"}[np.dtype(dtype)]


def harris(rgb: np.ndarray, k: float = 0.04, sobel_scale: float = 1.0, window: int = 0,
           precision: str = "f32", nthreads: int = 1) -> np.ndarray:
    """Harris coarsity of rgb[batch][3][H][W] (float32 or uint8) -> [batch][H-4][W-4].

    precision "f32": float32 arithmetic and result (the oracle); "f64": the same
    code in double (the referee).  A 3-D input is taken as one image and a 2-D
    result is returned.
    """
    lib = _load()
    single = rgb.ndim == 3
    a = np.ascontiguousarray(rgb[None] if single else rgb)
    if a.ndim != 4 or a.shape[1] != 3:
        raise ValueError("rgb must be [batch][3][H][W] or [3][H][W]")
    if a.dtype not in (np.float32, np.uint8):
        raise TypeError("rgb must be float32 or uint8")
    B, _, H, W = a.shape
    if H < 4 or W < 4:
        raise ValueError("H and W must be at least 4")
    out = np.zeros((B, H - 4, W - 4), dtype=np.float32 if precision == "f32" else np.float64)
    name = "harris_ref_%s%s" % ("u8_" if a.dtype == np.uint8 else "", precision)
    # Empty arrays have no usable data pointer; the C side never dereferences them.
    rc = getattr(lib, name)(_ptr(a), B, H, W, k, sobel_scale, window, _ptr(out) if out.size else None, nthreads)
    if rc != 0:
        raise RuntimeError("%s failed with status %d" % (name, rc))
    return out[0] if single else out


def gray(rgb: np.ndarray) -> np.ndarray:
    """Grayscale of one image [3][H][W] (float32 or float64)."""
    a = np.ascontiguousarray(rgb)
    _, H, W = a.shape
    out = np.empty((H, W), dtype=a.dtype)
    getattr(_load(), "harris_ref_gray_" + _sfx(a.dtype))(_ptr(a), H, W, _ptr(out))
    return out


def conv3x3(img: np.ndarray, weights: np.ndarray) -> np.ndarray:
    """3x3 correlation (valid region) of a 2-D image with a 3x3 weight matrix."""
    a = np.ascontiguousarray(img)
    w = np.ascontiguousarray(weights, dtype=a.dtype).reshape(9)
    H, W = a.shape
    out = np.empty((H - 2, W - 2), dtype=a.dtype)
    getattr(_load(), "harris_ref_conv3x3_" + _sfx(a.dtype))(_ptr(a), H, W, _ptr(w), _ptr(out))
    return out


def sobel(img: np.ndarray, which: str, scale: float = 1.0) -> np.ndarray:
    """Sobel stage: Sx ("x") or Sy ("y") of a 2-D gray image, weights times `scale`."""
    a = np.ascontiguousarray(img)
    H, W = a.shape
    out = np.empty((H - 2, W - 2), dtype=a.dtype)
    getattr(_load(), "harris_ref_sobel_" + _sfx(a.dtype))(_ptr(a), H, W, scale, 0 if which == "x" else 1, _ptr(out))
    return out


def mul(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Products: pointwise product."""
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b, dtype=a.dtype)
    out = np.empty_like(a)
    getattr(_load(), "harris_ref_mul_" + _sfx(a.dtype))(_ptr(a), _ptr(b), a.shape[0], a.shape[1], _ptr(out))
    return out


def sum3x3(img: np.ndarray) -> np.ndarray:
    """Window sums: unweighted 3x3 sums (valid region)."""
    a = np.ascontiguousarray(img)
    H, W = a.shape
    out = np.empty((H - 2, W - 2), dtype=a.dtype)
    getattr(_load(), "harris_ref_sum3x3_" + _sfx(a.dtype))(_ptr(a), H, W, _ptr(out))
    return out


def coarsity(sxx: np.ndarray, sxy: np.ndarray, syy: np.ndarray, k: float) -> np.ndarray:
    """Coarsity: det - k * trace^2 from the three structure-tensor sums."""
    sxx = np.ascontiguousarray(sxx)
    sxy = np.ascontiguousarray(sxy, dtype=sxx.dtype)
    syy = np.ascontiguousarray(syy, dtype=sxx.dtype)
    out = np.empty_like(sxx)
    getattr(_load(), "harris_ref_coarsity_" + _sfx(sxx.dtype))(_ptr(sxx), _ptr(sxy), _ptr(syy),
                                                              sxx.shape[0], sxx.shape[1], k, _ptr(out))
    return out


def round_to_16bit(values: np.ndarray, fmt: str) -> np.ndarray:
    """float32 array -> bit patterns (uint16, same shape) of the nearest binary16 ("f16") or
    bfloat16 ("bf16") values: round to nearest, ties to even, overflow to infinity."""
    a = np.ascontiguousarray(values, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    fn = {"f16": "harris_ref_round_binary16", "bf16": "harris_ref_round_bfloat16"}[fmt]
    getattr(_load(), fn)(_ptr(a), a.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    return out


def quantize_u8(values: np.ndarray, scale: float, offset: float) -> np.ndarray:
    """float32 array -> uint8 codes clamp(rint(fma(v, scale, offset)), 0, 255), same shape."""
    a = np.ascontiguousarray(values, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint8)
    _load().harris_ref_quantize_u8(_ptr(a), a.size, scale, offset, _ptr(out))
    return out


def max_trace_squared(rgb: np.ndarray, sobel_scale: float = 1.0, window: int = 0) -> float:
    """Largest (Sxx + Syy)^2 over all images of rgb[batch][3][H][W], from the float64 stages above.

    Not a result anybody is checked against: the scale of the rounding diagnostic.  Every term of
    the coarsity is bounded by trace^2, so float32 rounding of a correct implementation stays
    within a few eps * trace^2, whatever the cancellation in det."""
    a = rgb[None] if rgb.ndim == 3 else rgb
    binomial = np.array([[1, 2, 1], [2, 4, 2], [1, 2, 1]], dtype=np.float64)
    worst = 0.0
    for img in a:
        f = img.astype(np.float64)
        if img.dtype == np.uint8:
            f = f / 255.0
        g = gray(f)
        ix, iy = sobel(g, "x", sobel_scale), sobel(g, "y", sobel_scale)
        if window == 0:
            tr = sum3x3(mul(ix, ix)) + sum3x3(mul(iy, iy))
        else:
            tr = conv3x3(mul(ix, ix), binomial) + conv3x3(mul(iy, iy), binomial)
        if tr.size:
            worst = max(worst, float(tr.max()) ** 2)
    return worst
