"""ctypes binding of libharris (include/harris.h, include/harris_tuning.h): argument marshalling only.

The functions have the names and argument order of the C entry points.  Images
are torch tensors on a ROCm device; their data pointers and the current HIP stream
are handed to the library unchanged.  There is no fallback: if the shared library
is missing the first call raises.
"""
from __future__ import annotations

import ctypes
import os

HARRIS_F32, HARRIS_U8 = 0, 1
HARRIS_WINDOW_BOX, HARRIS_WINDOW_BINOMIAL = 0, 1
HARRIS_SCHEDULE_BANDS, HARRIS_SCHEDULE_TILES = 1, 2
HARRIS_TUNE_NO_ALTERNATE, HARRIS_TUNE_NO_XCD_REMAP, HARRIS_TUNE_CACHED_LOADS, HARRIS_TUNE_STREAM_LOADS = 1, 2, 4, 8
HARRIS_TUNE_ALIGNED_STORES, HARRIS_TUNE_PLAIN_STORES, HARRIS_TUNE_KEEP_SHARED_ROWS, HARRIS_TUNE_FLAG_HANDOFF = 16, 32, 64, 128

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libharris.so")

#: every symbol include/harris.h and include/harris_tuning.h declare
EXPORTS = ("harris_coarsity", "harris_coarsity_u8", "harris_coarsity_ex", "harris_plan", "harris_plan_typed",
           "harris_coarsity_pitched", "harris_coarsity_typed", "harris_coarsity_quantized", "harris_coarsity_grouped",
           "harris_grouped_workspace_bytes", "harris_coarsity_grouped_static", "harris_probe_copy", "harris_probe_stream", "harris_strerror", "harris_version")
HARRIS_OUT_F32, HARRIS_OUT_F16, HARRIS_OUT_BF16, HARRIS_OUT_U8 = 0, 1, 2, 3


class HarrisError(RuntimeError):
    """A libharris entry point returned a status other than HARRIS_OK."""

    def __init__(self, status: int, message: str):
        super().__init__("libharris: %s (status %d)" % (message, status))
        self.status = status


class HarrisLayout(ctypes.Structure):
    """Mirror of `harris_layout`: pitches in elements."""
    _fields_ = [("rgb_row_pitch", ctypes.c_longlong), ("rgb_plane_pitch", ctypes.c_longlong),
                ("rgb_image_pitch", ctypes.c_longlong), ("out_row_pitch", ctypes.c_longlong),
                ("out_image_pitch", ctypes.c_longlong)]


class HarrisTuning(ctypes.Structure):
    """Mirror of `harris_tuning`."""
    _fields_ = [("schedule", ctypes.c_int), ("px", ctypes.c_int), ("rows", ctypes.c_int), ("prefetch", ctypes.c_int),
                ("waves_per_block", ctypes.c_int), ("flags", ctypes.c_uint), ("lds_kb", ctypes.c_int)]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libharris.so from the package directory and declare its prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libharris.so is not built (expected at %s). Build it with "
            "`python -m paper_2212_12035_amd.build` from the repository root. "
            "There is no CPU fallback." % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    tp = ctypes.POINTER(HarrisTuning)
    lib.harris_coarsity.argtypes = [vp, ci, ci, ci, cf, vp, vp]
    lib.harris_coarsity_u8.argtypes = [vp, ci, ci, ci, cf, vp, vp]
    lib.harris_coarsity_ex.argtypes = [vp, ci, ci, ci, ci, cf, cf, ci, vp, tp, vp]
    lib.harris_plan.argtypes = [ci, ci, ci, ci, ci, ci, tp, tp, ctypes.POINTER(ctypes.c_longlong)]
    lib.harris_coarsity_pitched.argtypes = [vp, ci, ci, ci, ci, ctypes.POINTER(HarrisLayout), cf, cf, ci, vp, tp, vp]
    lib.harris_coarsity_pitched.restype = ci
    lib.harris_coarsity_typed.argtypes = [vp, ci, ci, ci, ci, ctypes.POINTER(HarrisLayout), cf, cf, ci, vp, ci, tp, vp]
    lib.harris_coarsity_typed.restype = ci
    lib.harris_coarsity_quantized.argtypes = [vp, ci, ci, ci, ci, ctypes.POINTER(HarrisLayout), cf, cf, ci, cf, cf, vp, tp, vp]
    lib.harris_coarsity_quantized.restype = ci
    lib.harris_plan_typed.argtypes = [ci, ci, ci, ci, ci, ci, ci, tp, tp, ctypes.POINTER(ctypes.c_longlong)]
    lib.harris_plan_typed.restype = ci
    lib.harris_coarsity_grouped.argtypes = [vp, ci, ci, ci, ci, cf, cf, ci, ci, vp, ctypes.c_longlong, vp, vp]
    lib.harris_coarsity_grouped_static.argtypes = [vp, ci, ci, ci, ci, cf, cf, ci, ci, vp, vp]
    lib.harris_coarsity_grouped_static.restype = ci
    lib.harris_grouped_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.harris_grouped_workspace_bytes.restype = ctypes.c_longlong
    lib.harris_probe_copy.argtypes = [vp, ci, ci, ci, ci, vp, vp]
    lib.harris_probe_copy.restype = ci
    lib.harris_probe_stream.argtypes = [ci, vp, vp, ctypes.c_longlong, vp]
    lib.harris_probe_stream.restype = ci
    for name in ("harris_coarsity", "harris_coarsity_u8", "harris_coarsity_ex", "harris_plan", "harris_version",
                 "harris_coarsity_grouped"):
        getattr(lib, name).restype = ci
    lib.harris_strerror.argtypes = [ci]
    lib.harris_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def harris_strerror(status: int) -> str:
    return load_library().harris_strerror(int(status)).decode()


def harris_version() -> int:
    return int(load_library().harris_version())


def _check(status: int):
    if status != 0:
        raise HarrisError(status, harris_strerror(status))


def _tuning_arg(tuning):
    if tuning is None:
        return None
    if isinstance(tuning, HarrisTuning):
        return ctypes.byref(tuning)
    return ctypes.byref(HarrisTuning(**tuning))


def _prepare(rgb, out, want_dtype):
    import torch
    if not isinstance(rgb, torch.Tensor) or rgb.device.type != "cuda":
        raise TypeError("rgb must be a torch tensor on a ROCm device")
    if rgb.dtype != want_dtype:
        raise TypeError("rgb must have dtype %s" % want_dtype)
    if rgb.dim() != 4 or rgb.shape[1] != 3:
        raise ValueError("rgb must have shape [batch][3][H][W]")
    if not rgb.is_contiguous():
        raise ValueError("rgb must be contiguous (dense planar layout)")
    B, _, H, W = rgb.shape
    if H < 4 or W < 4:
        raise HarrisError(-2, harris_strerror(-2))
    if out is None:
        out = torch.empty((B, H - 4, W - 4), dtype=torch.float32, device=rgb.device)
    else:
        if (not isinstance(out, torch.Tensor) or out.device != rgb.device or out.dtype != torch.float32
                or tuple(out.shape) != (B, H - 4, W - 4) or not out.is_contiguous()):
            raise ValueError("out must be a contiguous float32 tensor [batch][H-4][W-4] on rgb's device")
    return B, H, W, out


def _stream_ptr(stream, device):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(device)
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def harris_coarsity(rgb, k: float = 0.04, out=None, stream=None):
    """float32 rgb[batch][3][H][W] -> float32 out[batch][H-4][W-4]; integer Sobel, 3x3 sum."""
    import torch
    B, H, W, out = _prepare(rgb, out, torch.float32)
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity(rgb.data_ptr(), B, H, W, k, out.data_ptr(), _stream_ptr(stream, rgb.device)))
    return out


def harris_coarsity_u8(rgb, k: float = 0.04, out=None, stream=None):
    """uint8 rgb[batch][3][H][W] (taken as u/255) -> float32 out[batch][H-4][W-4]."""
    import torch
    B, H, W, out = _prepare(rgb, out, torch.uint8)
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_u8(rgb.data_ptr(), B, H, W, k, out.data_ptr(), _stream_ptr(stream, rgb.device)))
    return out


def harris_coarsity_ex(rgb, k: float = 0.04, sobel_scale: float = 1.0, window: int = HARRIS_WINDOW_BOX,
                       out=None, tuning=None, stream=None):
    """General form; the element type is taken from rgb.dtype (float32 or uint8)."""
    import torch
    if not isinstance(rgb, torch.Tensor) or rgb.dtype not in (torch.float32, torch.uint8):
        raise TypeError("rgb must be a float32 or uint8 torch tensor")
    B, H, W, out = _prepare(rgb, out, rgb.dtype)
    dtype = HARRIS_U8 if rgb.dtype == torch.uint8 else HARRIS_F32
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_ex(rgb.data_ptr(), dtype, B, H, W, k, sobel_scale, window,
                                                 out.data_ptr(), _tuning_arg(tuning), _stream_ptr(stream, rgb.device)))
    return out


def _strided(rgb, out, out_dtypes, what):
    """Checks of the entry points that take views; returns (B, H, W, layout, input dtype code).
    rgb [batch][3][H][W] and out [batch][H-4][W-4] may be views (padded rows, a region of
    interest, a slice of planes) as long as the last stride is 1; the pitches are the strides."""
    import torch
    if (not isinstance(rgb, torch.Tensor) or rgb.device.type != "cuda" or rgb.dtype not in (torch.float32, torch.uint8)
            or rgb.dim() != 4 or rgb.shape[1] != 3):
        raise TypeError("rgb must be a float32 or uint8 ROCm tensor of shape [batch][3][H][W]")
    B, _, H, W = rgb.shape
    if H < 4 or W < 4:
        raise HarrisError(-2, harris_strerror(-2))
    if (not isinstance(out, torch.Tensor) or out.device != rgb.device or out.dtype not in out_dtypes
            or tuple(out.shape) != (B, H - 4, W - 4)):
        raise ValueError("out must be a %s tensor [batch][H-4][W-4] on rgb's device" % what)
    if (W > 1 and rgb.stride(3) != 1) or (W - 4 > 1 and out.stride(2) != 1):
        raise ValueError("the last dimension of rgb and out must have stride 1")
    lay = HarrisLayout(rgb.stride(2) if H > 1 else W, rgb.stride(1), rgb.stride(0) if B > 1 else 3 * rgb.stride(1),
                       out.stride(1) if H - 4 > 1 else max(W - 4, 1), out.stride(0) if B > 1 else max(1, (H - 4) * out.stride(1)))
    return B, H, W, lay, HARRIS_U8 if rgb.dtype == torch.uint8 else HARRIS_F32


def harris_coarsity_pitched(rgb, out, k: float = 0.04, sobel_scale: float = 1.0, window: int = HARRIS_WINDOW_BOX,
                            tuning=None, stream=None):
    """General form for strided tensors (views); float32 result."""
    import torch
    B, H, W, lay, dtype = _strided(rgb, out, (torch.float32,), "float32")
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_pitched(rgb.data_ptr(), dtype, B, H, W, ctypes.byref(lay), k, sobel_scale, window,
                                                      out.data_ptr(), _tuning_arg(tuning), _stream_ptr(stream, rgb.device)))
    return out


def harris_coarsity_typed(rgb, out, k: float = 0.04, sobel_scale: float = 1.0, window: int = HARRIS_WINDOW_BOX,
                          tuning=None, stream=None):
    """harris_coarsity_pitched with the result type taken from `out`: float32, float16 or bfloat16."""
    import torch
    kinds = {torch.float32: HARRIS_OUT_F32, torch.float16: HARRIS_OUT_F16, torch.bfloat16: HARRIS_OUT_BF16}
    B, H, W, lay, dtype = _strided(rgb, out, kinds, "float32, float16 or bfloat16")
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_typed(rgb.data_ptr(), dtype, B, H, W, ctypes.byref(lay), k, sobel_scale, window,
                                                    out.data_ptr(), kinds[out.dtype], _tuning_arg(tuning),
                                                    _stream_ptr(stream, rgb.device)))
    return out


def harris_coarsity_quantized(rgb, out, q_scale: float, q_offset: float, k: float = 0.04, sobel_scale: float = 1.0,
                              window: int = HARRIS_WINDOW_BOX, tuning=None, stream=None):
    """8-bit result: out (uint8 [batch][H-4][W-4], may be a view) = clamp(rint(fma(v, q_scale, q_offset)), 0, 255)."""
    import torch
    B, H, W, lay, dtype = _strided(rgb, out, (torch.uint8,), "uint8")
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_quantized(rgb.data_ptr(), dtype, B, H, W, ctypes.byref(lay), k, sobel_scale, window,
                                                        q_scale, q_offset, out.data_ptr(), _tuning_arg(tuning),
                                                        _stream_ptr(stream, rgb.device)))
    return out


def harris_probe_copy(rgb, out=None, stream=None):
    """The streaming-copy probe: out[b][i] = sum over the three planes of their i-th element, i < (H-4)*(W-4)."""
    import torch
    if not isinstance(rgb, torch.Tensor) or rgb.dtype not in (torch.float32, torch.uint8):
        raise TypeError("rgb must be a float32 or uint8 torch tensor")
    B, H, W, out = _prepare(rgb, out, rgb.dtype)
    dtype = HARRIS_U8 if rgb.dtype == torch.uint8 else HARRIS_F32
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_probe_copy(rgb.data_ptr(), dtype, B, H, W, out.data_ptr(), _stream_ptr(stream, rgb.device)))
    return out


HARRIS_PROBE_READ, HARRIS_PROBE_WRITE, HARRIS_PROBE_NONE = 1, 2, 3


def harris_probe_stream(kind: int, src, dst, nbytes: int, stream=None):
    """A pure read (kind 1: src -> nowhere) or write (kind 2: pattern -> dst) stream of nbytes bytes, or a launch that
    moves nothing (kind 3: src, dst may be None)."""
    import torch
    device = dst.device if dst is not None else torch.device("cuda", torch.cuda.current_device())
    with torch.cuda.device(device):
        _check(load_library().harris_probe_stream(kind, src.data_ptr() if src is not None else None,
                                                  dst.data_ptr() if dst is not None else None, nbytes, _stream_ptr(stream, device)))


def harris_grouped_workspace_bytes(grouping: int, batch: int, H: int, W: int) -> int:
    return int(load_library().harris_grouped_workspace_bytes(grouping, batch, H, W))


def harris_coarsity_grouped(rgb, k: float = 0.04, sobel_scale: float = 1.0, window: int = HARRIS_WINDOW_BOX,
                            grouping: int = 1, workspace=None, out=None, stream=None):
    """The unfused / partly fused kernel groupings; `workspace` is a float32 device tensor (made here if None)."""
    import torch
    if not isinstance(rgb, torch.Tensor) or rgb.dtype not in (torch.float32, torch.uint8):
        raise TypeError("rgb must be a float32 or uint8 torch tensor")
    B, H, W, out = _prepare(rgb, out, rgb.dtype)
    need = harris_grouped_workspace_bytes(grouping, B, H, W)
    if need < 0:
        raise HarrisError(-3, harris_strerror(-3))
    if workspace is None:
        workspace = torch.empty(max(1, need // 4), dtype=torch.float32, device=rgb.device)
    dtype = HARRIS_U8 if rgb.dtype == torch.uint8 else HARRIS_F32
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_grouped(rgb.data_ptr(), dtype, B, H, W, k, sobel_scale, window, grouping,
                                                      workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                      out.data_ptr(), _stream_ptr(stream, rgb.device)))
    return out


HARRIS_GROUPED_SCRATCH_BYTES = 64 << 20


def harris_coarsity_grouped_static(rgb, out, k: float = 0.04, sobel_scale: float = 1.0, window: int = HARRIS_WINDOW_BOX,
                                   grouping: int = 1, stream=None):
    """harris_coarsity_grouped on the library's own fixed scratch array: nothing is allocated, here or
    in the library, so `out` (float32 [batch][H-4][W-4], contiguous) must be given."""
    import torch
    if not isinstance(rgb, torch.Tensor) or rgb.dtype not in (torch.float32, torch.uint8):
        raise TypeError("rgb must be a float32 or uint8 torch tensor")
    if out is None:
        raise ValueError("out must be given: this entry point allocates nothing")
    B, H, W, out = _prepare(rgb, out, rgb.dtype)
    dtype = HARRIS_U8 if rgb.dtype == torch.uint8 else HARRIS_F32
    with torch.cuda.device(rgb.device):
        _check(load_library().harris_coarsity_grouped_static(rgb.data_ptr(), dtype, B, H, W, k, sobel_scale, window, grouping,
                                                             out.data_ptr(), _stream_ptr(stream, rgb.device)))
    return out


def harris_plan(dtype: int, batch: int, H: int, W: int, rgb_align: int = 16, out_align: int = 16, tuning=None):
    """(launch shape as a dict, number of workgroups) the library would use; host only."""
    chosen = HarrisTuning()
    blocks = ctypes.c_longlong(0)
    _check(load_library().harris_plan(dtype, batch, H, W, rgb_align, out_align, _tuning_arg(tuning),
                                      ctypes.byref(chosen), ctypes.byref(blocks)))
    return chosen.as_dict(), int(blocks.value)


def harris_plan_typed(dtype: int, out_dtype: int, batch: int, H: int, W: int, rgb_align: int = 16, out_align: int = 16,
                      tuning=None):
    """harris_plan for a result of type out_dtype (HARRIS_OUT_*)."""
    chosen = HarrisTuning()
    blocks = ctypes.c_longlong(0)
    _check(load_library().harris_plan_typed(dtype, out_dtype, batch, H, W, rgb_align, out_align, _tuning_arg(tuning),
                                            ctypes.byref(chosen), ctypes.byref(blocks)))
    return chosen.as_dict(), int(blocks.value)
