"""Harris corner-detection coarsity on AMD MI355X (gfx950).

Thin Python binding over the C interface declared in include/harris.h; every step
of the computation runs in the library's HIP kernel.  PyTorch only supplies device
memory and streams.
"""
from .binding import (  # noqa: F401
    HARRIS_F32, HARRIS_U8, HARRIS_WINDOW_BOX, HARRIS_WINDOW_BINOMIAL,
    HARRIS_SCHEDULE_BANDS, HARRIS_SCHEDULE_TILES, HARRIS_TUNE_NO_ALTERNATE, HARRIS_TUNE_NO_XCD_REMAP,
    HARRIS_TUNE_CACHED_LOADS, HARRIS_TUNE_STREAM_LOADS, HARRIS_TUNE_ALIGNED_STORES, HARRIS_TUNE_PLAIN_STORES, HARRIS_TUNE_KEEP_SHARED_ROWS, HARRIS_TUNE_FLAG_HANDOFF,
    HARRIS_OUT_F32, HARRIS_OUT_F16, HARRIS_OUT_BF16, HARRIS_OUT_U8, harris_coarsity_typed, harris_coarsity_quantized,
    harris_plan_typed,
    HarrisError, HarrisTuning, HarrisLayout, library_path, load_library, harris_coarsity_pitched,
    harris_coarsity, harris_coarsity_u8, harris_coarsity_ex, harris_plan, harris_strerror, harris_version,
    harris_coarsity_grouped, harris_grouped_workspace_bytes, harris_probe_copy,
    harris_coarsity_grouped_static, HARRIS_GROUPED_SCRATCH_BYTES, harris_probe_stream, HARRIS_PROBE_READ, HARRIS_PROBE_WRITE, HARRIS_PROBE_NONE,
)
