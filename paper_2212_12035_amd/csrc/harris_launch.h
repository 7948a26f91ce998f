// Internal to libharris: what the host-side planner hands to the kernel launcher.
#ifndef HARRIS_LAUNCH_H
#define HARRIS_LAUNCH_H

#include <stddef.h>

#include "harris_tuning.h"

namespace harris_launch {

// Lanes of a 64-lane wavefront that produce result columns when each lane holds px
// columns: the remaining lane(s) only supply the 4-column halo to the right.
constexpr int valid_lanes(int px) { return 64 - (4 + px - 1) / px; }

// Division of a 32-bit unsigned number by a divisor fixed at launch, as one multiply-high, an
// addition and two shifts (Granlund and Montgomery, "Division by invariant integers using
// multiplication", 1994, the unsigned algorithm for a run-time invariant divisor): with
// l = ceil(log2 d), mul = floor(2^32 (2^l - d) / d) + 1, sh1 = min(l, 1), sh2 = max(l - 1, 0),
// floor(x / d) = (t + ((x - t) >> sh1)) >> sh2 where t = high word of mul * x.  Exact for every
// x < 2^32 and 1 <= d < 2^32.  A workgroup decomposes its index with it before its first load
// (a hardware integer division costs some 25 dependent scalar instructions).
struct FastDiv {
    unsigned mul, sh1, sh2;
};

inline FastDiv make_fastdiv(unsigned d) {
    FastDiv f;
    unsigned l = 0;
    while (l < 32 && (1ull << l) < d) ++l;
    f.mul = (unsigned)((((1ull << l) - d) << 32) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l < 1 ? 0 : l - 1;
    return f;
}

#if defined(__HIPCC__)
#define HARRIS_HOST_DEVICE __host__ __device__
#else
#define HARRIS_HOST_DEVICE
#endif
HARRIS_HOST_DEVICE inline unsigned fastdiv(unsigned x, const FastDiv& f) {
    const unsigned t = (unsigned)(((unsigned long long)f.mul * x) >> 32);
    return (t + ((x - t) >> f.sh1)) >> f.sh2;
}

// Kernel arguments (passed by value).  What the tile kernel reads before its first load sits
// together, so that a few wide scalar loads fetch it at once.
struct Params {
    const void* rgb;        // device, [batch][3][H][W] with the pitches below
    void* out;              // device, [batch][n][m] with the pitches below; element type given by out_kind
    long long in_row_pitch, in_plane_pitch, in_image_pitch;   // in input elements
    long long out_row_pitch, out_image_pitch;                 // in result elements
    int H, W;               // input rows, columns
    int n, m;               // result rows, columns (H-4, W-4)
    int rows_per_band;      // result rows per band (BANDS) or per tile (TILES)
    unsigned n_strips;      // strips per band
    unsigned strip_pitch;   // result columns per strip (a multiple of px, at most valid_lanes(px)*px; 12 less with aligned stores)
    unsigned tiles_per_image;  // n_bands * n_strips (TILES: one workgroup each)
    FastDiv by_tiles_per_image, by_n_strips;   // TILES: division by these two
    unsigned n_blocks;      // workgroups of the launch (the grid size)
    unsigned waves_per_block;  // wavefronts per workgroup (the block size / 64)
    float wr, wg, wb;       // gray weights, times the Sobel scale (and 1/255 for 8-bit input)
    float k;                // coarsity constant
    unsigned flags;         // HARRIS_TUNE_* bits
    unsigned out_kind;      // a harris_out_dtype (other than float32: tile kernel only)
    float q_scale, q_offset;   // 8-bit results: code = clamp(rint(fma(v, q_scale, q_offset)), 0, 255)
    int binomial;           // 1: window [1 2 1; 2 4 2; 1 2 1], 0: unweighted 3x3 sum
    unsigned lds_bytes;     // TILES: dynamic LDS per workgroup (the tile's rows, or more to bound the resident workgroups)
    int in_shifted;         // 1: 8-bit rows that start on any byte, loaded as aligned words and shifted (tile kernel, px 4)
    unsigned n_bands;       // bands (BANDS) or tiles down the image (TILES)
    unsigned blocks_x;      // BANDS: workgroups across a row of bands
    unsigned blocks_per_image;  // BANDS: workgroups per image
};

// Enqueue the fused kernel.  `shape` must come from harris_plan (all fields set).
// Returns a harris_status.
int launch(const Params& p, const harris_tuning& shape, long long n_blocks, int dtype, void* stream);

// The translation units that hold the kernels: each enqueues the instance that `shape` names
// with `grid` workgroups of `block` threads and returns the hipError_t of the launch as int
// (hipErrorInvalidValue for a shape it has no kernel for).
int launch_tiles_f32(const Params& p, const harris_tuning& shape, unsigned grid, unsigned block, void* stream);
int launch_tiles_u8(const Params& p, const harris_tuning& shape, unsigned grid, unsigned block, void* stream);
int launch_bands(const Params& p, const harris_tuning& shape, int dtype, unsigned grid, unsigned block, void* stream);

// Floats of workspace the grouped (unfused) pipelines need; 0 for an unknown grouping.
size_t grouped_workspace_floats(int grouping, int batch, int H, int W);

// Enqueue grouping 1, 2 or 3 (see harris_coarsity_grouped).  Returns a harris_status.
int launch_grouped(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale, int binomial,
                   int grouping, float* workspace, float* out, void* stream);

// Device address, on the current device, of the library's fixed scratch array of
// HARRIS_GROUPED_SCRATCH_BYTES bytes (see harris_coarsity_grouped_static); NULL on failure.
float* scratch_of_current_device();

// Enqueue the streaming-copy probe (see harris_probe_copy).  Returns a harris_status.
int launch_copy_probe(const void* rgb, int dtype, int batch, int H, int W, float* out, void* stream);

// Enqueue a pure read or write stream (see harris_probe_stream).  Returns a harris_status.
int launch_stream_probe(int kind, const void* src, void* dst, long long bytes, void* stream);

}  // namespace harris_launch

#endif
