// Internal to libharris: what the host-side planner hands to the kernel launcher.
#ifndef HARRIS_LAUNCH_H
#define HARRIS_LAUNCH_H

#include <stddef.h>

#include "harris.h"

namespace harris_launch {

// Lanes of a 64-lane wavefront that produce result columns when each lane holds px
// columns: the remaining lane(s) only supply the 4-column halo to the right.
constexpr int valid_lanes(int px) { return 64 - (4 + px - 1) / px; }

// Kernel arguments (passed by value).
struct Params {
    const void* rgb;        // device, [batch][3][H][W] with the pitches below
    float* out;             // device, [batch][n][m] with the pitches below
    long long in_row_pitch, in_plane_pitch, in_image_pitch;   // in input elements
    long long out_row_pitch, out_image_pitch;                 // in floats
    int H, W;               // input rows, columns
    int n, m;               // result rows, columns (H-4, W-4)
    int rows_per_band;      // result rows per band (BANDS) or per tile (TILES)
    unsigned n_strips;      // strips per band
    unsigned strip_pitch;   // result columns per strip (a multiple of px, at most valid_lanes(px)*px)
    unsigned n_bands;       // bands (BANDS) or tiles down the image (TILES)
    unsigned tiles_per_image;  // n_bands * n_strips (TILES: one workgroup each)
    unsigned blocks_x;      // BANDS: workgroups across a row of bands
    unsigned blocks_per_image;  // BANDS: workgroups per image
    float wr, wg, wb;       // gray weights, times the Sobel scale (and 1/255 for 8-bit input)
    float k;                // coarsity constant
    int binomial;           // 1: window [1 2 1; 2 4 2; 1 2 1], 0: unweighted 3x3 sum
    unsigned flags;         // HARRIS_TUNE_* bits
};

// Enqueue the fused kernel.  `shape` must come from harris_plan (all fields set).
// Returns a harris_status.
int launch(const Params& p, const harris_tuning& shape, long long n_blocks, int dtype, void* stream);

// Floats of workspace the grouped (unfused) pipelines need; 0 for an unknown grouping.
size_t grouped_workspace_floats(int grouping, int batch, int H, int W);

// Enqueue grouping 1, 2 or 3 (see harris_coarsity_grouped).  Returns a harris_status.
int launch_grouped(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale, int binomial,
                   int grouping, float* workspace, float* out, void* stream);

}  // namespace harris_launch

#endif
