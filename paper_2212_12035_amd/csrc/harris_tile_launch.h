// Host-side selection of a tile-kernel instance from a planned launch; included by the two
// translation units that instantiate harris_tile_kernel (one per input type, so that they
// compile in parallel).
#ifndef HARRIS_TILE_LAUNCH_H
#define HARRIS_TILE_LAUNCH_H

#include "harris_kernels.h"

namespace {

template <typename In, int PX, int RW>
hipError_t launch_tiles(const harris_launch::Params& p, dim3 grid, dim3 block, hipStream_t stream) {
    // The four gray rows each wavefront publishes; the planner may reserve more to bound the
    // number of workgroups resident on a CU.
    const size_t lds_needed = (size_t)(block.x / kWave) * 4 * kWave * PX * sizeof(float);
    const size_t lds = p.lds_bytes > lds_needed ? p.lds_bytes : lds_needed;
    const bool cached = p.flags & HARRIS_TUNE_CACHED_LOADS;
    if (p.in_shifted) {
        // 8-bit rows on any byte: kernels for 4 and 8 rows per wavefront, barrier hand-over.
        if constexpr (std::is_same<In, uint8_t>::value && PX == 4 && (RW == 4 || RW == 8)) {
            if (p.flags & HARRIS_TUNE_FLAG_HANDOFF) return hipErrorInvalidValue;
            const bool keep = p.flags & HARRIS_TUNE_KEEP_SHARED_ROWS;
            if (p.binomial) {
                if (keep) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxKeepShared, true, false, true>), grid, block, lds, stream, p);
                else if (cached) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxDefault, true, false, true>), grid, block, lds, stream, p);
                else hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxNonTemporal, true, false, true>), grid, block, lds, stream, p);
            } else {
                if (keep) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxKeepShared, false, false, true>), grid, block, lds, stream, p);
                else if (cached) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxDefault, false, false, true>), grid, block, lds, stream, p);
                else hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxNonTemporal, false, false, true>), grid, block, lds, stream, p);
            }
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    if constexpr (PX == 4) {
        // Kernels that exist for 16-byte lanes only (the planner asks for them nowhere else);
        // ready flags for float32 input only.
        if (p.flags & HARRIS_TUNE_FLAG_HANDOFF) {
            if constexpr (std::is_same<In, float>::value) {
                if (p.binomial) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxNonTemporal, true, true>), grid, block, lds, stream, p);
                else hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxNonTemporal, false, true>), grid, block, lds, stream, p);
                return hipGetLastError();
            } else {
                return hipErrorInvalidValue;
            }
        }
        if (p.flags & HARRIS_TUNE_KEEP_SHARED_ROWS) {
            if (p.binomial) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxKeepShared, true, false>), grid, block, lds, stream, p);
            else hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxKeepShared, false, false>), grid, block, lds, stream, p);
            return hipGetLastError();
        }
    }
    if (p.binomial) {
        if (cached) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxDefault, true, false>), grid, block, lds, stream, p);
        else hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxNonTemporal, true, false>), grid, block, lds, stream, p);
    } else {
        if (cached) hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxDefault, false, false>), grid, block, lds, stream, p);
        else hipLaunchKernelGGL((harris_tile_kernel<In, PX, RW, kAuxNonTemporal, false, false>), grid, block, lds, stream, p);
    }
    return hipGetLastError();
}

// Tile kernels exist for 4 rows per wavefront at every lane width, and for 5, 6, 8, 9 and 10
// rows with four pixels per lane.
template <typename In>
hipError_t launch_tiles_any(const harris_launch::Params& p, const harris_tuning& t, dim3 grid, dim3 block, hipStream_t stream) {
    if (t.rows == 4) {
        switch (t.px) {
            case 1: return launch_tiles<In, 1, 4>(p, grid, block, stream);
            case 2: return launch_tiles<In, 2, 4>(p, grid, block, stream);
            case 4: return launch_tiles<In, 4, 4>(p, grid, block, stream);
            default: return hipErrorInvalidValue;
        }
    }
    if (t.px != 4) return hipErrorInvalidValue;
    switch (t.rows) {
        case 5: return launch_tiles<In, 4, 5>(p, grid, block, stream);
        case 6: return launch_tiles<In, 4, 6>(p, grid, block, stream);
        case 8: return launch_tiles<In, 4, 8>(p, grid, block, stream);
        case 9: return launch_tiles<In, 4, 9>(p, grid, block, stream);
        case 10: return launch_tiles<In, 4, 10>(p, grid, block, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

#endif  // HARRIS_TILE_LAUNCH_H
