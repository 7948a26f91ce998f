// The tile-schedule kernels for 8-bit input (see harris_kernels.h).
#include "harris_tile_launch.h"

namespace harris_launch {

int launch_tiles_u8(const Params& p, const harris_tuning& shape, unsigned grid, unsigned block, void* stream) {
    return (int)launch_tiles_any<uint8_t>(p, shape, dim3(grid), dim3(block), static_cast<hipStream_t>(stream));
}

}  // namespace harris_launch
