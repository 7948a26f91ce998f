// Hands a planned launch to the translation unit that holds its kernels.
#include "harris_tuning.h"
#include "harris_launch.h"

namespace harris_launch {

int launch(const Params& p, const harris_tuning& shape, long long n_blocks, int dtype, void* stream) {
    if (n_blocks != (long long)p.n_blocks || shape.waves_per_block != (int)p.waves_per_block) return HARRIS_ERR_LAUNCH;
    const unsigned grid = (unsigned)n_blocks, block = (unsigned)shape.waves_per_block * 64u;
    int e;
    if (shape.schedule == HARRIS_SCHEDULE_TILES) e = dtype == HARRIS_U8 ? launch_tiles_u8(p, shape, grid, block, stream) : launch_tiles_f32(p, shape, grid, block, stream);
    else e = launch_bands(p, shape, dtype, grid, block, stream);
    return e == 0 ? HARRIS_OK : HARRIS_ERR_LAUNCH;     // 0 is hipSuccess
}

}  // namespace harris_launch
