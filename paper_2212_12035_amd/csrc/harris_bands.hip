// The band-schedule kernels (see harris_kernels.h): float32 results only, three input rows in
// flight per wavefront, 1, 2 or 4 pixels per lane.
#include "harris_kernels.h"

namespace {

constexpr int kRowsInFlight = 3;

template <typename In, int PX>
hipError_t launch_bands_px(const harris_launch::Params& p, dim3 grid, dim3 block, hipStream_t stream) {
    const bool cached = p.flags & HARRIS_TUNE_CACHED_LOADS;
    if (p.binomial) {
        if (cached) hipLaunchKernelGGL((harris_fused_kernel<In, PX, kRowsInFlight, kAuxDefault, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((harris_fused_kernel<In, PX, kRowsInFlight, kAuxNonTemporal, true>), grid, block, 0, stream, p);
    } else {
        if (cached) hipLaunchKernelGGL((harris_fused_kernel<In, PX, kRowsInFlight, kAuxDefault, false>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((harris_fused_kernel<In, PX, kRowsInFlight, kAuxNonTemporal, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

template <typename In>
hipError_t launch_bands_in(const harris_launch::Params& p, const harris_tuning& t, dim3 grid, dim3 block, hipStream_t stream) {
    if (p.out_kind != HARRIS_OUT_F32 || t.prefetch != kRowsInFlight) return hipErrorInvalidValue;
    switch (t.px) {
        case 1: return launch_bands_px<In, 1>(p, grid, block, stream);
        case 2: return launch_bands_px<In, 2>(p, grid, block, stream);
        case 4: return launch_bands_px<In, 4>(p, grid, block, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

namespace harris_launch {

int launch_bands(const Params& p, const harris_tuning& shape, int dtype, unsigned grid, unsigned block, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    return (int)(dtype == HARRIS_U8 ? launch_bands_in<uint8_t>(p, shape, dim3(grid), dim3(block), s)
                                    : launch_bands_in<float>(p, shape, dim3(grid), dim3(block), s));
}

}  // namespace harris_launch
