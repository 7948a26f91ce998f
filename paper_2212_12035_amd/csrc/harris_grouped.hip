// Unfused and partly fused Harris pipelines: the kernel groupings of the thesis's chapter 3,
// section "Explicit Kernel Execution", subsection "Evaluating the Boilerplate Avoided through
// Kernel Execution" (table "Four different kernel groupings"), as plain HIP kernels that keep
// every intermediate image in device memory.
//
//   grouping 1: [gray] [Sx] [Sy] [x] [x] [x] [+] [+] [+] [coarsity]
//   grouping 2: [gray] [Sx, Sy, x]  [+, coarsity]
//   grouping 3: [gray] [Sx, Sy]     [x, +, coarsity]
//   grouping 4: everything in one kernel: that is harris_coarsity_ex itself
//
// (The thesis's table starts from a grayscale image; the grayscale stage is a kernel
// of its own here.)  They exist to measure what fusion buys on this GPU with the same
// harness, and as a second GPU implementation that shares no code with the fused
// kernels: one thread per result pixel, every tap a global load, no LDS, no lane
// exchange, no separation of the 3x3 kernels.  They are baselines, not tuned.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>

#include "harris_launch.h"

// Intermediate images for harris_coarsity_grouped_static: callers that cannot allocate (code
// under stream capture, serving loops) get the groupings' workspace from here.  Each GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.
// Host code never uses this name as an address: it asks for the device's address once per
// device (scratch_of_current_device) and hands that pointer to the kernels.
static __device__ __align__(256) float scratch[HARRIS_GROUPED_SCRATCH_BYTES / sizeof(float)];

namespace {

constexpr int kTileX = 64, kTileY = 4;      // 256 threads: 64 consecutive columns of 4 rows

__device__ __forceinline__ bool pixel(int w, int h, int& x, int& y) {
    x = blockIdx.x * kTileX + threadIdx.x;
    y = blockIdx.y * kTileY + threadIdx.y;
    return x < w && y < h;
}

// Conversion and grayscale.  rgb[b][3][H][W] -> gray[b][H][W]; in_scale is 1 (float32) or 1/255 (uint8).
template <typename In>
__global__ void gray_kernel(const In* rgb, float* gray, int H, int W, float in_scale) {
    int x, y;
    if (!pixel(W, H, x, y)) return;
    const size_t plane = (size_t)H * W, img = (size_t)blockIdx.z * 3 * plane, at = (size_t)y * W + x;
    const float r = (float)rgb[img + at] * in_scale, g = (float)rgb[img + plane + at] * in_scale, b = (float)rgb[img + 2 * plane + at] * in_scale;
    gray[(size_t)blockIdx.z * plane + at] = 0.299f * r + 0.587f * g + 0.114f * b;
}

// The two Sobel responses at result pixel (y, x) of an h x w result; in is (h+2) x (w+2).
__device__ __forceinline__ void sobel_at(const float* in, int w, int y, int x, float s, float& ix, float& iy) {
    const float* r0 = in + (size_t)y * (w + 2) + x;
    const float* r1 = r0 + (w + 2);
    const float* r2 = r1 + (w + 2);
    ix = s * ((r0[2] - r0[0]) + 2.0f * (r1[2] - r1[0]) + (r2[2] - r2[0]));
    iy = s * ((r2[0] - r0[0]) + 2.0f * (r2[1] - r0[1]) + (r2[2] - r0[2]));
}

// Sobel stage, one response per launch: which = 0 for Sx, 1 for Sy.  in[b][h+2][w+2] -> out[b][h][w].
__global__ void sobel_kernel(const float* in, float* out, int h, int w, float s, int which) {
    int x, y;
    if (!pixel(w, h, x, y)) return;
    float ix, iy;
    sobel_at(in + (size_t)blockIdx.z * (h + 2) * (w + 2), w, y, x, s, ix, iy);
    out[(size_t)blockIdx.z * h * w + (size_t)y * w + x] = which == 0 ? ix : iy;
}

// Sobel stage, both responses.
__global__ void sobel_pair_kernel(const float* in, float* ix_out, float* iy_out, int h, int w, float s) {
    int x, y;
    if (!pixel(w, h, x, y)) return;
    float ix, iy;
    sobel_at(in + (size_t)blockIdx.z * (h + 2) * (w + 2), w, y, x, s, ix, iy);
    const size_t at = (size_t)blockIdx.z * h * w + (size_t)y * w + x;
    ix_out[at] = ix;
    iy_out[at] = iy;
}

// Sobel pair and products.
__global__ void sobel_products_kernel(const float* in, float* ixx, float* ixy, float* iyy, int h, int w, float s) {
    int x, y;
    if (!pixel(w, h, x, y)) return;
    float ix, iy;
    sobel_at(in + (size_t)blockIdx.z * (h + 2) * (w + 2), w, y, x, s, ix, iy);
    const size_t at = (size_t)blockIdx.z * h * w + (size_t)y * w + x;
    ixx[at] = ix * ix;
    ixy[at] = ix * iy;
    iyy[at] = iy * iy;
}

// Products, one per launch.
__global__ void mul_kernel(const float* a, const float* b, float* out, size_t count) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = a[i] * b[i];
}

// 3x3 window weights: all ones, or [1 2 1; 2 4 2; 1 2 1].
__device__ __forceinline__ float window_weight(int i, int j, int binomial) {
    return binomial ? (float)((2 - (i > 1 ? i - 1 : 1 - i)) * (2 - (j > 1 ? j - 1 : 1 - j))) : 1.0f;
}

// Window sums, one per launch.  in[b][h+2][w+2] -> out[b][h][w].
__global__ void window_kernel(const float* in, float* out, int h, int w, int binomial) {
    int x, y;
    if (!pixel(w, h, x, y)) return;
    const float* p = in + (size_t)blockIdx.z * (h + 2) * (w + 2) + (size_t)y * (w + 2) + x;
    float acc = 0.0f;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) acc += window_weight(i, j, binomial) * p[(size_t)i * (w + 2) + j];
    out[(size_t)blockIdx.z * h * w + (size_t)y * w + x] = acc;
}

__device__ __forceinline__ float coarsity_of(float sxx, float sxy, float syy, float k) {
    const float det = sxx * syy - sxy * sxy, tr = sxx + syy;
    return det - k * tr * tr;
}

// Coarsity.
__global__ void coarsity_kernel(const float* sxx, const float* sxy, const float* syy, float* out, size_t count, float k) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = coarsity_of(sxx[i], sxy[i], syy[i], k);
}

// Window sums and coarsity from the three product images.
__global__ void window_coarsity_kernel(const float* ixx, const float* ixy, const float* iyy, float* out, int h, int w, float k, int binomial) {
    int x, y;
    if (!pixel(w, h, x, y)) return;
    const size_t at = (size_t)blockIdx.z * (h + 2) * (w + 2) + (size_t)y * (w + 2) + x;
    float sxx = 0.0f, sxy = 0.0f, syy = 0.0f;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) {
            const float wt = window_weight(i, j, binomial);
            const size_t q = at + (size_t)i * (w + 2) + j;
            sxx += wt * ixx[q];
            sxy += wt * ixy[q];
            syy += wt * iyy[q];
        }
    out[(size_t)blockIdx.z * h * w + (size_t)y * w + x] = coarsity_of(sxx, sxy, syy, k);
}

// Products, window sums and coarsity from the two Sobel images.
__global__ void products_window_coarsity_kernel(const float* ix, const float* iy, float* out, int h, int w, float k, int binomial) {
    int x, y;
    if (!pixel(w, h, x, y)) return;
    const size_t at = (size_t)blockIdx.z * (h + 2) * (w + 2) + (size_t)y * (w + 2) + x;
    float sxx = 0.0f, sxy = 0.0f, syy = 0.0f;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) {
            const float wt = window_weight(i, j, binomial);
            const size_t q = at + (size_t)i * (w + 2) + j;
            const float gx = ix[q], gy = iy[q];
            sxx += wt * gx * gx;
            sxy += wt * gx * gy;
            syy += wt * gy * gy;
        }
    out[(size_t)blockIdx.z * h * w + (size_t)y * w + x] = coarsity_of(sxx, sxy, syy, k);
}

dim3 grid2d(int w, int h, int batch) { return dim3((w + kTileX - 1) / kTileX, (h + kTileY - 1) / kTileY, batch); }
dim3 grid1d(size_t count) { return dim3((unsigned)((count + 255) / 256)); }

}  // namespace

namespace harris_launch {

size_t grouped_workspace_floats(int grouping, int batch, int H, int W) {
    const size_t n0 = (size_t)H * W, n2 = (size_t)(H - 2) * (W - 2), n4 = (size_t)(H - 4) * (W - 4);
    switch (grouping) {
        case 1: return (size_t)batch * (n0 + 5 * n2 + 3 * n4);   // gray, Ix, Iy, Ixx, Ixy, Iyy, Sxx, Sxy, Syy
        case 2: return (size_t)batch * (n0 + 3 * n2);            // gray, Ixx, Ixy, Iyy
        case 3: return (size_t)batch * (n0 + 2 * n2);            // gray, Ix, Iy
        default: return 0;
    }
}

int launch_grouped(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale, int binomial,
                   int grouping, float* ws, float* out, void* stream_) {
    hipStream_t st = static_cast<hipStream_t>(stream_);
    if (batch > 65535) return HARRIS_ERR_SHAPE;        // images ride on gridDim.z
    const int h2 = H - 2, w2 = W - 2, h4 = H - 4, w4 = W - 4;
    const size_t n0 = (size_t)batch * H * W, n2 = (size_t)batch * h2 * w2, n4 = (size_t)batch * h4 * w4;
    const dim3 blk2(kTileX, kTileY), blk1(256);
    float* gray = ws;
    if (dtype == HARRIS_U8) hipLaunchKernelGGL(gray_kernel<uint8_t>, grid2d(W, H, batch), blk2, 0, st, static_cast<const uint8_t*>(rgb), gray, H, W, 1.0f / 255.0f);
    else hipLaunchKernelGGL(gray_kernel<float>, grid2d(W, H, batch), blk2, 0, st, static_cast<const float*>(rgb), gray, H, W, 1.0f);
    if (grouping == 1) {
        float *ix = gray + n0, *iy = ix + n2, *ixx = iy + n2, *ixy = ixx + n2, *iyy = ixy + n2, *sxx = iyy + n2, *sxy = sxx + n4, *syy = sxy + n4;
        hipLaunchKernelGGL(sobel_kernel, grid2d(w2, h2, batch), blk2, 0, st, gray, ix, h2, w2, sobel_scale, 0);
        hipLaunchKernelGGL(sobel_kernel, grid2d(w2, h2, batch), blk2, 0, st, gray, iy, h2, w2, sobel_scale, 1);
        hipLaunchKernelGGL(mul_kernel, grid1d(n2), blk1, 0, st, ix, ix, ixx, n2);
        hipLaunchKernelGGL(mul_kernel, grid1d(n2), blk1, 0, st, ix, iy, ixy, n2);
        hipLaunchKernelGGL(mul_kernel, grid1d(n2), blk1, 0, st, iy, iy, iyy, n2);
        hipLaunchKernelGGL(window_kernel, grid2d(w4, h4, batch), blk2, 0, st, ixx, sxx, h4, w4, binomial);
        hipLaunchKernelGGL(window_kernel, grid2d(w4, h4, batch), blk2, 0, st, ixy, sxy, h4, w4, binomial);
        hipLaunchKernelGGL(window_kernel, grid2d(w4, h4, batch), blk2, 0, st, iyy, syy, h4, w4, binomial);
        hipLaunchKernelGGL(coarsity_kernel, grid1d(n4), blk1, 0, st, sxx, sxy, syy, out, n4, k);
    } else if (grouping == 2) {
        float *ixx = gray + n0, *ixy = ixx + n2, *iyy = ixy + n2;
        hipLaunchKernelGGL(sobel_products_kernel, grid2d(w2, h2, batch), blk2, 0, st, gray, ixx, ixy, iyy, h2, w2, sobel_scale);
        hipLaunchKernelGGL(window_coarsity_kernel, grid2d(w4, h4, batch), blk2, 0, st, ixx, ixy, iyy, out, h4, w4, k, binomial);
    } else {
        float *ix = gray + n0, *iy = ix + n2;
        hipLaunchKernelGGL(sobel_pair_kernel, grid2d(w2, h2, batch), blk2, 0, st, gray, ix, iy, h2, w2, sobel_scale);
        hipLaunchKernelGGL(products_window_coarsity_kernel, grid2d(w4, h4, batch), blk2, 0, st, ix, iy, out, h4, w4, k, binomial);
    }
    return hipGetLastError() == hipSuccess ? HARRIS_OK : HARRIS_ERR_LAUNCH;
}

// Device address of `scratch` on the current device, looked up once per device (with that
// device current, as now) and kept.  NULL if the runtime cannot say.
float* scratch_of_current_device() {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static float* known[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(lock);
    if (known[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        known[dev] = static_cast<float*>(ptr);
    }
    return known[dev];
}

}  // namespace harris_launch
