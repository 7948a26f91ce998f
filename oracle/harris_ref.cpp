// TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// Plain, slow, stage-by-stage CPU statement of the Harris coarsity pipeline, used
// only to check the GPU library and to be timed beside it as a CPU baseline.
// Nothing in the GPU library includes, links or calls this file, and this file
// uses nothing from the GPU library.
//
// What it follows (thesis chapter 4, "Image Processing Pipelines"):
//   * Listing "Harris operator algorithm in Halide" (section 4.2.1): gray, Ix,
//     Iy, Ixx/Ixy/Iyy, sum3x3, det, trace, output = det - 0.04 * trace^2; no
//     border padding, so the output is 4 pixels smaller than the input in each
//     dimension.
//   * Listings "High-level pointwise operators in Rise", "High-level stencil
//     operators in Rise" and "High-level Harris operator in Rise" (section
//     4.2.2): grayscale = dot [0.299 0.587 0.114] over the channel dimension;
//     conv3x3 = dot (join weights) (join window), i.e. a correlation (no kernel
//     flip) accumulated row-major from 0; Sx, Sy weight matrices; +3x3 = reduce +
//     0 (join window); coarsity = det - kappa * trace * trace.
// The two listings state the same function; where they order a sum differently
// (the Sobel taps) the Halide order is taken, because the thesis names the Halide
// algorithm as its reference and that order cancels exactly on flat images.
// Each stage writes a complete array before the next one starts: no fusion, no
// tiling, no separation of the 3x3 kernels, no reordering of the sums.
//
// Every stage is a template over the real type: `float` is the precision the
// thesis fixes (all arrays are f32); `double` is the same code in (nearly) exact
// arithmetic and serves as referee for rounding questions.  Compile with
// -ffp-contract=off so that no multiply-add is fused.
//
// Parity pins for this file live in tests/test_oracle_pins.py: exact zeros on
// constant images, closed forms on ramps and step edges, a hand-expanded 6x6
// case, a hand-computed integer example, transpose/flip symmetry, power-of-two
// homogeneity, library cross-checks of each stage, and the scale relation.
//
// All pointers are HOST pointers.  Layouts are dense, row-major, x fastest:
// rgb[batch][3][H][W], out[batch][H-4][W-4].

#include <cstdint>
#include <cstddef>
#include <cmath>
#include <thread>
#include <vector>
#include <algorithm>
#include <type_traits>

namespace {

// Run fn(y_begin, y_end) over [0, rows) split into nthreads contiguous row bands.
// Each output row is produced by exactly one thread from read-only inputs, so the
// result does not depend on nthreads.
template <typename F>
void for_row_bands(int rows, int nthreads, F fn) {
    if (rows <= 0) return;
    nthreads = std::max(1, std::min(nthreads, rows));
    if (nthreads == 1) { fn(0, rows); return; }
    std::vector<std::thread> pool;
    for (int t = 0; t < nthreads; ++t) {
        int y0 = (int)((long long)rows * t / nthreads);
        int y1 = (int)((long long)rows * (t + 1) / nthreads);
        pool.emplace_back([=] { fn(y0, y1); });
    }
    for (auto& th : pool) th.join();
}

// Conversion (only for 8-bit input): v = u / 255, one correctly rounded division.
template <typename T>
void normalise_u8(const uint8_t* u, size_t count, T* v, int nthreads) {
    const int rows = (int)std::min<size_t>(count, 1 << 16);
    for_row_bands(rows, nthreads, [=](int r0, int r1) {
        size_t i0 = count * (size_t)r0 / rows, i1 = count * (size_t)r1 / rows;
        for (size_t i = i0; i < i1; ++i) v[i] = (T)u[i] / (T)255;
    });
}

// Grayscale: dot product of [0.299 0.587 0.114] with the (R, G, B)
// triple of each pixel, accumulated from 0 in channel order.
template <typename T>
void grayscale(const T* rgb, int H, int W, T* gray, int nthreads) {
    const T w[3] = {(T)0.299f, (T)0.587f, (T)0.114f};
    const size_t plane = (size_t)H * W;
    for_row_bands(H, nthreads, [=](int y0, int y1) {
        for (int y = y0; y < y1; ++y)
            for (int x = 0; x < W; ++x) {
                T acc = 0;
                for (int c = 0; c < 3; ++c) acc = acc + w[c] * rgb[c * plane + (size_t)y * W + x];
                gray[(size_t)y * W + x] = acc;
            }
    });
}

// conv3x3 as the Rise listing states it: out[y][x] = sum over i, j of
// weights[i][j] * in[y+i][x+j], accumulated row-major from 0 (a correlation: the
// weights are not flipped).  in is H x W, out is (H-2) x (W-2).  Used for the
// weighted (binomial) window of the window-sum stage, and by the tests to confirm that the
// Sobel pair below equals conv3x3 with the Sx / Sy matrices.
template <typename T>
void conv3x3(const T* in, int H, int W, const T weights[3][3], T* out, int nthreads) {
    const int oh = H - 2, ow = W - 2;
    T wt[3][3];
    for (int i = 0; i < 3; ++i) for (int j = 0; j < 3; ++j) wt[i][j] = weights[i][j];
    for_row_bands(oh, nthreads, [=](int y0, int y1) {
        for (int y = y0; y < y1; ++y)
            for (int x = 0; x < ow; ++x) {
                T acc = 0;
                for (int i = 0; i < 3; ++i)
                    for (int j = 0; j < 3; ++j)
                        acc = acc + wt[i][j] * in[(size_t)(y + i) * W + (x + j)];
                out[(size_t)y * ow + x] = acc;
            }
    });
}

// Products: pointwise product of two images of the same size.
template <typename T>
void mul2d(const T* a, const T* b, int H, int W, T* out, int nthreads) {
    for_row_bands(H, nthreads, [=](int y0, int y1) {
        for (size_t i = (size_t)y0 * W; i < (size_t)y1 * W; ++i) out[i] = a[i] * b[i];
    });
}

// Window sums, +3x3: out[y][x] = sum of the nine in[y+i][x+j], accumulated row-major
// from 0.  in is H x W, out is (H-2) x (W-2).
template <typename T>
void sum3x3(const T* in, int H, int W, T* out, int nthreads) {
    const int oh = H - 2, ow = W - 2;
    for_row_bands(oh, nthreads, [=](int y0, int y1) {
        for (int y = y0; y < y1; ++y)
            for (int x = 0; x < ow; ++x) {
                T acc = 0;
                for (int i = 0; i < 3; ++i)
                    for (int j = 0; j < 3; ++j)
                        acc = acc + in[(size_t)(y + i) * W + (x + j)];
                out[(size_t)y * ow + x] = acc;
            }
    });
}

// Coarsity: det = sxx*syy - sxy*sxy; trace = sxx + syy;
// out = det - kappa * trace * trace (evaluated left to right).
template <typename T>
void coarsity(const T* sxx, const T* sxy, const T* syy, int H, int W, T kappa, T* out, int nthreads) {
    for_row_bands(H, nthreads, [=](int y0, int y1) {
        for (size_t i = (size_t)y0 * W; i < (size_t)y1 * W; ++i) {
            T det = sxx[i] * syy[i] - sxy[i] * sxy[i];
            T trace = sxx[i] + syy[i];
            out[i] = det - kappa * trace * trace;
        }
    });
}

// The Sobel pair, in the term order of the Halide listing: the six
// non-zero taps, each negative tap directly followed by its positive mirror, so
// that a constant image gives exactly 0.  Weights are scale*{1, 2}; the thesis and
// its Halide reference use scale = 1/12, the integer matrices are scale = 1.
// in is H x W (gray), ix and iy are (H-2) x (W-2); output (y, x) is centred on
// input (y+1, x+1).  x is the fastest (column) index, y the row index.
template <typename T>
void sobel_xy(const T* in, int H, int W, T scale, T* ix, T* iy, int nthreads) {
    const int oh = H - 2, ow = W - 2;
    const T w1 = (T)1 * scale, w2 = (T)2 * scale;
    for_row_bands(oh, nthreads, [=](int y0, int y1) {
        for (int y = y0; y < y1; ++y)
            for (int x = 0; x < ow; ++x) {
                const T* up = in + (size_t)y * W + x;        // row y-1 of the centre, column x-1
                const T* mid = up + W;
                const T* dn = mid + W;
                if (iy)
                    iy[(size_t)y * ow + x] = up[0] * -w1 + dn[0] * w1 +
                                             up[1] * -w2 + dn[1] * w2 +
                                             up[2] * -w1 + dn[2] * w1;
                if (ix)
                    ix[(size_t)y * ow + x] = up[0] * -w1 + up[2] * w1 +
                                             mid[0] * -w2 + mid[2] * w2 +
                                             dn[0] * -w1 + dn[2] * w1;
            }
    });
}

// The whole pipeline on one image, as the composition in listing "High-level
// Harris operator in Rise".  window: 0 = the 3x3 sum of the thesis; 1 = the
// binomial window [1 2 1; 2 4 2; 1 2 1] that chapter 5 ("Evaluation", binomial
// rewrite goal) names as a common substitute for it.
template <typename T>
void harris_image(const T* rgb, int H, int W, T kappa, T sobel_scale, int window, T* out, int nthreads) {
    const int h2 = H - 2, w2 = W - 2, h4 = H - 4, w4 = W - 4;
    const size_t n0 = (size_t)H * W, n2 = (size_t)h2 * w2, n4 = (size_t)h4 * w4;
    std::vector<T> I(n0), Ix(n2), Iy(n2), Ixx(n2), Ixy(n2), Iyy(n2), Sxx(n4), Sxy(n4), Syy(n4);

    grayscale<T>(rgb, H, W, I.data(), nthreads);
    sobel_xy<T>(I.data(), H, W, sobel_scale, Ix.data(), Iy.data(), nthreads);
    mul2d<T>(Ix.data(), Ix.data(), h2, w2, Ixx.data(), nthreads);
    mul2d<T>(Ix.data(), Iy.data(), h2, w2, Ixy.data(), nthreads);
    mul2d<T>(Iy.data(), Iy.data(), h2, w2, Iyy.data(), nthreads);
    if (window == 0) {
        sum3x3<T>(Ixx.data(), h2, w2, Sxx.data(), nthreads);
        sum3x3<T>(Ixy.data(), h2, w2, Sxy.data(), nthreads);
        sum3x3<T>(Iyy.data(), h2, w2, Syy.data(), nthreads);
    } else {
        const T binom[3][3] = {{1, 2, 1}, {2, 4, 2}, {1, 2, 1}};
        conv3x3<T>(Ixx.data(), h2, w2, binom, Sxx.data(), nthreads);
        conv3x3<T>(Ixy.data(), h2, w2, binom, Sxy.data(), nthreads);
        conv3x3<T>(Iyy.data(), h2, w2, binom, Syy.data(), nthreads);
    }
    coarsity<T>(Sxx.data(), Sxy.data(), Syy.data(), h4, w4, kappa, out, nthreads);
}

// Whole batch; In is float or uint8_t, T the arithmetic type, Out the stored type.
template <typename T, typename In, typename Out>
int harris_batch(const In* rgb, int batch, int H, int W, float kappa, float sobel_scale, int window,
                 Out* out, int nthreads) {
    if (batch < 0 || H < 4 || W < 4 || (window != 0 && window != 1)) return -2;
    if (batch == 0 || H == 4 || W == 4) return 0;
    if (!rgb || !out) return -1;
    const size_t in_n = (size_t)3 * H * W, out_n = (size_t)(H - 4) * (W - 4);
    std::vector<T> img(in_n), res(out_n);
    for (int b = 0; b < batch; ++b) {
        const In* src = rgb + (size_t)b * in_n;
        if constexpr (std::is_same<In, uint8_t>::value) {
            normalise_u8<T>(src, in_n, img.data(), nthreads);
        } else {
            for (size_t i = 0; i < in_n; ++i) img[i] = (T)src[i];
        }
        harris_image<T>(img.data(), H, W, (T)kappa, (T)sobel_scale, window, res.data(), nthreads);
        Out* dst = out + (size_t)b * out_n;
        for (size_t i = 0; i < out_n; ++i) dst[i] = (Out)res[i];
    }
    return 0;
}

}  // namespace

extern "C" {

// Whole pipeline.  f32 arithmetic / f32 result: the oracle proper.
int harris_ref_f32(const float* rgb, int batch, int H, int W, float kappa, float sobel_scale, int window,
                   float* out, int nthreads) {
    return harris_batch<float, float, float>(rgb, batch, H, W, kappa, sobel_scale, window, out, nthreads);
}
int harris_ref_u8_f32(const uint8_t* rgb, int batch, int H, int W, float kappa, float sobel_scale, int window,
                      float* out, int nthreads) {
    return harris_batch<float, uint8_t, float>(rgb, batch, H, W, kappa, sobel_scale, window, out, nthreads);
}
// Same code in double arithmetic, double result: the referee.
int harris_ref_f64(const float* rgb, int batch, int H, int W, float kappa, float sobel_scale, int window,
                   double* out, int nthreads) {
    return harris_batch<double, float, double>(rgb, batch, H, W, kappa, sobel_scale, window, out, nthreads);
}
int harris_ref_u8_f64(const uint8_t* rgb, int batch, int H, int W, float kappa, float sobel_scale, int window,
                      double* out, int nthreads) {
    return harris_batch<double, uint8_t, double>(rgb, batch, H, W, kappa, sobel_scale, window, out, nthreads);
}

// Single stages, so that tests can enter and leave the pipeline anywhere.
void harris_ref_gray_f32(const float* rgb, int H, int W, float* gray) { grayscale<float>(rgb, H, W, gray, 1); }
void harris_ref_gray_f64(const double* rgb, int H, int W, double* gray) { grayscale<double>(rgb, H, W, gray, 1); }

void harris_ref_conv3x3_f32(const float* in, int H, int W, const float* w9, float* out) {
    float w[3][3]; for (int i = 0; i < 9; ++i) w[i / 3][i % 3] = w9[i];
    conv3x3<float>(in, H, W, w, out, 1);
}
void harris_ref_conv3x3_f64(const double* in, int H, int W, const double* w9, double* out) {
    double w[3][3]; for (int i = 0; i < 9; ++i) w[i / 3][i % 3] = w9[i];
    conv3x3<double>(in, H, W, w, out, 1);
}
// which: 0 = Sx, 1 = Sy.
void harris_ref_sobel_f32(const float* gray, int H, int W, float scale, int which, float* out) {
    sobel_xy<float>(gray, H, W, scale, which == 0 ? out : nullptr, which == 0 ? nullptr : out, 1);
}
void harris_ref_sobel_f64(const double* gray, int H, int W, double scale, int which, double* out) {
    sobel_xy<double>(gray, H, W, scale, which == 0 ? out : nullptr, which == 0 ? nullptr : out, 1);
}
void harris_ref_mul_f32(const float* a, const float* b, int H, int W, float* out) { mul2d<float>(a, b, H, W, out, 1); }
void harris_ref_mul_f64(const double* a, const double* b, int H, int W, double* out) { mul2d<double>(a, b, H, W, out, 1); }
void harris_ref_sum3x3_f32(const float* in, int H, int W, float* out) { sum3x3<float>(in, H, W, out, 1); }
void harris_ref_sum3x3_f64(const double* in, int H, int W, double* out) { sum3x3<double>(in, H, W, out, 1); }
void harris_ref_coarsity_f32(const float* sxx, const float* sxy, const float* syy, int H, int W, float kappa, float* out) {
    coarsity<float>(sxx, sxy, syy, H, W, kappa, out, 1);
}
void harris_ref_coarsity_f64(const double* sxx, const double* sxy, const double* syy, int H, int W, double kappa, double* out) {
    coarsity<double>(sxx, sxy, syy, H, W, kappa, out, 1);
}

// Rounding of a finished float32 result to a 16-bit storage format, for the library's
// reduced-precision result options (not part of the thesis, whose arrays are all f32; the
// definition is IEEE 754 round-to-nearest, ties to even, overflow to infinity).  Written from
// that definition in double arithmetic: find the binade, divide by the spacing of the target
// format there, round to an integer with the default rounding mode, rebuild the bit pattern.
//   binary16: 11 significant bits, exponents -14..15, subnormals spaced 2^-24.
//   bfloat16:  8 significant bits, exponents -126..127, subnormals spaced 2^-133.
static uint16_t round_to_16bit(float x, int significant_bits, int min_exponent, int exponent_bits) {
    const int bias = (1 << (exponent_bits - 1)) - 1;
    const int fraction_bits = significant_bits - 1;
    const uint16_t sign = std::signbit(x) ? (uint16_t)0x8000 : (uint16_t)0;
    const uint16_t all_ones_exponent = (uint16_t)(((1 << exponent_bits) - 1) << fraction_bits);
    if (std::isnan(x)) return (uint16_t)(sign | all_ones_exponent | (1 << (fraction_bits - 1)));   // quiet NaN
    if (std::isinf(x)) return (uint16_t)(sign | all_ones_exponent);
    const double a = std::fabs((double)x);
    if (a == 0.0) return sign;
    int e;
    std::frexp(a, &e);                         // a = f * 2^e with f in [0.5, 1): floor(log2 a) = e - 1
    int binade = e - 1;
    if (binade < min_exponent) binade = min_exponent;                   // subnormal range: fixed spacing
    const double spacing = std::ldexp(1.0, binade - fraction_bits);
    const double rounded = std::nearbyint(a / spacing) * spacing;        // ties to even (default rounding mode)
    if (rounded >= std::ldexp(1.0, bias + 1)) return (uint16_t)(sign | all_ones_exponent);   // past the largest finite value
    if (rounded < std::ldexp(1.0, min_exponent))                        // zero or subnormal: the fraction counts spacings
        return (uint16_t)(sign | (uint16_t)std::lround(rounded / std::ldexp(1.0, min_exponent - fraction_bits)));
    std::frexp(rounded, &e);
    const int exponent = e - 1;
    const double fraction = rounded / std::ldexp(1.0, exponent) - 1.0;  // in [0, 1), a multiple of 2^-fraction_bits
    return (uint16_t)(sign | (uint16_t)((exponent + bias) << fraction_bits) | (uint16_t)std::lround(std::ldexp(fraction, fraction_bits)));
}

void harris_ref_round_binary16(const float* in, long long count, uint16_t* out) {
    for (long long i = 0; i < count; ++i) out[i] = round_to_16bit(in[i], 11, -14, 5);
}

void harris_ref_round_bfloat16(const float* in, long long count, uint16_t* out) {
    for (long long i = 0; i < count; ++i) out[i] = round_to_16bit(in[i], 8, -126, 8);
}

// 8-bit result codes of the library's quantised result option (not part of the thesis):
// code = clamp(round_to_nearest_even(fma(v, scale, offset)), 0, 255), the multiply-add rounded
// once in float32 (std::fmaf is the exact fused operation), NaN -> 0.
void harris_ref_quantize_u8(const float* in, long long count, float scale, float offset, uint8_t* out) {
    for (long long i = 0; i < count; ++i) {
        const float t = std::fmaf(in[i], scale, offset);
        if (std::isnan(t)) { out[i] = 0; continue; }
        const float r = std::nearbyintf(t);                  // default rounding mode: ties to even
        out[i] = (uint8_t)(r <= 0.0f ? 0.0f : r >= 255.0f ? 255.0f : r);
    }
}

int harris_ref_hardware_threads(void) { return (int)std::max(1u, std::thread::hardware_concurrency()); }

}  // extern "C"
