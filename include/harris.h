/*
 * libharris: Harris corner-detection coarsity on one AMD MI355X (gfx950).
 *
 * The operation is the Harris operator of the thesis's chapter 4, section 4.2
 * (listing "Harris operator algorithm in Halide", and the Rise listings
 * "High-level pointwise operators", "High-level stencil operators" and
 * "High-level Harris operator"):
 *
 *   gray = 0.299 R + 0.587 G + 0.114 B
 *   Ix   = Sx gray,  Iy = Sy gray          3x3 Sobel correlations, valid region
 *   Ixx  = Ix*Ix, Ixy = Ix*Iy, Iyy = Iy*Iy
 *   Sxx, Sxy, Syy = 3x3 window sums of Ixx, Ixy, Iyy, valid region
 *   out  = (Sxx*Syy - Sxy*Sxy) - k * (Sxx + Syy)^2
 *
 * with no border padding: a 3 x H x W image gives an (H-4) x (W-4) result, and
 * out[y][x] depends on rgb[:, y..y+4, x..x+4].  All of it runs in one fused GPU
 * kernel; no intermediate image is written to device memory.
 *
 * Conventions common to every entry point
 *   - rgb and out are DEVICE pointers owned by the caller.  The library allocates
 *     nothing, keeps no state between calls and is re-entrant.
 *   - rgb is dense, planar, row-major: rgb[batch][3][H][W], x (the W index) fastest.
 *     out is dense: out[batch][H-4][W-4].  out must not overlap rgb.
 *   - Any pointer alignment natural to the element type and any H, W >= 4 are
 *     accepted.  The fastest path is taken when W is a multiple of 4 and both base
 *     pointers are 16-byte aligned (8-byte aligned and even W is next best).
 *   - The work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without waiting for it.
 *   - The return value is a harris_status.  Nothing is written to stdout/stderr and
 *     no C++ exception crosses this interface.  On any error nothing is enqueued.
 *   - batch == 0, H == 4 or W == 4 describe an empty result: HARRIS_OK, no work,
 *     pointers are not examined.
 */
#ifndef HARRIS_H
#define HARRIS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum harris_status {
    HARRIS_OK = 0,
    HARRIS_ERR_NULL = -1,    /* rgb or out is NULL although the result is not empty        */
    HARRIS_ERR_SHAPE = -2,   /* batch < 0, H < 4, W < 4, W > 2^28, H > 2^30, more than 2^31-1 tiles, or
                                pitches smaller than the image                               */
    HARRIS_ERR_ARG = -3,     /* k or sobel_scale not finite, unknown dtype/window/tuning,
                                misaligned pointer                                          */
    HARRIS_ERR_LAUNCH = -4,  /* the HIP runtime refused the kernel launch                   */
    HARRIS_ERR_SCRATCH = -5  /* harris_coarsity_grouped_static: the problem needs more than
                                HARRIS_GROUPED_SCRATCH_BYTES of intermediates               */
} harris_status;

/* Element type of the input image. */
typedef enum harris_dtype {
    HARRIS_F32 = 0,          /* float32 planes, values used as they are                     */
    HARRIS_U8 = 1            /* uint8 planes, each value divided by 255 inside the kernel   */
} harris_dtype;

/* The 3x3 window that accumulates Ixx, Ixy, Iyy. */
typedef enum harris_window {
    HARRIS_WINDOW_BOX = 0,      /* unweighted 3x3 sum: the "+3x3" operator of section 4.2      */
    HARRIS_WINDOW_BINOMIAL = 1  /* [1 2 1; 2 4 2; 1 2 1], the substitute named in chapter 5's
                                   evaluation (binomial rewrite goal)                         */
} harris_window;

/*
 * Launch-shape override for benchmarks and tests; NULL in ordinary use (the library then
 * chooses the shape from the problem).  The structure, its flag bits and the planning
 * calls are declared in harris_tuning.h, which is not needed to use the operator.
 * Results never depend on the launch shape beyond rounding.
 */
typedef struct harris_tuning harris_tuning;

/*
 * Harris coarsity of float32 images with the integer Sobel matrices
 * Sx = [-1 0 1; -2 0 2; -1 0 1], Sy = its transpose, and the unweighted 3x3 sum.
 * (Section 4.2; equals harris_coarsity_ex with HARRIS_F32, sobel_scale 1,
 * HARRIS_WINDOW_BOX, no tuning.)
 *   rgb   device, float32 [batch][3][H][W], read only
 *   k     the coarsity constant kappa (0.04 in the thesis)
 *   out   device, float32 [batch][H-4][W-4], fully overwritten
 */
int harris_coarsity(const float* rgb, int batch, int H, int W, float k, float* out, void* stream);

/* Same for uint8 images; each value is taken as u/255 (then section 4.2). */
int harris_coarsity_u8(const uint8_t* rgb, int batch, int H, int W, float k, float* out, void* stream);

/*
 * General form.
 *   rgb          device, element type given by `dtype` (a harris_dtype)
 *   sobel_scale  factor applied to both Sobel matrices.  1 gives the integer
 *                matrices; 1.0f/12 gives exactly the operator of the thesis's
 *                listings (section 4.2), whose results are those of scale 1
 *                divided by 12^4.
 *   window       a harris_window
 *   tuning       NULL, or a launch shape (harris_tuning.h)
 */
int harris_coarsity_ex(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale,
                       int window, float* out, const harris_tuning* tuning, void* stream);

/*
 * Distances between rows, planes and images, for images that are not dense: padded
 * rows (the thesis rounds rows up to the vector width, section 4.3 "Vectorisation"), a
 * region of interest inside a larger image, planes or images kept apart.  Element
 * (h, w) of plane c of image b is at rgb[b*rgb_image_pitch + c*rgb_plane_pitch +
 * h*rgb_row_pitch + w] (in input elements) and result (y, x) of image b at
 * out[b*out_image_pitch + y*out_row_pitch + x] (in floats).  Requirements, else
 * HARRIS_ERR_SHAPE: rgb_row_pitch >= W, rgb_plane_pitch >= (H-1)*rgb_row_pitch + W,
 * rgb_image_pitch >= 2*rgb_plane_pitch + (H-1)*rgb_row_pitch + W, out_row_pitch >= W-4,
 * out_image_pitch >= (H-5)*out_row_pitch + W-4.  Bytes outside the rows are never written.
 * They are never read either, except that rows of uint8 input that do not start on 4-byte
 * boundaries are loaded as the aligned 32-bit words that hold them: up to 3 bytes before a
 * row's first and after its last element may be read (never beyond those words) and are
 * discarded.
 */
typedef struct harris_layout {
    long long rgb_row_pitch, rgb_plane_pitch, rgb_image_pitch;
    long long out_row_pitch, out_image_pitch;
} harris_layout;

/*
 * harris_coarsity_ex for pitched images.  layout == NULL means dense.  Any pointers and
 * pitches the element types allow run with four pixels per lane; rows that all start on
 * 16-byte multiples (pointers and pitches, W % 4 == 0) also get moved strip borders
 * (see harris_tuning.h), worth a few percent.  `tuning` as in harris_coarsity_ex.
 */
int harris_coarsity_pitched(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
                            float k, float sobel_scale, int window, float* out,
                            const harris_tuning* tuning, void* stream);

/* Element type of the result. */
typedef enum harris_out_dtype {
    HARRIS_OUT_F32 = 0,      /* float32, as the thesis's pipeline produces it                     */
    HARRIS_OUT_F16 = 1,      /* IEEE binary16                                                     */
    HARRIS_OUT_BF16 = 2,     /* bfloat16                                                          */
    HARRIS_OUT_U8 = 3        /* 8-bit codes; only through harris_coarsity_quantized               */
} harris_out_dtype;

/*
 * harris_coarsity_pitched with a choice of result type, to cut the 4 bytes per pixel that the
 * float32 result costs (the thesis's arrays are all float32, section 4.2; this is an extension).
 * The coarsity is computed in float32 exactly as by the other entry points and rounded to the
 * result type when it is stored: to nearest, ties to even, values beyond the largest finite
 * number to infinity (binary16 overflows from 65520 on: with sobel_scale 1 and inputs in [0, 1]
 * results stay below that; larger inputs may not).
 *   out        device, element type given by out_dtype (HARRIS_OUT_F32, _F16 or _BF16), [batch][H-4][W-4]
 *              with the pitches of `layout` counted in result elements; fully overwritten
 *   tuning     as in harris_coarsity_ex, but 16-bit results exist only in the tile schedule
 *              (else HARRIS_ERR_ARG)
 * Four pixels per lane need 16-bit result rows that start on 4-byte boundaries (pointer and
 * pitches) and an even W, so that no 32-bit word of a store holds the last column of a row
 * together with something behind it; other shapes run with one pixel per lane.
 */
int harris_coarsity_typed(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
                          float k, float sobel_scale, int window, void* out, int out_dtype,
                          const harris_tuning* tuning, void* stream);

/*
 * 8-bit result, 1 byte per pixel instead of 4: every coarsity value v (float32, computed as by
 * the other entry points) is stored as the code
 *     clamp(round_to_nearest_even(fma(v, q_scale, q_offset)), 0, 255)
 * with the multiply-add rounded once, in float32; NaN gives 0.  (An extension: the thesis's
 * arrays are float32 and it defines no such code; q_scale and q_offset are the caller's.)
 *   out   device, uint8 [batch][H-4][W-4], pitches of `layout` in bytes; fully overwritten
 * Tile schedule only (else HARRIS_ERR_ARG), q_scale and q_offset finite (else HARRIS_ERR_ARG).
 * The fastest path needs 4-byte aligned result rows and W % 4 == 0.
 */
int harris_coarsity_quantized(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
                              float k, float sobel_scale, int window, float q_scale, float q_offset,
                              uint8_t* out, const harris_tuning* tuning, void* stream);

/*
 * The same result computed by several kernels that keep their intermediate images in
 * device memory: the kernel groupings of the thesis's chapter 3, section "Explicit Kernel
 * Execution", subsection "Evaluating the Boilerplate Avoided through Kernel Execution"
 * (table "Four different kernel groupings"), each preceded by a grayscale kernel.
 *   grouping 1  [Sx] [Sy] [x] [+] [coarsity], one kernel per operator and image (10 launches)
 *   grouping 2  [Sx, Sy, x] [+, coarsity]
 *   grouping 3  [Sx, Sy] [x, +, coarsity]
 *   grouping 4  one fused kernel: identical to harris_coarsity_ex without tuning
 * These are untuned baselines for measuring what fusion buys, and a second
 * implementation to cross-check the fused kernels; arguments as harris_coarsity_ex, plus
 *   workspace        device memory for the intermediates, 4-byte aligned, owned by the
 *                    caller, contents undefined afterwards; may be NULL for grouping 4
 *   workspace_bytes  its size; at least harris_grouped_workspace_bytes(...) or
 *                    HARRIS_ERR_ARG.  batch must not exceed 65535 for groupings 1-3.
 */
int harris_coarsity_grouped(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale,
                            int window, int grouping, void* workspace, long long workspace_bytes,
                            float* out, void* stream);

/* Workspace bytes harris_coarsity_grouped needs; 0 for grouping 4; -1 for invalid arguments. Host only. */
long long harris_grouped_workspace_bytes(int grouping, int batch, int H, int W);

/*
 * harris_coarsity_grouped (groupings 1-3) for callers that cannot allocate and have no
 * workspace to bring: code under HIP stream capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The intermediate images live in a fixed array of HARRIS_GROUPED_SCRATCH_BYTES that
 * is part of the library's device code (each GPU the library runs on holds it until the process
 * ends); this call allocates and frees nothing, on the host or on the device.
 *   - The problem must fit: harris_grouped_workspace_bytes(grouping, batch, H, W) <=
 *     HARRIS_GROUPED_SCRATCH_BYTES (64 MiB: grouping 3 up to about 5.5 million pixels per call,
 *     grouping 2 up to 4.1 million, e.g. one 1536 x 2560 image, grouping 1 up to 1.8 million),
 *     else HARRIS_ERR_SCRATCH and nothing is enqueued.  Grouping 4 needs no intermediates and
 *     takes any size.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different
 *     streams, or one stream and a replaying graph) race on it and must be serialised by the
 *     caller.  Nothing in it needs clearing: every kernel writes the intermediates it produces
 *     completely before a later kernel reads them, whatever an earlier call left there.
 *   - The device whose stream is given must be the current device of the calling thread.  The
 *     first call on a device looks up the array's address there (and, like any first launch,
 *     lets the runtime load the library's device code): make it outside stream capture.
 * Other arguments, results and errors as harris_coarsity_grouped.
 */
#define HARRIS_GROUPED_SCRATCH_BYTES (64u << 20)
int harris_coarsity_grouped_static(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale,
                                   int window, int grouping, float* out, void* stream);

/* Static, NUL-terminated description of a harris_status value. */
const char* harris_strerror(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int harris_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HARRIS_H */
