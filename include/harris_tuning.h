/*
 * libharris: launch shapes, planning and measurement aids.
 *
 * Not needed to use the operator (harris.h): these declarations let a benchmark or a test
 * choose the launch shape of the fused kernel, ask which shape the library would choose, and
 * time a plain streaming copy with the operator's traffic.  The names of the kernel's knobs
 * may change between versions; the entry points of harris.h do not.
 */
#ifndef HARRIS_TUNING_H
#define HARRIS_TUNING_H

#include "harris.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional launch shape, for benchmarking and tests.  Pass NULL (or zero fields)
 * to let the library choose.  Results never depend on it beyond rounding.
 *
 *   schedule  HARRIS_SCHEDULE_BANDS: one wavefront walks a band of `rows` result rows of
 *             one strip from top to bottom (or bottom to top), with `prefetch` input rows
 *             in flight.  HARRIS_SCHEDULE_TILES: a workgroup of `waves_per_block`
 *             wavefronts loads a tile of waves_per_block * rows input rows at once and
 *             hands the gray rows that two wavefronts share through LDS.  0 = chosen
 *             from the size.
 *   px        pixels per lane along x: 1, 2 or 4.  A lane's loads and stores
 *             must be naturally aligned in every row (px divides W, pointers and pitches are
 *             multiples of the access size), else HARRIS_ERR_ARG; except that TILES with px = 4
 *             takes any width and any row alignment the element type allows, as long as result
 *             rows start on 4-byte boundaries, are not 8-bit codes and, if 16-bit, have an even
 *             number of columns (vector accesses on 4-byte boundaries; 8-bit input rows on any
 *             byte are loaded as aligned words and shifted).  0 = 4 where that holds, else the
 *             widest of 2, 1 that fits.
 *   rows      BANDS: result rows per band (>= 1).  TILES: input rows per wavefront: 4, and
 *             with px = 4 also 5, 6, 8, 9 or 10 (4 or 8 for 8-bit input rows off 4-byte
 *             boundaries).  0 = chosen from the size.
 *   prefetch  BANDS only: input rows kept in flight per wavefront: 3 (0 = the same).  A
 *             non-zero value with schedule 0 selects BANDS.
 *   waves_per_block  BANDS: 1, 2 or 4 (2: two bands of a strip that start on shared rows;
 *             4: the same for two adjacent strips).  TILES: 2 to 16.  0 = default.
 *   flags     HARRIS_TUNE_* bits.
 *   lds_kb    TILES only: kilobytes of LDS to reserve per workgroup, 0 to 64.  A tile needs 4 KB
 *             per wavefront (px = 4); reserving more bounds the workgroups resident on a CU
 *             (160 KB of LDS per CU: 64 -> 2, 48 -> 3, 36 -> 4, 28 -> 5).  Many-tile float32
 *             launches are faster with 10 to 16 wavefronts per CU in flight than with the 28 to
 *             32 that the registers would allow.  0 = chosen from the size (plans report the
 *             reservation in force, at least the tile's own need).
 */
struct harris_tuning {
    int schedule;
    int px;
    int rows;
    int prefetch;
    int waves_per_block;
    unsigned flags;
    int lds_kb;
};

#define HARRIS_SCHEDULE_BANDS 1
#define HARRIS_SCHEDULE_TILES 2

#define HARRIS_TUNE_NO_ALTERNATE 1u  /* BANDS: all bands walk downwards (default: odd bands walk
                                        upwards, so that neighbouring bands read their shared rows
                                        at the same time)                                            */
#define HARRIS_TUNE_NO_XCD_REMAP 2u  /* workgroup i takes tile group i (default: tiles are dealt so
                                        that each of the 8 XCDs gets one contiguous run of tiles)   */
#define HARRIS_TUNE_CACHED_LOADS 4u  /* load input rows with the default cache policy             */
#define HARRIS_TUNE_STREAM_LOADS 8u  /* load input rows non-temporal.  With neither bit the library
                                        decides from the size of the problem                        */
#define HARRIS_TUNE_KEEP_SHARED_ROWS 64u /* TILES with px = 4 and non-temporal loads only: the input rows
                                        that two vertically adjacent tiles both read (the first and the
                                        last four of a tile) are loaded with the default policy instead,
                                        so that the second reader finds them in L2                   */
#define HARRIS_TUNE_FLAG_HANDOFF 128u /* TILES with px = 4, float32 input and plain non-temporal loads
                                        only: a wavefront
                                        waits for a ready flag of the wavefront below it instead of
                                        the workgroup's barrier (and a barrier holds the stores back
                                        until the workgroup's loads are in): for few, large tiles     */
#define HARRIS_TUNE_ALIGNED_STORES 16u /* TILES with px = 4 and naturally aligned lanes only: in every result row the border between
                                        two strips is moved right to the next 64-byte boundary of the
                                        row's address, so that no 64-byte block of the result is
                                        written by two wavefronts; strips are then at most 240
                                        columns wide instead of 252                                 */
#define HARRIS_TUNE_PLAIN_STORES 32u /* strips end at the same column in every row.  With neither bit
                                        the library decides                                         */

/*
 * The launch shape harris_coarsity_ex would use for this problem (after applying
 * `tuning`, which may be NULL), written to *chosen; also the number of workgroups
 * in *n_blocks if n_blocks is not NULL.  rgb_align / out_align are the byte
 * alignments of the base pointers (pass 16 for ordinary allocations).  Host only;
 * touches no device.  Returns a harris_status.
 */
int harris_plan(int dtype, int batch, int H, int W, int rgb_align, int out_align,
                const harris_tuning* tuning, harris_tuning* chosen, long long* n_blocks);

/* The same for harris_coarsity_typed: out_dtype is a harris_out_dtype. */
int harris_plan_typed(int dtype, int out_dtype, int batch, int H, int W, int rgb_align, int out_align,
                      const harris_tuning* tuning, harris_tuning* chosen, long long* n_blocks);

/*
 * Measurement aid, not the Harris operator: a plain streaming kernel with the traffic of one
 * Harris launch.  For every image it reads the first (H-4)*(W-4) elements of each of the three
 * planes (taken as flat arrays) and writes their sum as float32 to out[b][i]: 3*e + 4 bytes per
 * result pixel, e = 4 or 1, against the 3*e*H*W + 4*(H-4)*(W-4) of the operator.  Its duration
 * beside harris_coarsity's shows what this read/write mix reaches on the GPU at hand.
 * Requires dense arrays, 16-byte aligned rgb and out, H*W*e and (H-4)*(W-4)*4 multiples of 16,
 * batch <= 65535 (else HARRIS_ERR_ARG / HARRIS_ERR_SHAPE); arguments otherwise as harris_coarsity.
 */
int harris_probe_copy(const void* rgb, int dtype, int batch, int H, int W, float* out, void* stream);

/*
 * Measurement aid: a pure stream of `bytes` bytes, for the ceilings of reads alone and of writes
 * alone beside harris_probe_copy's mix.
 *   kind HARRIS_PROBE_READ   every byte of src[0 .. bytes) is loaded once (16 bytes per lane,
 *                            non-temporal) and nothing is stored; dst must point to at least 4
 *                            writable bytes (a sink that keeps the loads alive and stays untouched).
 *   kind HARRIS_PROBE_WRITE  every byte of dst[0 .. bytes) is written once with a pattern of no
 *                            meaning; src is ignored.
 *   kind HARRIS_PROBE_NONE   a launch of 256 workgroups of 256 threads that touch no memory: what
 *                            the GPU needs for a kernel launch by itself (many of them in a
 *                            captured graph give the period that the host's launch rate does not
 *                            bound).  src, dst and bytes (>= 0) are ignored and may be NULL and 0.
 * src and dst are device pointers, 16-byte aligned, bytes a multiple of 16 (else HARRIS_ERR_ARG);
 * bytes == 0 succeeds without work (kinds READ and WRITE).
 */
#define HARRIS_PROBE_READ 1
#define HARRIS_PROBE_WRITE 2
#define HARRIS_PROBE_NONE 3
int harris_probe_stream(int kind, const void* src, void* dst, long long bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HARRIS_TUNING_H */
