// Device code of the fused Harris coarsity kernels for gfx950 (MI355X): included by the
// translation units that instantiate them (harris_tiles_f32.hip, harris_tiles_u8.hip,
// harris_bands.hip), never by host-only code.
//
// One kernel computes every stage of the Harris operator (thesis chapter 4,
// section 4.2: grayscale, Sobel pair, products, 3x3 window sums, coarsity) and
// touches device memory only to read the RGB planes once and to write the result
// once.  The schedule is this library's own; what it keeps from the thesis's
// section 4.3 is the idea of a pipeline over image lines with separated 3x3
// kernels and rotating registers, re-cut for a 64-lane wavefront:
//
//  * A wavefront owns a vertical strip of the image.  Lane l holds PX adjacent
//    columns; one row of one plane is a single coalesced load of 64*PX elements
//    (128 bits per lane for float32 at PX = 4).
//  * Vertical taps never touch memory: the last two gray rows and the last two
//    rows of (Ix^2, Ix*Iy, Iy^2) live in registers ("register rotation").  Row steps
//    are unrolled, so the rotation is a renaming, not a copy.
//  * Both 3x3 stages are separated (section 4.3, "Convolution Separation"):
//    [1 2 1]^T/[-1 0 1]^T down the column from registers first, then the horizontal
//    taps.  Horizontal neighbours come from the lane to the right through a DPP
//    wave shift; each stage consumes two columns from the right, so a lane's
//    output columns start at the lane's own first input column and the result row
//    is stored with aligned vector stores.
//  * The strip of a wavefront overlaps its right neighbour by the 4-column halo;
//    the last lane(s) only supply that halo.
//
// Two schedules run this pipeline:
//  * Tiles (the default, harris_tile_kernel): a workgroup of NW wavefronts takes NW*RW
//    input rows of one strip; every wavefront requests its RW rows at once, hands its
//    first four gray rows to the wavefront above through LDS (one barrier), and
//    stores its RW result rows in one burst at the end.
//  * Bands (harris_fused_kernel): one long-lived wavefront walks a band of R result
//    rows with a register queue of D input rows in flight; no LDS, no barrier.  Odd
//    bands walk upwards, so two neighbouring bands begin on the rows they share.
// In both, tiles are dealt to workgroups so that each XCD (own L2) gets one
// contiguous run of tiles.
#ifndef HARRIS_KERNELS_H
#define HARRIS_KERNELS_H

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <type_traits>

#include "harris_tuning.h"
#include "harris_launch.h"

namespace {

constexpr int kWave = 64;

// ---------------------------------------------------------------- small helpers

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int gcd_c(int a, int b) { return b == 0 ? a : gcd_c(b, a % b); }
constexpr int lcm_c(int a, int b) { return a / gcd_c(a, b) * b; }

// Value of v in the lane to the right (lane + 1); lanes without one get 0.
// DPP control 0x130 is "wave shift left by 1": lane i reads lane i + 1.
__device__ __forceinline__ float from_right(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, true));
}

// The two columns to the right of a lane's PX columns: a[PX], a[PX+1].
template <int PX>
__device__ __forceinline__ void fetch_halo(float (&a)[PX + 2]) {
    if constexpr (PX == 1) {
        a[1] = from_right(a[0]);
        a[2] = from_right(a[1]);
    } else {
        a[PX] = from_right(a[0]);
        a[PX + 1] = from_right(a[1]);
    }
}

// ---------------------------------------------------------------- row loads and stores

// Cache policy of the accesses (the "aux" operand of the buffer instructions): bit 0 = sc0,
// bit 1 = nt (non-temporal), bit 4 = sc1.  0 is the default policy.  Results are never read
// back, so they are always stored non-temporal.  Input rows are loaded non-temporal when the
// whole problem fits the last-level cache anyway, and with the default policy otherwise: then
// the line that two neighbouring strips share, and the rows that two neighbouring
// bands share, are found in the CU's vector cache by the second wavefront of the
// same workgroup.
// The policies are compile-time constants of the instructions; the macros exist so that a build
// with other values can be timed against this one.  Measured (us, interleaved runs on one GPU):
//   stores nt + sc1 (written through at device scope) instead of nt, many small tiles:
//     8192x8192 uint8 83.1 against 84.8, 2832x4256 32.6 / 32.9, 64x1080x1920 351.9 / 353.9;
//     one tile per CU, 1536x2560: 12.7 against 12.0 -- so only the many-tile kernels take it;
//   default-policy stores: 13.4 (1536x2560), 97.6 (8192x8192 uint8), 39.8 (2832x4256);
//   loads nt + sc1: 12.8 on 1536x2560, no change on the large workloads; sc1 without nt, or
//     sc1 on the rows two tiles share: 4 to 22 % slower.
#ifndef HARRIS_LOAD_AUX
#define HARRIS_LOAD_AUX 2
#endif
#ifndef HARRIS_STORE_AUX
#define HARRIS_STORE_AUX 2
#endif
#ifndef HARRIS_MANY_STORE_AUX
#define HARRIS_MANY_STORE_AUX 18
#endif
constexpr int kAuxDefault = 0;
constexpr int kAuxNonTemporal = HARRIS_LOAD_AUX;
// Tile kernel only, not a hardware value: non-temporal, except that the first and the last
// four input rows of a tile, which the tile above or below reads as well, are loaded with the
// default policy.  The launches that use it are those of many small tiles; their stores are
// written through (kAuxManyStore).
constexpr int kAuxKeepShared = -1;
constexpr int kAuxStore = HARRIS_STORE_AUX, kAuxManyStore = HARRIS_MANY_STORE_AUX;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Buffer descriptor over `bytes` bytes at p: raw (unstrided) 32-bit data.  A lane
// whose byte offset is not below `bytes` loads 0 and stores nothing.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// One row segment of the three planes as raw 32-bit words, PX pixels per lane.
template <typename In, int PX>
struct RawRow {
    static constexpr int NW = std::is_same<In, float>::value ? PX : (PX + 3) / 4;
    uint32_t w[3][NW];
};

// row points at column 0 of the row in plane 0; voff is the lane's byte offset in the row.
template <typename In, int PX, int AUX>
__device__ __forceinline__ void load_row(RawRow<In, PX>& r, const In* row, size_t plane, uint32_t row_bytes, uint32_t voff) {
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(row + c * plane, row_bytes);
        constexpr int BYTES = PX * (int)sizeof(In);
        if constexpr (BYTES >= 16) {
#pragma unroll
            for (int j = 0; j < BYTES / 16; ++j) {
                u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 16 * j, 0, AUX);
                r.w[c][4 * j + 0] = v.x; r.w[c][4 * j + 1] = v.y; r.w[c][4 * j + 2] = v.z; r.w[c][4 * j + 3] = v.w;
            }
        } else if constexpr (BYTES == 8) {
            u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, 0, AUX);
            r.w[c][0] = v.x; r.w[c][1] = v.y;
        } else if constexpr (BYTES == 4) {
            r.w[c][0] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, 0, AUX);
        } else if constexpr (BYTES == 2) {
            r.w[c][0] = __builtin_amdgcn_raw_buffer_load_b16(rs, voff, 0, AUX);
        } else {
            r.w[c][0] = __builtin_amdgcn_raw_buffer_load_b8(rs, voff, 0, AUX);
        }
    }
}

// 8-bit rows that start on any byte, four pixels per lane: every lane loads the aligned 32-bit
// word at its offset from the row's address rounded down to 4 bytes, so no access is
// misaligned and none leaves the aligned words that hold the row's bytes.  With the row
// starting `shift` bytes into its first word, a lane's four pixels are the upper bytes of its
// word and the lower bytes of the word of the lane to its right (realign_row).
// voff is the lane's first column (a multiple of 4); shift[c] is kept for realign_row.
template <int AUX>
__device__ __forceinline__ void load_row_shifted(RawRow<uint8_t, 4>& r, uint32_t (&shift)[3], const uint8_t* row, size_t plane,
                                                 uint32_t row_bytes, uint32_t voff) {
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(row + c * plane);
        shift[c] = (uint32_t)a & 3u;
        const uint32_t bytes = row_bytes ? (row_bytes + shift[c] + 3u) & ~3u : 0u;
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(reinterpret_cast<const void*>(a & ~(uintptr_t)3), bytes);
        r.w[c][0] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, 0, AUX);
    }
}

__device__ __forceinline__ void realign_row(RawRow<uint8_t, 4>& r, const uint32_t (&shift)[3]) {
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const uint32_t own = r.w[c][0];
        const uint32_t right = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0x130, 0xf, 0xf, true);
        r.w[c][0] = __builtin_amdgcn_alignbyte(right, own, shift[c]);
    }
}

// PX results of one lane to a result row described by rs (its size is the row's
// bytes, or 0 to store nothing); voff is the lane's byte offset in the row.
template <int PX, int AUX = kAuxStore>
__device__ __forceinline__ void store_row(const float (&o)[PX], __amdgpu_buffer_rsrc_t rs, uint32_t voff) {
    if constexpr (PX >= 4) {
#pragma unroll
        for (int j = 0; j < PX / 4; ++j) {
            u32x4 v = {__float_as_uint(o[4 * j]), __float_as_uint(o[4 * j + 1]), __float_as_uint(o[4 * j + 2]), __float_as_uint(o[4 * j + 3])};
            __builtin_amdgcn_raw_buffer_store_b128(v, rs, voff + 16 * j, 0, AUX);
        }
    } else if constexpr (PX == 2) {
        u32x2 v = {__float_as_uint(o[0]), __float_as_uint(o[1])};
        __builtin_amdgcn_raw_buffer_store_b64(v, rs, voff, 0, AUX);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[0]), rs, voff, 0, AUX);
    }
}

// float32 -> bit pattern of the nearest binary16 / bfloat16 value (ties to even, overflow to
// infinity, NaN stays NaN), by the hardware conversions: round-to-nearest-even is the mode
// HIP kernels run in, and gfx950 converts two float32 values to a bfloat16 pair in one
// instruction.
__device__ __forceinline__ uint32_t to_f16_bits(float x) {
    return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)x);
}
__device__ __forceinline__ uint32_t to_bf16_bits(float x) {
    return (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)x);
}
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// Two values in one 32-bit word: lo in bits 0..15, hi in bits 16..31.
template <bool BF>
__device__ __forceinline__ uint32_t to_16bit_pair(float lo, float hi) {
    const f32x2 v = {lo, hi};
    if constexpr (BF) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// PX results of one lane as 16-bit values (BF: bfloat16, else binary16); voff is the lane's
// byte offset in the row (2 bytes per column).
template <int PX, bool BF, int AUX = kAuxStore>
__device__ __forceinline__ void store_row_16(const float (&o)[PX], __amdgpu_buffer_rsrc_t rs, uint32_t voff) {
    if constexpr (PX >= 4) {
#pragma unroll
        for (int j = 0; j < PX / 4; ++j) {
            const u32x2 v = {to_16bit_pair<BF>(o[4 * j], o[4 * j + 1]), to_16bit_pair<BF>(o[4 * j + 2], o[4 * j + 3])};
            __builtin_amdgcn_raw_buffer_store_b64(v, rs, voff + 8 * j, 0, AUX);
        }
    } else if constexpr (PX == 2) {
        __builtin_amdgcn_raw_buffer_store_b32(to_16bit_pair<BF>(o[0], o[1]), rs, voff, 0, AUX);
    } else {
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(BF ? to_bf16_bits(o[0]) : to_f16_bits(o[0])), rs, voff, 0, AUX);
    }
}

// PX results of one lane as 8-bit codes clamp(rint(fma(v, scale, offset)), 0, 255); NaN gives 0.
// The hardware's float-to-byte conversion does the rounding (to nearest, ties to even), the
// clamp and the packing into byte i of a word in one instruction per value.  voff is the
// lane's byte offset in the row (1 byte per column).
template <int PX, int AUX = kAuxStore>
__device__ __forceinline__ void store_row_8(const float (&o)[PX], float scale, float offset, __amdgpu_buffer_rsrc_t rs, uint32_t voff) {
    constexpr int WORDS = (PX + 3) / 4;
    uint32_t w[WORDS];
#pragma unroll
    for (int j = 0; j < WORDS; ++j) w[j] = 0u;
#pragma unroll
    for (int i = 0; i < PX; ++i) w[i / 4] = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(o[i], scale, offset), (uint32_t)(i % 4), w[i / 4]);
    if constexpr (PX >= 4) {
#pragma unroll
        for (int j = 0; j < WORDS; ++j) __builtin_amdgcn_raw_buffer_store_b32(w[j], rs, voff + 4 * j, 0, AUX);
    } else if constexpr (PX == 2) {
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)w[0], rs, voff, 0, AUX);
    } else {
        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)w[0], rs, voff, 0, AUX);
    }
}

// Conversion and grayscale: element i of plane c as float (8-bit values are converted; their
// 1/255 is folded into the gray weights), then gray = wr*R + wg*G + wb*B.
template <typename In, int PX>
__device__ __forceinline__ void gray_row(const RawRow<In, PX>& r, float wr, float wg, float wb, float (&g)[PX]) {
#pragma unroll
    for (int i = 0; i < PX; ++i) {
        float ch[3];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            if constexpr (std::is_same<In, float>::value) ch[c] = __uint_as_float(r.w[c][i]);
            else ch[c] = (float)((r.w[c][i / 4] >> (8 * (i % 4))) & 0xffu);
        }
        g[i] = fmaf(wb, ch[2], fmaf(wg, ch[1], wr * ch[0]));
    }
}

// ---------------------------------------------------------------- the pipeline state of one lane

template <int PX>
struct LineBuffers {
    float g[3][PX];       // ring of the last three gray rows
    float p[3][3][PX];    // ring of the last three rows of (Ix*Ix, Ix*Iy, Iy*Iy)
};

// One row step.  GS is the ring slot that receives this step's gray row.
// STAGE 0: gray only (first two rows of a band); 1: also Sobel and products (next
// two rows); 2: also window sums and coarsity: one result row in o, for the caller to store.
template <int STAGE, int GS, int PX, bool BINOM>
__device__ __forceinline__ void row_step(LineBuffers<PX>& lb, const float (&gc)[PX], float k, float (&o)[PX]) {
    constexpr int PS = (GS + 1) % 3;          // product slot written at this step
#pragma unroll
    for (int i = 0; i < PX; ++i) lb.g[GS][i] = gc[i];
    if constexpr (STAGE >= 1) {
        // Sobel pair, separated: down the column from the register ring, then along the row.
        const float (&ga)[PX] = lb.g[(GS + 1) % 3];   // two rows back
        const float (&gb)[PX] = lb.g[(GS + 2) % 3];   // one row back (the centre row)
        float vs[PX + 2], vd[PX + 2];
#pragma unroll
        for (int i = 0; i < PX; ++i) {
            vs[i] = fmaf(2.0f, gb[i], ga[i] + gc[i]);  // [1 2 1] down the column
            vd[i] = gc[i] - ga[i];                     // [-1 0 1] down the column
        }
        fetch_halo<PX>(vs);
        fetch_halo<PX>(vd);
#pragma unroll
        for (int i = 0; i < PX; ++i) {
            float ix = vs[i + 2] - vs[i];                        // [-1 0 1] along the row
            float iy = fmaf(2.0f, vd[i + 1], vd[i] + vd[i + 2]); // [1 2 1] along the row
            // Products.
            lb.p[PS][0][i] = ix * ix;
            lb.p[PS][1][i] = ix * iy;
            lb.p[PS][2][i] = iy * iy;
        }
    }
    if constexpr (STAGE >= 2) {
        // Window sums, separated: [1 c 1] down the column, then along the row (c = 1 for the
        // unweighted sum, 2 for the binomial window).  Along the row neighbouring results
        // share a pair sum, and every value that comes from the lane to the right is an
        // operand of an addition, so that its lane shift rides on that addition.
        float s[3][PX];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            float v[PX + 2];
#pragma unroll
            for (int i = 0; i < PX; ++i) {
                const float ends = lb.p[(PS + 1) % 3][q][i] + lb.p[PS][q][i];
                const float mid = lb.p[(PS + 2) % 3][q][i];
                v[i] = BINOM ? fmaf(2.0f, mid, ends) : ends + mid;
            }
            fetch_halo<PX>(v);
            if constexpr (BINOM) {
                float pair[PX + 1];                       // v[i] + v[i+1]
#pragma unroll
                for (int i = 0; i <= PX; ++i) pair[i] = v[i + 1] + v[i];
#pragma unroll
                for (int i = 0; i < PX; ++i) s[q][i] = pair[i] + pair[i + 1];   // v[i] + 2 v[i+1] + v[i+2]
            } else if constexpr (PX == 1) {
                s[q][0] = (v[1] + v[0]) + v[2];
            } else {
#pragma unroll
                for (int j = 0; j < PX / 2; ++j) {
                    const float pair = v[2 * j + 2] + v[2 * j + 1];
                    s[q][2 * j] = v[2 * j] + pair;
                    s[q][2 * j + 1] = v[2 * j + 3] + pair;
                }
            }
        }
        // Coarsity.
#pragma unroll
        for (int i = 0; i < PX; ++i) {
            float det = fmaf(s[0][i], s[2][i], -(s[1][i] * s[1][i]));
            float tr = s[0][i] + s[2][i];
            o[i] = fmaf(-(k * tr), tr, det);
        }
    }
}

// ---------------------------------------------------------------- the kernel

// Tiles are numbered image-major, then band, then strip.  Workgroup b of the grid is
// placed on XCD b % 8 by the hardware dispatcher; this gives XCD x the x-th contiguous
// run of workgroup-sized tile groups.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned nb) {
    const unsigned q = nb / 8, r = nb % 8, x = b % 8, j = b / 8;
    return x * q + min(x, r) + j;       // XCDs 0..r-1 take q + 1 groups each, the others q
}

template <typename In, int PX, int D, int LAUX, bool BINOM>
__global__ __launch_bounds__(256) void harris_fused_kernel(const harris_launch::Params p) {
    constexpr int U = lcm_c(3, D);            // row steps per loop trip: ring slots stay static

    const unsigned lane = threadIdx.x % kWave;
    const unsigned wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const unsigned waves_per_block = blockDim.x / kWave;
    unsigned blk = blockIdx.x;
    blk = (p.flags & HARRIS_TUNE_NO_XCD_REMAP) ? blk : xcd_contiguous(blk, p.n_blocks);

    // A workgroup of 2 or 4 wavefronts holds two vertically adjacent bands (of one strip,
    // or of two adjacent strips): band 2j walks upwards and band 2j+1 downwards, so both
    // begin on the four input rows they share, and the second request for those rows (and
    // for the cache line two adjacent strips share) is served by the CU's vector cache.
    const unsigned group_h = waves_per_block >= 2 ? 2u : 1u;
    const unsigned group_w = waves_per_block / group_h;
    const unsigned img = blk / p.blocks_per_image;
    const unsigned rem = blk % p.blocks_per_image;
    const int band = (int)((rem / p.blocks_x) * group_h + wave / group_w);
    const int strip = (int)((rem % p.blocks_x) * group_w + wave % group_w);
    if (band >= (int)p.n_bands || strip >= (int)p.n_strips) return;   // uniform per wavefront; no barrier is ever used

    const int y0 = band * p.rows_per_band;                      // first result row of the band
    const int rows = min(p.rows_per_band, p.n - y0);            // result rows of this band (>= 1)
    const int steps = rows + 4;                                 // input rows consumed
    const bool up = !(p.flags & HARRIS_TUNE_NO_ALTERNATE) && !(band & 1);

    // A strip yields p.strip_pitch result columns (at most 64*PX - 4, the same for every
    // strip so that all wavefronts carry the same load); the lanes beyond only supply halo.
    const unsigned col = (unsigned)strip * p.strip_pitch + lane * PX; // first column of this lane (input and result)
    const unsigned lcol = min(col, (unsigned)(p.W - PX));       // loads stay inside the row
    // Lanes beyond the strip's columns and its 4-column halo request nothing (out-of-range offset).
    const uint32_t load_voff = lane * PX < p.strip_pitch + 4 ? lcol * (uint32_t)sizeof(In) : 0x80000000u;
    // Halo-only lanes store nothing: an offset beyond any row.  Lanes whose columns lie
    // right of the result row are dropped by the buffer's range check.
    const uint32_t store_voff = lane * PX < p.strip_pitch ? col * 4u : 0x80000000u;
    const uint32_t in_row_bytes = (uint32_t)p.W * (uint32_t)sizeof(In);
    const uint32_t out_row_bytes = (uint32_t)p.m * 4u;

    const size_t plane = (size_t)p.in_plane_pitch;
    const In* img_in = static_cast<const In*>(p.rgb) + (size_t)img * (size_t)p.in_image_pitch;
    float* img_out = static_cast<float*>(p.out) + (size_t)img * (size_t)p.out_image_pitch;   // float32 results only

    // Input row read at step t.  Steps past the band's end (the loop runs in trips of U
    // steps, and the queue reads D rows ahead) get an empty descriptor: such a load
    // returns zeros and moves no data.
    auto in_row_ptr = [&](int t) -> const In* {
        int r = up ? y0 + rows + 3 - t : y0 + t;
        r = max(0, min(p.H - 1, r));
        return img_in + (size_t)r * (size_t)p.in_row_pitch;
    };
    auto in_row_size = [&](int t) -> uint32_t { return t < steps ? in_row_bytes : 0u; };

    RawRow<In, PX> queue[D];
    static_for<0, D>([&](auto d) {
        constexpr int dd = decltype(d)::value;
        load_row<In, PX, LAUX>(queue[dd], in_row_ptr(dd), plane, in_row_size(dd), load_voff);
        __builtin_amdgcn_sched_barrier(0);
    });

    LineBuffers<PX> lb;
    float gc[PX], o[PX];

    // Rows 0..3 of the band fill the pipeline.
    static_for<0, 4>([&](auto tt) {
        constexpr int t = decltype(tt)::value;
        gray_row<In, PX>(queue[t % D], p.wr, p.wg, p.wb, gc);
        __builtin_amdgcn_sched_barrier(0);
        load_row<In, PX, LAUX>(queue[t % D], in_row_ptr(t + D), plane, in_row_size(t + D), load_voff);
        __builtin_amdgcn_sched_barrier(0);
        row_step<(t < 2 ? 0 : 1), t % 3, PX, BINOM>(lb, gc, p.k, o);
    });

    for (int t0 = 4; t0 < steps; t0 += U) {
        static_for<0, U>([&](auto uu) {
            constexpr int u = decltype(uu)::value;
            const int t = t0 + u;
            // The slot's registers are free as soon as its gray row exists: refill it at
            // once, so that D rows stay in flight while the rest of the step computes.
            gray_row<In, PX>(queue[(4 + u) % D], p.wr, p.wg, p.wb, gc);
            __builtin_amdgcn_sched_barrier(0);
            load_row<In, PX, LAUX>(queue[(4 + u) % D], in_row_ptr(t + D), plane, in_row_size(t + D), load_voff);
            __builtin_amdgcn_sched_barrier(0);
            // Result row: the top row of the 5-row window that this step completes.  Steps
            // past the band's end get an empty descriptor and store nothing.
            const int orow = max(0, min(p.n - 1, up ? y0 + rows + 3 - t : y0 + t - 4));
            const __amdgpu_buffer_rsrc_t out_rs = make_rsrc(img_out + (size_t)orow * (size_t)p.out_row_pitch, t < steps ? out_row_bytes : 0u);
            row_step<2, (4 + u) % 3, PX, BINOM>(lb, gc, p.k, o);
            store_row<PX>(o, out_rs, store_voff);
        });
    }
}


// Makes the compiler finish these values here: without it the last multiply-add of a result
// is moved down to the stores, and its three operands stay in registers instead of the one
// result (the tile kernel holds RW rows of results until its store burst).
template <int PX>
__device__ __forceinline__ void pin_values(float (&v)[PX]) {
#pragma unroll
    for (int i = 0; i < PX; ++i) asm volatile("" : "+v"(v[i]));
}

// ---------------------------------------------------------------- the tile kernel
//
// The default schedule: a
// workgroup of NW wavefronts owns a tile of NW*RW input rows of one strip, and every
// wavefront requests its RW rows (3*RW loads) at once, so no wavefront goes through a
// chain of dependent memory round trips.  Wavefront w turns its rows into gray,
// publishes its first four gray rows in LDS and, after one barrier, takes the four
// gray rows below its own from wavefront w+1 there: nothing is read twice inside a
// tile.  Each wavefront then runs the same register pipeline as the band kernel over
// its RW+4 gray rows and stores RW result rows (the last wavefront has no neighbour
// below and stores RW-4).  A tile yields NW*RW-4 result rows; the tile below re-reads
// four rows.
//
// HANDOFF selects how a wavefront learns that the rows below its own are in LDS.  false: the
// workgroup's barrier, after every wavefront has worked through its own rows.  true: a ready
// flag per wavefront in LDS, set as soon as its first four gray rows are written; a wavefront
// waits only for the flag of the one below it, and a barrier before the store burst keeps the
// stores behind the workgroup's loads.  With one large tile per CU the last wavefront's data
// arrives long after the first's, and without the flags every wavefront's last four rows would
// wait for it and then be computed by all at once (1536x2560: 12.2 against 12.4 us); with many
// small tiles the barrier is faster (720x1280: 6.1 against 6.4 us).
//
// SHIFTED (8-bit input, four pixels per lane): rows start on any byte and are loaded as the
// aligned 32-bit words that hold them (load_row_shifted, realign_row).
template <typename In, int PX, int RW, int LAUX, bool BINOM, bool HANDOFF, bool SHIFTED = false>
__global__ __launch_bounds__(1024) void harris_tile_kernel(const harris_launch::Params p) {
    static_assert(!SHIFTED || (std::is_same<In, uint8_t>::value && PX == 4), "shifted rows: 8-bit input, four pixels per lane");
    extern __shared__ __align__(16) float halo_lds[];           // [NW][4][64][PX]
    __shared__ unsigned ready[16];                              // HANDOFF: wavefront w has published its four rows

    const unsigned lane = threadIdx.x % kWave;
    const unsigned wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    if constexpr (HANDOFF) {
        // Every flag is cleared before any wavefront can look at one (the barrier orders the
        // clearing stores before every later access of the workgroup).  At this point the
        // wavefronts of a workgroup are a few hundred cycles apart: the barrier costs nothing measurable.
        if (lane == 0) __hip_atomic_store(&ready[wave], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __syncthreads();
    }
    const unsigned n_waves = p.waves_per_block;                 // == blockDim.x / 64
    unsigned tile = blockIdx.x;
    // The grid size is read with all other arguments, not in a branch of its own: one wait
    // for the arguments instead of two before the first load can be issued.
    unsigned n_blocks = p.n_blocks;
    asm volatile("" : "+s"(n_blocks));
    tile = (p.flags & HARRIS_TUNE_NO_XCD_REMAP) ? tile : xcd_contiguous(tile, n_blocks);
    // The grid has p.n_blocks == n_tiles workgroups: every workgroup has a tile and every
    // wavefront reaches the barrier.

    const unsigned img = harris_launch::fastdiv(tile, p.by_tiles_per_image);
    const unsigned rem = tile - img * p.tiles_per_image;
    const int band = (int)harris_launch::fastdiv(rem, p.by_n_strips);
    const int strip = (int)(rem - (unsigned)band * p.n_strips);

    const int tile_rows = p.rows_per_band;                      // result rows per tile: NW*RW - 4
    const int y_wave = band * tile_rows + (int)wave * RW;       // first input row = first result row of this wavefront
    const int y_end = min(p.n, (band + 1) * tile_rows);         // result rows of this tile end here
    const int out_rows = max(0, min(RW, y_end - y_wave));       // result rows this wavefront stores

    const unsigned col = (unsigned)strip * p.strip_pitch + lane * PX;
    // Lanes right of the row load what the last lane with a column of the row loads (nobody
    // uses what they compute).  That lane may straddle the end of the row (a width that is no
    // multiple of PX): it gets zeros for the words beyond the end, since each 32-bit word of a
    // load is checked against the descriptor's size by itself.
    const unsigned lcol = min(col, ((unsigned)p.W - 1u) & ~(unsigned)(PX - 1));
    // Results are float32, 16-bit or 8-bit: esh is log2 of a result element's bytes.
    const unsigned esh = p.out_kind == HARRIS_OUT_F32 ? 2u : p.out_kind == HARRIS_OUT_U8 ? 0u : 1u;
    // With aligned stores the border between this strip and the next lies, in each result row,
    // on the first 64-byte boundary of that row's address at or after the nominal border: up to
    // 12 (float32), 28 (16-bit) or 60 (8-bit) columns further right.  border_mask is the number
    // of columns per 64 bytes, minus one (15, 31 or 63), or 0.
    const unsigned border_mask = (p.flags & HARRIS_TUNE_ALIGNED_STORES) ? (64u >> esh) - 1u : 0u;
    const unsigned x0 = (unsigned)strip * p.strip_pitch;        // first result column of this strip
    // Lanes beyond the strip's columns, the border's reach and the 4-column halo request nothing
    // (out-of-range offset).
    const uint32_t load_voff = lane * PX < p.strip_pitch + 4 + (border_mask & ~3u) ? lcol * (uint32_t)sizeof(In) : 0x80000000u;
    const uint32_t in_row_bytes = (uint32_t)p.W * (uint32_t)sizeof(In);

    const size_t plane = (size_t)p.in_plane_pitch;
    const In* img_in = static_cast<const In*>(p.rgb) + (size_t)img * (size_t)p.in_image_pitch;
    const uintptr_t img_out = reinterpret_cast<uintptr_t>(p.out) + (((size_t)img * (size_t)p.out_image_pitch) << esh);

    // All RW rows of this wavefront at once; rows below the image get an empty descriptor.
    RawRow<In, PX> raw[RW];
    [[maybe_unused]] uint32_t shift[RW][3];                     // SHIFTED: byte offset of each row in its first word
    // Shifted rows: every lane within reach loads the word at its own column (one lane further
    // right than otherwise, which supplies the last lane's missing bytes); the descriptor's
    // size stops the lanes right of the row.
    [[maybe_unused]] const uint32_t shifted_voff = lane * PX < p.strip_pitch + 8 ? col : 0x80000000u;
    static_for<0, RW>([&](auto tt) {
        constexpr int t = decltype(tt)::value;
        const int r = y_wave + t;
        const In* row_in = img_in + (size_t)min(r, p.H - 1) * (size_t)p.in_row_pitch;
        const uint32_t row_bytes = r < p.H ? in_row_bytes : 0u;
        if constexpr (SHIFTED) {
            if constexpr (LAUX == kAuxKeepShared) {
                const bool shared = (t < 4 && wave == 0) || (t >= RW - 4 && wave + 1 == n_waves);
                if (shared) load_row_shifted<kAuxDefault>(raw[t], shift[t], row_in, plane, row_bytes, shifted_voff);
                else load_row_shifted<kAuxNonTemporal>(raw[t], shift[t], row_in, plane, row_bytes, shifted_voff);
            } else {
                load_row_shifted<LAUX>(raw[t], shift[t], row_in, plane, row_bytes, shifted_voff);
            }
        } else if constexpr (LAUX == kAuxKeepShared) {
            const bool shared = (t < 4 && wave == 0) || (t >= RW - 4 && wave + 1 == n_waves);
            if (shared) load_row<In, PX, kAuxDefault>(raw[t], row_in, plane, row_bytes, load_voff);
            else load_row<In, PX, kAuxNonTemporal>(raw[t], row_in, plane, row_bytes, load_voff);
        } else {
            load_row<In, PX, LAUX>(raw[t], row_in, plane, row_bytes, load_voff);
        }
    });
    __builtin_amdgcn_sched_barrier(0);

    // Descriptors of the RW result rows, worked out while the loads are in flight (scalar
    // arithmetic that would otherwise sit between the last result and the first store).
    // Result row j of this wavefront is row y_wave + j; rows past the tile or the image get
    // an empty descriptor, whose address is never used.  The descriptor covers this strip's
    // columns [b0, b1) of the row; a lane's offset is relative to b0 and wraps to a huge
    // value for lanes left of it, so lanes outside store nothing.
    __amdgpu_buffer_rsrc_t out_rs[RW];
    uint32_t out_lead[RW];                                      // byte offset of column x0 from column b0 (<= 0, wrapped)
    // The empty statement makes everything below depend on values defined after the loads:
    // none of this arithmetic is moved in front of them.
    unsigned sx0 = x0;
    int sy = y_wave;
    asm volatile("" : "+s"(sx0), "+s"(sy) : : "memory");
    const unsigned sx1 = sx0 + p.strip_pitch;
    const uintptr_t out_first = img_out + (((size_t)sy * (size_t)p.out_row_pitch) << esh);
    static_for<0, RW>([&](auto jj) {
        constexpr int j = decltype(jj)::value;
        const uintptr_t row_addr = out_first + (size_t)j * ((size_t)p.out_row_pitch << esh);
        const unsigned a = (unsigned)(row_addr >> esh);         // address in result elements
        const unsigned b0 = sx0 == 0 ? 0u : sx0 + ((0u - (a + sx0)) & border_mask);
        const unsigned b1 = min((unsigned)p.m, sx1 + ((0u - (a + sx1)) & border_mask));
        const uint32_t bytes = (j < out_rows && b1 > b0) ? (b1 - b0) << esh : 0u;
        out_rs[j] = make_rsrc(reinterpret_cast<const void*>(row_addr + ((size_t)b0 << esh)), bytes);
        out_lead[j] = (sx0 - b0) << esh;
        asm volatile("" : "+s"(out_lead[j]));                   // finished here, not next to the store
    });
    uint32_t lane_bytes = (lane * PX) << esh;
    asm volatile("" : "+v"(lane_bytes));
    __builtin_amdgcn_sched_barrier(0);

    LineBuffers<PX> lb;
    float gc[PX], none[PX];
    // The RW result rows stay in registers until the wavefront has used up all its loads and
    // are stored together at the end: bursts of reads and bursts of writes use the memory
    // better than a fine mixture (measured on 1536x2560: 13.0 us against 14.4 us).
    float results[RW][PX];
    float* my_halo = halo_lds + ((size_t)wave * 4 * kWave + lane) * PX;

    static_for<0, RW>([&](auto tt) {
        constexpr int t = decltype(tt)::value;
        if constexpr (SHIFTED) realign_row(raw[t], shift[t]);
        gray_row<In, PX>(raw[t], p.wr, p.wg, p.wb, gc);
        if constexpr (t < 4) {
#pragma unroll
            for (int i = 0; i < PX; ++i) my_halo[(size_t)t * kWave * PX + i] = gc[i];
        }
        if constexpr (HANDOFF && t == 3) {
            // Publish.  The lanes' writes of the four rows are ordered before lane 0's release
            // store by a release fence, a barrier and an acquire fence at wavefront scope; the
            // release store at workgroup scope then carries them to whoever acquires the flag.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (lane == 0) __hip_atomic_store(&ready[wave], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if constexpr (t < 4) {
            row_step<(t < 2 ? 0 : 1), t % 3, PX, BINOM>(lb, gc, p.k, none);
        } else {
            row_step<2, t % 3, PX, BINOM>(lb, gc, p.k, results[t - 4]);
            pin_values<PX>(results[t - 4]);
        }
        // Each row is worked through as soon as it has arrived: without this the compiler
        // gathers the arithmetic of all rows behind the wait for the last one.
        __builtin_amdgcn_sched_barrier(0);
    });

    if constexpr (!HANDOFF) __syncthreads();

    if (wave + 1 < n_waves) {
        if constexpr (HANDOFF) {
            // Acquire load of the neighbour's flag: pairs with its release store, so the rows read
            // below are the published ones.  The wait ends: all wavefronts of a workgroup are
            // resident on the CU together (a workgroup is dispatched as a whole), and wavefront
            // wave + 1 reaches its release store without waiting for anybody (every wavefront
            // runs through the code above unconditionally; its loads always return).
            while (__hip_atomic_load(&ready[wave + 1], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0u)
                __builtin_amdgcn_s_sleep(4);
        }
        const float* below = halo_lds + ((size_t)(wave + 1) * 4 * kWave + lane) * PX;
        static_for<RW, RW + 4>([&](auto tt) {
            constexpr int t = decltype(tt)::value;
#pragma unroll
            for (int i = 0; i < PX; ++i) gc[i] = below[(size_t)(t - RW) * kWave * PX + i];
            row_step<2, t % 3, PX, BINOM>(lb, gc, p.k, results[t - 4]);
            pin_values<PX>(results[t - 4]);
        });
    }

    // The last wavefront skips the four rows it has no data for.
    if constexpr (HANDOFF) __syncthreads();                     // stores only after all of the workgroup's loads
    __builtin_amdgcn_sched_barrier(0);
    constexpr int SAUX = LAUX == kAuxKeepShared ? kAuxManyStore : kAuxStore;
    if (__builtin_expect(p.out_kind == HARRIS_OUT_F32, 1)) {
        static_for<0, RW>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            if (j < RW - 4 || wave + 1 < n_waves) store_row<PX, SAUX>(results[j], out_rs[j], lane_bytes + out_lead[j]);
        });
    } else if (p.out_kind == HARRIS_OUT_F16) {
        static_for<0, RW>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            if (j < RW - 4 || wave + 1 < n_waves) store_row_16<PX, false, SAUX>(results[j], out_rs[j], lane_bytes + out_lead[j]);
        });
    } else if (p.out_kind == HARRIS_OUT_BF16) {
        static_for<0, RW>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            if (j < RW - 4 || wave + 1 < n_waves) store_row_16<PX, true, SAUX>(results[j], out_rs[j], lane_bytes + out_lead[j]);
        });
    } else {
        static_for<0, RW>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            if (j < RW - 4 || wave + 1 < n_waves) store_row_8<PX, SAUX>(results[j], p.q_scale, p.q_offset, out_rs[j], lane_bytes + out_lead[j]);
        });
    }
}

}  // namespace

#endif  // HARRIS_KERNELS_H
