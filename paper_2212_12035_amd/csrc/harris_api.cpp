// C interface of libharris: argument checks, launch-shape planning, dispatch.
// Everything here runs on the host and touches no device memory.

#include <math.h>
#include <stdint.h>

#include "harris_tuning.h"
#include "harris_launch.h"

namespace {

constexpr int kVersion = 400;   // 0.4.0

bool power_of_two_aligned(uintptr_t p, unsigned bytes) { return (p & (uintptr_t)(bytes - 1)) == 0; }

int elem_size(int dtype) { return dtype == HARRIS_U8 ? 1 : 4; }
int out_elem_size(int out_dtype) { return out_dtype == HARRIS_OUT_F32 ? 4 : out_dtype == HARRIS_OUT_U8 ? 1 : 2; }
bool known_out_dtype(int d) { return d == HARRIS_OUT_F32 || d == HARRIS_OUT_F16 || d == HARRIS_OUT_BF16 || d == HARRIS_OUT_U8; }

// Can every lane load px input elements and store its result columns with single, naturally
// aligned vector accesses?  Loads are px*elem bytes wide up to 16; stores are min(px,4) result elements.
bool px_fits(int px, int dtype, int out_dtype, int W, int rgb_align, int out_align) {
    if (px < 1 || W % px != 0) return false;
    int load_bytes = px * elem_size(dtype);
    if (load_bytes > 16) load_bytes = 16;
    int store_bytes = (px < 4 ? px : 4) * out_elem_size(out_dtype);
    return rgb_align % load_bytes == 0 && out_align % store_bytes == 0;
}

// Four pixels per lane without natural alignment (a width that is no multiple of 4, padded
// rows, an offset view); tile kernel only.  float32 rows start on 4-byte boundaries: buffer
// accesses of several 32-bit words need only 4-byte alignment, and the hardware checks each
// word of such an access against the end of the row by itself, so the lane that straddles the
// end of a row loads zeros beyond it and stores nothing there.  8-bit rows may start on any
// byte: the kernel loads the aligned words that hold them and shifts.  Results: float32, or
// 16-bit with rows that start on 4-byte boundaries and have an even number of columns: the
// range check works on whole 32-bit words, so a word that held the last column of an odd row
// together with two bytes behind it would either be dropped or written whole.  (8-bit codes
// are stored as one word per lane and keep the narrower lanes.)
bool px4_fits_word_aligned(int dtype, int out_dtype, int W, int rgb_align, int out_align) {
    if (dtype == HARRIS_F32 && rgb_align % 4 != 0) return false;
    if (out_dtype == HARRIS_OUT_U8 || out_align % 4 != 0) return false;
    return out_dtype == HARRIS_OUT_F32 || W % 2 == 0;
}

int plan(int dtype, int out_dtype, int batch, int H, int W, int rgb_align, int out_align, const harris_tuning* tuning,
         harris_tuning* chosen, long long* n_blocks, harris_launch::Params* params) {
    if (dtype != HARRIS_F32 && dtype != HARRIS_U8) return HARRIS_ERR_ARG;
    if (!known_out_dtype(out_dtype)) return HARRIS_ERR_ARG;
    if (batch < 0 || H < 4 || W < 4) return HARRIS_ERR_SHAPE;
    if (W > (1 << 28)) return HARRIS_ERR_SHAPE;      // byte offsets within a row are 32-bit
    if (H > (1 << 30)) return HARRIS_ERR_SHAPE;      // row indices plus a tile's height stay within int
    // Byte counts below are 64-bit: 16 bytes per pixel of at most 2^58 pixels would not fit.
    if (batch > 0 && (long long)H * W > (1LL << 56) / batch) return HARRIS_ERR_SHAPE;
    if (rgb_align < 1 || out_align < out_elem_size(out_dtype)) return HARRIS_ERR_ARG;
    harris_tuning t = {0, 0, 0, 0, 0, 0u, 0};
    if (tuning) t = *tuning;
    if (t.flags & ~(HARRIS_TUNE_NO_ALTERNATE | HARRIS_TUNE_NO_XCD_REMAP | HARRIS_TUNE_CACHED_LOADS | HARRIS_TUNE_STREAM_LOADS |
                    HARRIS_TUNE_ALIGNED_STORES | HARRIS_TUNE_PLAIN_STORES | HARRIS_TUNE_KEEP_SHARED_ROWS | HARRIS_TUNE_FLAG_HANDOFF)) return HARRIS_ERR_ARG;
    if ((t.flags & HARRIS_TUNE_CACHED_LOADS) && (t.flags & HARRIS_TUNE_STREAM_LOADS)) return HARRIS_ERR_ARG;
    if ((t.flags & HARRIS_TUNE_KEEP_SHARED_ROWS) && !(t.flags & HARRIS_TUNE_STREAM_LOADS)) return HARRIS_ERR_ARG;
    if ((t.flags & HARRIS_TUNE_FLAG_HANDOFF) && (t.flags & (HARRIS_TUNE_CACHED_LOADS | HARRIS_TUNE_KEEP_SHARED_ROWS))) return HARRIS_ERR_ARG;
    if ((t.flags & HARRIS_TUNE_ALIGNED_STORES) && (t.flags & HARRIS_TUNE_PLAIN_STORES)) return HARRIS_ERR_ARG;
    if (t.schedule != 0 && t.schedule != HARRIS_SCHEDULE_BANDS && t.schedule != HARRIS_SCHEDULE_TILES) return HARRIS_ERR_ARG;

    const int n = H - 4, m = W - 4;
    const bool tiles_allowed = (t.schedule == 0 || t.schedule == HARRIS_SCHEDULE_TILES) && t.prefetch == 0;
    const bool word_aligned_px4 = tiles_allowed && px4_fits_word_aligned(dtype, out_dtype, W, rgb_align, out_align);
    if (t.px == 0) {
        t.px = 1;
        if (px_fits(4, dtype, out_dtype, W, rgb_align, out_align) || word_aligned_px4) t.px = 4;
        else if (px_fits(2, dtype, out_dtype, W, rgb_align, out_align)) t.px = 2;
    } else if (!((t.px == 1 || t.px == 2 || t.px == 4) &&
                 (px_fits(t.px, dtype, out_dtype, W, rgb_align, out_align) || (t.px == 4 && word_aligned_px4)))) {
        return HARRIS_ERR_ARG;
    }
    if (t.rows < 0 || t.prefetch < 0 || t.waves_per_block < 0 || t.lds_kb < 0 || t.lds_kb > 64) return HARRIS_ERR_ARG;
    // A prefetch depth exists only in the band schedule.
    if (t.schedule == 0) t.schedule = t.prefetch == 0 ? HARRIS_SCHEDULE_TILES : HARRIS_SCHEDULE_BANDS;
    if (out_dtype != HARRIS_OUT_F32 && t.schedule != HARRIS_SCHEDULE_TILES) return HARRIS_ERR_ARG;   // 16- and 8-bit results: tile kernel only
    // Strip borders on 64-byte boundaries of the result rows: the tile kernel with 16-byte lanes.
    // (A lane's stores must then be naturally aligned: borders can only lie between lanes.)
    const bool tile4 = t.schedule == HARRIS_SCHEDULE_TILES && t.px == 4;
    const bool can_align = tile4 && px_fits(4, dtype, out_dtype, W, rgb_align, out_align);
    if ((t.flags & HARRIS_TUNE_ALIGNED_STORES) && !can_align) return HARRIS_ERR_ARG;
    if ((t.flags & (HARRIS_TUNE_KEEP_SHARED_ROWS | HARRIS_TUNE_FLAG_HANDOFF)) && !tile4) return HARRIS_ERR_ARG;
    // Measured, moved against fixed borders: 378 against 393 us on 64x1080x1920 float32, 12.5
    // against 12.8 us on 1536x2560, 37.0 against 37.3 us on 2832x4256, 89 against 93 us on
    // 8192x8192 uint8.
    // 16-bit results pay more for moved borders (strips of 224 instead of 252 columns; 192 for
    // 8-bit results, which never get them by default): worth it only for large float32 inputs (64x1080x1920: 341 against 359 us; 1536x2560: 12.8 against
    // 12.4 us; 8192x8192 uint8: 81 against 74 us).
    if (!(t.flags & (HARRIS_TUNE_ALIGNED_STORES | HARRIS_TUNE_PLAIN_STORES))) {
        const long long bytes = (long long)batch * (3LL * H * W * elem_size(dtype) + (long long)out_elem_size(out_dtype) * n * m);
        const bool align = can_align && (out_dtype == HARRIS_OUT_F32 || (out_dtype != HARRIS_OUT_U8 && dtype == HARRIS_F32 && bytes > (128LL << 20)));
        t.flags |= align ? HARRIS_TUNE_ALIGNED_STORES : HARRIS_TUNE_PLAIN_STORES;
    }
    // As few strips as 64-lane wavefronts allow, all of the same width.  A moved border lies up
    // to one 64-byte block less a lane (12 float32 or 28 16-bit columns) right of the strip's
    // nominal end, and the wavefront must reach that far.
    const long long border_reach = (t.flags & HARRIS_TUNE_ALIGNED_STORES) ? 64 / out_elem_size(out_dtype) - 4 : 0;
    // 8-bit rows loaded as aligned words and shifted: the last lane only supplies bytes to its left neighbour.
    const bool in_shifted = dtype == HARRIS_U8 && tile4 && !can_align;
    const long long max_pitch = (long long)harris_launch::valid_lanes(t.px) * t.px - border_reach - (in_shifted ? 4 : 0);
    const long long n_strips = m > 0 ? (m + max_pitch - 1) / max_pitch : 0;
    const long long pitch = n_strips > 0 ? ((m + n_strips - 1) / n_strips + t.px - 1) / t.px * t.px : max_pitch;

    // Bytes the launch moves.
    const long long elem = elem_size(dtype);
    const long long footprint = (long long)batch * (3LL * H * W * elem + (long long)out_elem_size(out_dtype) * n * m);

    // Default tile shape.  A problem that one pass over the 256 CUs can hold is fastest as one
    // tile per CU: all CUs then carry the same load and finish together (measured on
    // 1536x2560: 12.2 us against 13.5 us for small tiles and 14.6 us for the best band shape).
    // The tile must cover `need` input rows; it is NW wavefronts x RW rows with the smallest
    // NW * RW, RW taken from a list in order of measured preference, some with a handicap.
    // Short tiles are better off with few rows per wavefront (a wavefront's RW + 4 row steps are
    // a serial chain, which shows once the data is there quickly: 768x1024 5.0 us with 5 x 4
    // against 5.7 us with 10 x 2; 1024x1024 5.8 us with 6 x 4 against 6.3 us with 8 x 3), tall
    // ones with 8, 6 or 9 (1440x2560 11.8 us with 8 x 9 against 12.2 us with 10 x 7 and 12.0 us
    // with 5 x 14; but 2160x3840 22.6 us with 10 x 14 against 24.1 us with 9 x 16).
    // Larger problems take many small tiles, which keep the memory system busiest (measured
    // on 2832x4256, 64x1080x1920 and 8192x8192 uint8).
    int tile_rw = 4, tile_nw = 4, tile_lds_kb = 0;
    bool one_per_cu = false;
    if (footprint <= (128LL << 20) && t.px == 4 && batch > 0 && n_strips > 0 && (long long)batch * n_strips <= 256) {
        const long long max_bands = 256 / ((long long)batch * n_strips);
        const long long need = (n + max_bands - 1) / max_bands + 4;         // input rows per tile
        // {rows per wavefront, rows of handicap}, in order of preference among equals.
        static const int kShort[][2] = {{5, 0}, {4, 0}, {6, 0}, {0, 0}};
        static const int kMedium[][2] = {{6, 0}, {5, 0}, {8, 0}, {0, 0}};
        static const int kTall[][2] = {{8, 0}, {6, 0}, {9, 0}, {10, 3}, {5, 3}, {0, 0}};
        // 8-bit input has more arithmetic per byte and does better with fewer rows per wavefront
        // (1536x2560: 7.8 us with 12 x 6 against 8.8 us with 9 x 8; 2160x3840: 13.2 us with 16 x 9
        // against 14.1 us with 14 x 10).
        static const int kTall8[][2] = {{6, 0}, {5, 3}, {8, 2}, {9, 2}, {10, 6}, {0, 0}};
        static const int kShifted[][2] = {{4, 0}, {8, 0}, {0, 0}};      // the kernels that exist for shifted 8-bit rows
        const int (*list)[2] = in_shifted ? kShifted : need <= 20 ? kShort : need <= 48 ? kMedium : dtype == HARRIS_U8 ? kTall8 : kTall;
        // Tiles of 26 to 32 rows (40 for 8-bit input), and several images with tiles of up to
        // 48 rows, are faster as many small tiles (960x1280: 6.2 against 6.5 us, 8-bit 5.1 / 5.6;
        // 1080x1920 8-bit: 5.5 / 5.9, but float32 8.4 / 8.2) -- for float32 input as long as there
        // are at most two of them per CU: a third one on some CUs costs more than it saves
        // (900x1600, 525 small tiles: 7.5 us against 6.9 with one tile of 5 x 6 rows per CU;
        // 1050x1400: 7.7 / 6.9; two images of 720x1280: 7.9 / 7.6).
        const long long small_count = (long long)batch * n_strips * ((n + 11) / 12);     // tiles of 4 x 4 rows
        const bool small_tiles = ((batch > 1 && need <= 48) || (need >= 26 && need <= (dtype == HARRIS_U8 ? 40 : 32))) &&
                                 (dtype == HARRIS_U8 || small_count <= 512);
        long long best = -1;
        for (; (*list)[0] && !small_tiles; ++list) {
            const int rw = (*list)[0];
            long long nw = (need + rw - 1) / rw;
            if (nw < 2) nw = 2;
            if (nw > 16) continue;
            const long long cost = nw * rw + (*list)[1];
            if (best < 0 || cost < best) { best = cost; tile_rw = rw; tile_nw = (int)nw; one_per_cu = true; }
        }
    }
    if (!one_per_cu && tile4 && dtype == HARRIS_F32) {
        // Many tiles of float32 input.  Such launches are fastest with 10 to 16 wavefronts in
        // flight per CU, not with the 28 to 32 the registers allow (every wavefront requests all
        // its rows at once; with fewer in flight the requests stay within what L2 and the memory
        // controllers handle well), so the planner reserves LDS to hold the resident tiles down:
        // 36 KB -> 4 tiles per CU, 48 KB -> 3, 64 KB -> 2.  Measured (shape x reservation swept
        // together; 4 x 4 rows without reservation in brackets):
        //   float32 results, up to 400 MB: 4 wavefronts x 5 rows, 3 per CU (2832x4256 32.7 [34.8]
        //     us, 2x2160x3840 44.5 [49.1], 8192x8192 at 1 GB 174.6 [191.6]);
        //   beyond, 8 images or more: 5 x 5, 2 per CU (16x1080x1920 87.1 [103.7] us, 64x1080x1920
        //     351 [378], 128x720x1280 318 [350]); fewer, larger images: 5 x 6, 2 per CU
        //     (4320x7680 92.2 [105.7] us, 8192x8192 176.6);
        //   16-bit results and 8-bit codes above 128 MB: 4 x 6, 3 per CU (2832x4256 to binary16
        //     29.1 [31.2] us, 16x1080x1920 75.7 [89.7], 64x1080x1920 331 [355], 4320x7680 80.8
        //     [94.2]); one image beyond 800 MB: 5 x 6, 2 per CU (8192x8192 161 [184] us, 175
        //     with 4 x 6);
        //   up to 128 MB (several images, too many tiles for one per CU): 4 x 4, 4 per CU
        //     (32x512x512 24.9 [25.6] us).
        // 8-bit input is the opposite: every reservation costs time (8192x8192 uint8: 93 us with
        // none, 102 us with 4 tiles per CU), so it keeps 4 x 4 and all the wavefronts that fit.
        if (footprint <= (128LL << 20)) { tile_rw = 4; tile_nw = 4; tile_lds_kb = 36; }
        else if (out_dtype != HARRIS_OUT_F32 && batch == 1 && footprint > (800LL << 20)) { tile_rw = 6; tile_nw = 5; tile_lds_kb = 64; }
        else if (out_dtype != HARRIS_OUT_F32) { tile_rw = 6; tile_nw = 4; tile_lds_kb = 48; }
        else if (footprint <= (400LL << 20)) { tile_rw = 5; tile_nw = 4; tile_lds_kb = 48; }
        else if (batch >= 8) { tile_rw = 5; tile_nw = 5; tile_lds_kb = 64; }
        else { tile_rw = 6; tile_nw = 5; tile_lds_kb = 64; }
    }

    long long tile_rows;       // result rows per band or tile
    if (t.schedule == HARRIS_SCHEDULE_TILES) {
        if (t.rows == 0 && t.waves_per_block == 0) { t.rows = tile_rw; t.waves_per_block = tile_nw; if (t.lds_kb == 0) t.lds_kb = tile_lds_kb; }
        if (t.rows == 0) t.rows = 4;
        if (t.waves_per_block == 0) t.waves_per_block = 4;
        const bool rows_ok = t.rows == 4 || (t.px == 4 && (t.rows == 5 || t.rows == 6 || t.rows == 8 || t.rows == 9 || t.rows == 10));
        if (!rows_ok || t.waves_per_block < 2 || t.waves_per_block > 16) return HARRIS_ERR_ARG;
        if (in_shifted && !(t.rows == 4 || t.rows == 8)) return HARRIS_ERR_ARG;
        if (dtype == HARRIS_U8 && (t.flags & HARRIS_TUNE_FLAG_HANDOFF)) return HARRIS_ERR_ARG;   // ready flags: float32 input only
        if (t.prefetch != 0) return HARRIS_ERR_ARG;
        tile_rows = (long long)t.rows * t.waves_per_block - 4;
        // The reservation in force: at least the four gray rows each wavefront publishes.
        const int need_kb = (int)(((long long)t.waves_per_block * 4 * 64 * t.px * 4 + 1023) / 1024);
        if (t.lds_kb < need_kb) t.lds_kb = need_kb;
    } else {
        if (t.lds_kb != 0) return HARRIS_ERR_ARG;                       // the band schedule uses no LDS
        const bool large = footprint > (256LL << 20);
        if (t.prefetch == 0) t.prefetch = 3;
        if (t.prefetch != 3) return HARRIS_ERR_ARG;                     // the one depth the band kernels are built for
        if (t.waves_per_block == 0) t.waves_per_block = large ? 4 : 1;
        if (!(t.waves_per_block == 1 || t.waves_per_block == 2 || t.waves_per_block == 4)) return HARRIS_ERR_ARG;
        if (t.rows == 0) {
            if (large) {
                t.rows = 32;       // thousands of bands in any case: measured best trade of halo rows against run length
            } else {
                // Everything is resident at once.  Take the shortest band of 16..64 rows that
                // needs no more wavefronts than the chip has SIMDs (1024): every wavefront then
                // has a SIMD to itself, the 256 CUs hold at most 4 each, and all of them start
                // and end together.  (Measured on 1536x2560 and 2832x4256: launches whose
                // wavefront count lies just below a multiple of 256 are the fast ones.)
                const long long per_band = (long long)batch * n_strips;
                long long best_r = 64;
                for (long long r = 16; r <= 64; ++r)
                    if (((n + r - 1) / r) * per_band <= 1024) { best_r = r; break; }
                t.rows = (int)best_r;
            }
        }
        tile_rows = t.rows;
    }
    const long long n_bands = n > 0 ? ((long long)n + tile_rows - 1) / tile_rows : 0;
    const long long tiles_per_image = n_bands * n_strips;
    const long long n_tiles = tiles_per_image * batch;

    // Load policy, measured.  One tile per CU (at most 256 tiles): everything non-temporal (1536x2560:
    // 12.2 us against 12.6 us with the shared rows kept).  Many tiles: non-temporal except the rows
    // two tiles share, which the default policy keeps in L2 for the second reader (2832x4256: 34.6 us
    // against 37.1 us all-default and 39.7 us all-non-temporal; 4096x4096: 49.7 / 53.8 / 54.6 us;
    // 32x512x512: 25.7 / 27.0 / 26.8 us; 8192x8192 uint8: 91.1 / 105 / 91.8 us; 16x1080x1920 with
    // tiles of 5 x 6: 98.2 / 101.8 us all-default; 64x1080x1920 with 5 x 8: 374.4 / 378.4 us).
    // Bands and lanes narrower than 16 bytes have no mixed policy: default-policy loads from 128 MB on.
    const bool one_tile_per_cu = t.schedule == HARRIS_SCHEDULE_TILES && n_tiles <= 256;
    if (!(t.flags & (HARRIS_TUNE_CACHED_LOADS | HARRIS_TUNE_STREAM_LOADS))) {
        if (t.flags & HARRIS_TUNE_FLAG_HANDOFF) t.flags |= HARRIS_TUNE_STREAM_LOADS;
        else if (tile4 && !one_tile_per_cu) t.flags |= HARRIS_TUNE_STREAM_LOADS | HARRIS_TUNE_KEEP_SHARED_ROWS;
        else if (dtype == HARRIS_F32 && footprint > (128LL << 20)) t.flags |= HARRIS_TUNE_CACHED_LOADS;
        else t.flags |= HARRIS_TUNE_STREAM_LOADS;
        // Ready flags instead of the barrier where tiles are few and tall and the input float32
        // (measured: 1536x2560 12.1 against 12.3 us, 2048x2048 12.7 / 13.2, 2x1536x2560 22.6 / 23.3,
        // 1080x1920 8.4 / 8.4; 720x1280, 3 wavefronts per tile, 6.4 / 6.1; 2048x4096 uint8 18.1 / 15.2).
        if (one_tile_per_cu && tile4 && dtype == HARRIS_F32 && t.waves_per_block >= 5 &&
            t.flags == (t.flags & ~(HARRIS_TUNE_CACHED_LOADS | HARRIS_TUNE_KEEP_SHARED_ROWS)))
            t.flags |= HARRIS_TUNE_FLAG_HANDOFF;
    }
    // TILES: one workgroup per tile.  BANDS: one wavefront per band of a strip; a workgroup
    // of 2 or 4 wavefronts takes 2 bands x 1 or 2 strips.
    const long long group_h = t.waves_per_block >= 2 ? 2 : 1, group_w = t.waves_per_block / group_h;
    const long long blocks_x = (n_strips + group_w - 1) / group_w;
    const long long blocks_per_image = blocks_x * ((n_bands + group_h - 1) / group_h);
    const long long blocks = t.schedule == HARRIS_SCHEDULE_TILES ? n_tiles : blocks_per_image * batch;
    if (tiles_per_image > 0x7fffffffLL || n_tiles > 0x7fffffffLL || blocks > 0x7fffffffLL) return HARRIS_ERR_SHAPE;

    if (chosen) *chosen = t;
    if (n_blocks) *n_blocks = blocks;
    if (params) {
        params->H = H; params->W = W; params->n = n; params->m = m;
        params->rows_per_band = (int)tile_rows;
        params->n_strips = (unsigned)n_strips;
        params->strip_pitch = (unsigned)pitch;
        params->n_bands = (unsigned)n_bands;
        params->tiles_per_image = (unsigned)tiles_per_image;
        params->by_tiles_per_image = harris_launch::make_fastdiv(tiles_per_image > 0 ? (unsigned)tiles_per_image : 1u);
        params->by_n_strips = harris_launch::make_fastdiv(n_strips > 0 ? (unsigned)n_strips : 1u);
        params->blocks_x = (unsigned)blocks_x;
        params->blocks_per_image = (unsigned)blocks_per_image;
        params->n_blocks = (unsigned)blocks;
        params->waves_per_block = (unsigned)t.waves_per_block;
        params->flags = t.flags;
        params->out_kind = (unsigned)out_dtype;
        params->in_shifted = in_shifted ? 1 : 0;
        params->lds_bytes = (unsigned)t.lds_kb * 1024u;
    }
    return HARRIS_OK;
}

unsigned pointer_alignment(const void* p) {
    uintptr_t v = (uintptr_t)p;
    unsigned a = 1;
    while (a < 256 && power_of_two_aligned(v, a * 2)) a *= 2;
    return a;
}

}  // namespace

extern "C" {

int harris_plan(int dtype, int batch, int H, int W, int rgb_align, int out_align,
                const harris_tuning* tuning, harris_tuning* chosen, long long* n_blocks) {
    return plan(dtype, HARRIS_OUT_F32, batch, H, W, rgb_align, out_align, tuning, chosen, n_blocks, nullptr);
}

int harris_plan_typed(int dtype, int out_dtype, int batch, int H, int W, int rgb_align, int out_align,
                      const harris_tuning* tuning, harris_tuning* chosen, long long* n_blocks) {
    return plan(dtype, out_dtype, batch, H, W, rgb_align, out_align, tuning, chosen, n_blocks, nullptr);
}

}  // extern "C"

namespace {

// Every entry point of the fused kernel ends here.
int run(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
        float k, float sobel_scale, int window, void* out, int out_dtype, float q_scale, float q_offset,
        const harris_tuning* tuning, void* stream) {
    if (dtype != HARRIS_F32 && dtype != HARRIS_U8) return HARRIS_ERR_ARG;
    if (!known_out_dtype(out_dtype)) return HARRIS_ERR_ARG;
    if (!isfinite(q_scale) || !isfinite(q_offset)) return HARRIS_ERR_ARG;
    if (batch < 0 || H < 4 || W < 4) return HARRIS_ERR_SHAPE;
    if (!isfinite(k) || !isfinite(sobel_scale)) return HARRIS_ERR_ARG;
    if (window != HARRIS_WINDOW_BOX && window != HARRIS_WINDOW_BINOMIAL) return HARRIS_ERR_ARG;
    const long long n = H - 4, m = W - 4;
    harris_layout lay;
    if (layout) {
        lay = *layout;
    } else {
        lay.rgb_row_pitch = W; lay.rgb_plane_pitch = (long long)H * W; lay.rgb_image_pitch = 3LL * H * W;
        lay.out_row_pitch = m; lay.out_image_pitch = n * m;
    }
    const long long in_rows_span = (long long)(H - 1) * lay.rgb_row_pitch + W;
    if (lay.rgb_row_pitch < W || lay.rgb_plane_pitch < in_rows_span || lay.rgb_image_pitch < 2 * lay.rgb_plane_pitch + in_rows_span)
        return HARRIS_ERR_SHAPE;
    if (lay.out_row_pitch < m || (n > 0 && lay.out_image_pitch < (n - 1) * lay.out_row_pitch + m)) return HARRIS_ERR_SHAPE;
    const bool empty = batch == 0 || H == 4 || W == 4;
    if (!empty && (rgb == nullptr || out == nullptr)) return HARRIS_ERR_NULL;
    if (!empty && (int)pointer_alignment(out) < out_elem_size(out_dtype)) return HARRIS_ERR_ARG;
    if (!empty && dtype == HARRIS_F32 && pointer_alignment(rgb) < 4) return HARRIS_ERR_ARG;

    // Alignment that every row start shares: the base pointer's and each pitch's (in bytes).
    auto common_alignment = [](unsigned a, long long pitch_bytes) {
        while (a > 1 && pitch_bytes % a != 0) a /= 2;
        return a;
    };
    unsigned rgb_align = 16, out_align = 16;
    if (!empty) {
        const long long e = elem_size(dtype);
        rgb_align = pointer_alignment(rgb);
        if (rgb_align > 16) rgb_align = 16;
        rgb_align = common_alignment(rgb_align, lay.rgb_row_pitch * e);
        rgb_align = common_alignment(rgb_align, lay.rgb_plane_pitch * e);
        rgb_align = common_alignment(rgb_align, lay.rgb_image_pitch * e);
        out_align = pointer_alignment(out);
        if (out_align > 16) out_align = 16;
        out_align = common_alignment(out_align, lay.out_row_pitch * out_elem_size(out_dtype));
        out_align = common_alignment(out_align, lay.out_image_pitch * out_elem_size(out_dtype));
    }

    harris_launch::Params p;
    harris_tuning shape;
    long long n_blocks = 0;
    int rc = plan(dtype, out_dtype, batch, H, W, (int)rgb_align, (int)out_align, tuning, &shape, &n_blocks, &p);
    if (rc != HARRIS_OK) return rc;
    if (empty) return HARRIS_OK;

    p.rgb = rgb;
    p.out = out;
    p.in_row_pitch = lay.rgb_row_pitch; p.in_plane_pitch = lay.rgb_plane_pitch; p.in_image_pitch = lay.rgb_image_pitch;
    p.out_row_pitch = lay.out_row_pitch; p.out_image_pitch = lay.out_image_pitch;
    // The Sobel scale multiplies Ix and Iy, which are linear in gray: fold it (and the
    // 1/255 of 8-bit input) into the three gray weights.
    const float in_scale = dtype == HARRIS_U8 ? sobel_scale / 255.0f : sobel_scale;
    p.wr = 0.299f * in_scale;
    p.wg = 0.587f * in_scale;
    p.wb = 0.114f * in_scale;
    p.k = k;
    p.binomial = window == HARRIS_WINDOW_BINOMIAL ? 1 : 0;
    p.q_scale = q_scale;
    p.q_offset = q_offset;
    return harris_launch::launch(p, shape, n_blocks, dtype, stream);
}

}  // namespace

extern "C" {

int harris_coarsity_typed(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
                          float k, float sobel_scale, int window, void* out, int out_dtype,
                          const harris_tuning* tuning, void* stream) {
    if (out_dtype == HARRIS_OUT_U8) return HARRIS_ERR_ARG;          // needs a scale: harris_coarsity_quantized
    return run(rgb, dtype, batch, H, W, layout, k, sobel_scale, window, out, out_dtype, 1.0f, 0.0f, tuning, stream);
}

int harris_coarsity_quantized(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
                              float k, float sobel_scale, int window, float q_scale, float q_offset,
                              uint8_t* out, const harris_tuning* tuning, void* stream) {
    return run(rgb, dtype, batch, H, W, layout, k, sobel_scale, window, out, HARRIS_OUT_U8, q_scale, q_offset, tuning, stream);
}

int harris_coarsity_pitched(const void* rgb, int dtype, int batch, int H, int W, const harris_layout* layout,
                            float k, float sobel_scale, int window, float* out,
                            const harris_tuning* tuning, void* stream) {
    return harris_coarsity_typed(rgb, dtype, batch, H, W, layout, k, sobel_scale, window, out, HARRIS_OUT_F32, tuning, stream);
}

int harris_coarsity_ex(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale,
                       int window, float* out, const harris_tuning* tuning, void* stream) {
    return harris_coarsity_pitched(rgb, dtype, batch, H, W, nullptr, k, sobel_scale, window, out, tuning, stream);
}

int harris_coarsity(const float* rgb, int batch, int H, int W, float k, float* out, void* stream) {
    return harris_coarsity_ex(rgb, HARRIS_F32, batch, H, W, k, 1.0f, HARRIS_WINDOW_BOX, out, nullptr, stream);
}

int harris_coarsity_u8(const uint8_t* rgb, int batch, int H, int W, float k, float* out, void* stream) {
    return harris_coarsity_ex(rgb, HARRIS_U8, batch, H, W, k, 1.0f, HARRIS_WINDOW_BOX, out, nullptr, stream);
}

long long harris_grouped_workspace_bytes(int grouping, int batch, int H, int W) {
    if (grouping < 1 || grouping > 4 || batch < 0 || H < 4 || W < 4) return -1;
    return (long long)(harris_launch::grouped_workspace_floats(grouping, batch, H, W) * sizeof(float));
}

int harris_coarsity_grouped(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale,
                            int window, int grouping, void* workspace, long long workspace_bytes,
                            float* out, void* stream) {
    if (grouping < 1 || grouping > 4) return HARRIS_ERR_ARG;
    if (grouping == 4) return harris_coarsity_ex(rgb, dtype, batch, H, W, k, sobel_scale, window, out, nullptr, stream);
    if (dtype != HARRIS_F32 && dtype != HARRIS_U8) return HARRIS_ERR_ARG;
    if (batch < 0 || H < 4 || W < 4) return HARRIS_ERR_SHAPE;
    if (!isfinite(k) || !isfinite(sobel_scale)) return HARRIS_ERR_ARG;
    if (window != HARRIS_WINDOW_BOX && window != HARRIS_WINDOW_BINOMIAL) return HARRIS_ERR_ARG;
    if (batch == 0 || H == 4 || W == 4) return HARRIS_OK;
    if (rgb == nullptr || out == nullptr || workspace == nullptr) return HARRIS_ERR_NULL;
    if (pointer_alignment(out) < 4 || pointer_alignment(workspace) < 4) return HARRIS_ERR_ARG;
    if (dtype == HARRIS_F32 && pointer_alignment(rgb) < 4) return HARRIS_ERR_ARG;
    if (workspace_bytes < harris_grouped_workspace_bytes(grouping, batch, H, W)) return HARRIS_ERR_ARG;
    return harris_launch::launch_grouped(rgb, dtype, batch, H, W, k, sobel_scale, window == HARRIS_WINDOW_BINOMIAL,
                                         grouping, static_cast<float*>(workspace), out, stream);
}

int harris_coarsity_grouped_static(const void* rgb, int dtype, int batch, int H, int W, float k, float sobel_scale,
                                   int window, int grouping, float* out, void* stream) {
    if (grouping < 1 || grouping > 4) return HARRIS_ERR_ARG;
    if (grouping == 4) return harris_coarsity_ex(rgb, dtype, batch, H, W, k, sobel_scale, window, out, nullptr, stream);
    if (batch < 0 || H < 4 || W < 4) return HARRIS_ERR_SHAPE;
    if (batch == 0 || H == 4 || W == 4)      // empty result: the remaining argument checks, no work, no scratch
        return harris_coarsity_grouped(rgb, dtype, batch, H, W, k, sobel_scale, window, grouping, nullptr, 0, out, stream);
    // The gray image alone is 4 bytes per pixel; checked in doubles first, since the exact count
    // below is 64-bit arithmetic and absurd shapes would not fit it.
    if (4.0 * (double)batch * (double)H * (double)W > (double)HARRIS_GROUPED_SCRATCH_BYTES) return HARRIS_ERR_SCRATCH;
    const long long need = harris_grouped_workspace_bytes(grouping, batch, H, W);
    if (need < 0 || need > (long long)HARRIS_GROUPED_SCRATCH_BYTES) return HARRIS_ERR_SCRATCH;
    if (rgb == nullptr || out == nullptr) return HARRIS_ERR_NULL;
    float* ws = harris_launch::scratch_of_current_device();
    if (ws == nullptr) return HARRIS_ERR_LAUNCH;
    return harris_coarsity_grouped(rgb, dtype, batch, H, W, k, sobel_scale, window, grouping, ws, need, out, stream);
}

int harris_probe_copy(const void* rgb, int dtype, int batch, int H, int W, float* out, void* stream) {
    if (dtype != HARRIS_F32 && dtype != HARRIS_U8) return HARRIS_ERR_ARG;
    if (batch < 0 || H < 4 || W < 4) return HARRIS_ERR_SHAPE;
    if (batch == 0 || H == 4 || W == 4) return HARRIS_OK;
    if (rgb == nullptr || out == nullptr) return HARRIS_ERR_NULL;
    const long long e = elem_size(dtype);
    if (pointer_alignment(rgb) < 16 || pointer_alignment(out) < 16) return HARRIS_ERR_ARG;
    if (((long long)H * W * e) % 16 != 0 || ((long long)(H - 4) * (W - 4) * 4) % 16 != 0) return HARRIS_ERR_ARG;
    return harris_launch::launch_copy_probe(rgb, dtype, batch, H, W, out, stream);
}

int harris_probe_stream(int kind, const void* src, void* dst, long long bytes, void* stream) {
    if (kind != HARRIS_PROBE_READ && kind != HARRIS_PROBE_WRITE && kind != HARRIS_PROBE_NONE) return HARRIS_ERR_ARG;
    if (bytes < 0) return HARRIS_ERR_SHAPE;
    if (kind == HARRIS_PROBE_NONE) return harris_launch::launch_stream_probe(kind, nullptr, nullptr, 0, stream);
    if (bytes == 0) return HARRIS_OK;
    if (dst == nullptr || (kind == HARRIS_PROBE_READ && src == nullptr)) return HARRIS_ERR_NULL;
    if (bytes % 16 != 0 || pointer_alignment(dst) < 16 || (kind == HARRIS_PROBE_READ && pointer_alignment(src) < 16)) return HARRIS_ERR_ARG;
    return harris_launch::launch_stream_probe(kind, src, dst, bytes, stream);
}

const char* harris_strerror(int status) {
    switch (status) {
        case HARRIS_OK: return "success";
        case HARRIS_ERR_NULL: return "rgb or out is NULL for a non-empty result";
        case HARRIS_ERR_SHAPE: return "invalid shape: batch < 0, H < 4, W < 4, too many tiles, or pitches smaller than the image";
        case HARRIS_ERR_ARG: return "invalid argument: non-finite k or sobel_scale, misaligned pointer, unknown dtype, window, grouping or tuning, workspace too small";
        case HARRIS_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        case HARRIS_ERR_SCRATCH: return "the problem needs more scratch memory than the library's fixed buffer holds (HARRIS_GROUPED_SCRATCH_BYTES)";
        default: return "unknown harris_status";
    }
}

int harris_version(void) { return kVersion; }

}  // extern "C"
