"""Host-side checks of libharris that need no GPU: the library loads, exports every
symbol include/harris.h declares, plans launches sensibly and rejects bad arguments
before anything is enqueued."""
import ctypes
import os
import re
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_2212_12035_amd as p
    if not os.path.exists(p.library_path()):
        from paper_2212_12035_amd import build
        build.build_library()
    p.load_library()
    return p


def test_every_declared_symbol_is_exported(pkg):
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(harris_[a-z0-9_]+)\s*\(", header))
    assert declared == set(pkg.binding.EXPORTS)
    # the operator's own header stands alone: no launch-shape knobs in it
    public = open(os.path.join(ROOT, "include", "harris.h")).read()
    assert "HARRIS_TUNE_" not in re.sub(r"/\*.*?\*/", "", public, flags=re.S) and "harris_plan" not in public
    lib = ctypes.CDLL(pkg.library_path())
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_strerror(pkg):
    assert pkg.harris_version() >= 100
    assert pkg.harris_strerror(0) == "success"
    msgs = {pkg.harris_strerror(s) for s in (-1, -2, -3, -4, -5)}
    assert len(msgs) == 5 and all(m and m != "unknown harris_status" for m in msgs)
    assert pkg.harris_strerror(-99) == "unknown harris_status"


def test_plan_picks_widest_vector_path(pkg):
    shape, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560)
    assert shape["px"] == 4 and blocks > 128 and shape["rows"] >= 4
    # The tile kernel keeps four pixels per lane for any width and any row alignment the element
    # type allows (word-aligned vector accesses; 8-bit rows loaded as aligned words and shifted);
    # strip borders then stay where they are.
    for args, kw in (((pkg.HARRIS_F32, 1, 64, 98), {}), ((pkg.HARRIS_F32, 1, 64, 97), {}),
                     ((pkg.HARRIS_F32, 1, 64, 96), dict(rgb_align=4)), ((pkg.HARRIS_F32, 1, 64, 96), dict(out_align=8)),
                     ((pkg.HARRIS_U8, 1, 64, 96), dict(rgb_align=1)), ((pkg.HARRIS_U8, 1, 64, 99), dict(rgb_align=1, out_align=4))):
        shape = pkg.harris_plan(*args, **kw)[0]
        assert shape["px"] == 4 and shape["schedule"] == pkg.HARRIS_SCHEDULE_TILES and shape["flags"] & pkg.HARRIS_TUNE_PLAIN_STORES, (args, kw)
        with pytest.raises(pkg.HarrisError) as e:           # moved borders need naturally aligned lanes
            pkg.harris_plan(*args, tuning=dict(flags=pkg.HARRIS_TUNE_ALIGNED_STORES), **kw)
        assert e.value.status == -3
    # shifted 8-bit rows: strips of at most 248 columns (the last lane only supplies bytes): 500 columns take 3, not 2
    plain = dict(rows=4, waves_per_block=4, flags=pkg.HARRIS_TUNE_PLAIN_STORES)
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 64, 504, tuning=plain)[1] == 2 * 5
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 64, 504, rgb_align=1, tuning=plain)[1] == 3 * 5
    # the band schedule keeps naturally aligned lanes: narrower ones for such rows
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 64, 98, tuning=dict(schedule=1))[0]["px"] == 2
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 64, 97, tuning=dict(schedule=1))[0]["px"] == 1
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 64, 96, rgb_align=4, tuning=dict(schedule=1))[0]["px"] == 1
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 64, 96, out_align=8, tuning=dict(schedule=1))[0]["px"] == 2
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 64, 96, rgb_align=1, tuning=dict(schedule=1))[0]["px"] == 1
    # 8-bit codes are one word per lane: rows of codes off 4-byte boundaries take narrower lanes
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_U8, 1, 64, 98, out_align=1)[0]["px"] == 1
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_F16, 1, 64, 98, out_align=4)[0]["px"] == 4
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_F16, 1, 64, 97, out_align=2)[0]["px"] == 1
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 8192, 8192)[0]["px"] == 4


def test_plan_tile_arithmetic(pkg):
    # 252 result columns per wavefront at px = 4; 2556 columns -> 11 strips; 1532 rows in
    # bands of 16 -> 96 bands; 4 wavefronts per workgroup.
    t = dict(schedule=pkg.HARRIS_SCHEDULE_BANDS, px=4, rows=16, prefetch=3, waves_per_block=4, flags=pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_PLAIN_STORES)
    shape, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560, tuning=t)
    assert shape == dict(t, lds_kb=0) and blocks == 6 * 48          # 2 strips x 2 bands per workgroup: ceil(11/2) x ceil(96/2)
    shape, blocks = pkg.harris_plan(pkg.HARRIS_F32, 3, 9, 9, tuning=dict(schedule=1, px=1, rows=2, prefetch=3, waves_per_block=1, flags=3))
    assert blocks == 3 * 3 * 1
    # tiles: 8 wavefronts x 8 rows give 60 result rows per tile -> 26 tiles down, 11 across,
    # one workgroup each
    t = dict(schedule=pkg.HARRIS_SCHEDULE_TILES, px=4, rows=8, prefetch=0, waves_per_block=8, flags=pkg.HARRIS_TUNE_CACHED_LOADS | pkg.HARRIS_TUNE_PLAIN_STORES)
    shape, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560, tuning=t)
    assert shape == dict(t, lds_kb=32) and blocks == 26 * 11      # 8 wavefronts publish 4 KB each
    # strip borders moved to 64-byte boundaries: strips of at most 240 columns; 4252 columns
    # take 18 of them instead of 17, 2556 columns still 11
    aligned = dict(t, flags=pkg.HARRIS_TUNE_CACHED_LOADS | pkg.HARRIS_TUNE_ALIGNED_STORES)
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560, tuning=aligned) == (dict(aligned, lds_kb=32), 26 * 11)
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 4256, tuning=aligned)[1] == 26 * 18
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 4256, tuning=t)[1] == 26 * 17
    # empty results plan to zero workgroups
    assert pkg.harris_plan(pkg.HARRIS_F32, 0, 64, 64)[1] == 0
    assert pkg.harris_plan(pkg.HARRIS_F32, 2, 4, 64)[1] == 0
    assert pkg.harris_plan(pkg.HARRIS_F32, 2, 64, 4)[1] == 0


def test_plan_defaults_follow_the_problem_size(pkg):
    small, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560)
    # one tile per CU: 11 strips x 23 tiles of 9 wavefronts x 8 rows (68 result rows) = 253 workgroups
    assert small["schedule"] == pkg.HARRIS_SCHEDULE_TILES and (small["rows"], small["waves_per_block"]) == (8, 9) and blocks == 253
    assert small["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_ALIGNED_STORES | pkg.HARRIS_TUNE_FLAG_HANDOFF
    # few, tall tiles take ready flags instead of the barrier; tiles of fewer than 5 wavefronts keep the barrier
    assert not pkg.harris_plan(pkg.HARRIS_F32, 1, 720, 1280)[0]["flags"] & pkg.HARRIS_TUNE_FLAG_HANDOFF
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1080, 1920)[0]["flags"] & pkg.HARRIS_TUNE_FLAG_HANDOFF
    assert not pkg.harris_plan(pkg.HARRIS_U8, 1, 2048, 4096)[0]["flags"] & pkg.HARRIS_TUNE_FLAG_HANDOFF     # 8-bit input keeps the barrier
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560, tuning=dict(flags=pkg.HARRIS_TUNE_STREAM_LOADS))[0]["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_ALIGNED_STORES
    # short tiles take few rows per wavefront, and several images with short tiles take many small tiles
    assert [pkg.harris_plan(pkg.HARRIS_F32, 1, 768, 1024)[0][key] for key in ("rows", "waves_per_block")] == [5, 4]
    assert [pkg.harris_plan(pkg.HARRIS_F32, 1, 1024, 1024)[0][key] for key in ("rows", "waves_per_block")] == [6, 4]
    assert [pkg.harris_plan(pkg.HARRIS_F32, 1, 2160, 3840)[0][key] for key in ("rows", "waves_per_block")] == [10, 14]
    # 8-bit input: fewer rows per wavefront for tall tiles
    assert [pkg.harris_plan(pkg.HARRIS_U8, 1, 1536, 2560)[0][key] for key in ("rows", "waves_per_block")] == [6, 12]
    assert [pkg.harris_plan(pkg.HARRIS_U8, 1, 2160, 3840)[0][key] for key in ("rows", "waves_per_block")] == [9, 16]
    # tiles of 26 to 32 rows (40 for 8-bit input) give way to many small tiles
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 960, 1280)[1] == 6 * 80 and pkg.harris_plan(pkg.HARRIS_F32, 1, 1080, 1920)[1] <= 256
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 1080, 1920)[1] == 8 * 90
    # ... for float32 input only while at most two small tiles come to lie on a CU (512 in all): 900x1600 would be 525
    mid, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 900, 1600)
    assert (mid["rows"], mid["waves_per_block"]) == (6, 5) and blocks == 7 * 35 and mid["flags"] & pkg.HARRIS_TUNE_FLAG_HANDOFF
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1024, 1280)[1] == 6 * 85
    two, blocks = pkg.harris_plan(pkg.HARRIS_F32, 2, 720, 1280)
    assert (two["rows"], two["waves_per_block"]) == (5, 8) and blocks == 2 * 6 * 20
    several, blocks = pkg.harris_plan(pkg.HARRIS_F32, 4, 480, 640)
    assert (several["rows"], several["waves_per_block"]) == (4, 4) and blocks == 4 * 3 * 40
    # beyond one tile per CU: many tiles, non-temporal loads except the rows two tiles share, which stay in L2,
    # and an LDS reservation that holds the tiles resident on a CU down (160 KB per CU).
    # float32 results of 128 to 400 MB: 4 wavefronts x 5 rows (16 result rows per tile), 3 tiles per CU
    mid, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 2832, 4256)
    assert (mid["schedule"], mid["rows"], mid["waves_per_block"], mid["lds_kb"]) == (2, 5, 4, 48) and blocks == 18 * 177
    assert mid["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS | pkg.HARRIS_TUNE_ALIGNED_STORES
    assert [pkg.harris_plan(pkg.HARRIS_F32, 2, 2160, 3840)[0][key] for key in ("rows", "waves_per_block", "lds_kb")] == [5, 4, 48]
    # beyond 400 MB: 8 images or more 5 wavefronts x 5 rows (21 result rows per tile), fewer images 5 x 6; 2 tiles per CU
    assert [pkg.harris_plan(pkg.HARRIS_F32, 16, 1080, 1920)[0][key] for key in ("rows", "waves_per_block", "lds_kb")] == [5, 5, 64]
    assert [pkg.harris_plan(pkg.HARRIS_F32, 1, 8192, 8192)[0][key] for key in ("rows", "waves_per_block", "lds_kb")] == [6, 5, 64]
    big, blocks = pkg.harris_plan(pkg.HARRIS_F32, 64, 1080, 1920)
    assert (big["rows"], big["waves_per_block"], big["lds_kb"]) == (5, 5, 64) and blocks == 64 * 52 * 8
    assert big["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS | pkg.HARRIS_TUNE_ALIGNED_STORES
    # 16-bit results above 128 MB: 4 x 6, 3 tiles per CU; one image beyond 800 MB: 5 x 6, 2 per CU
    half, _ = pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_F16, 64, 1080, 1920)
    assert (half["rows"], half["waves_per_block"], half["lds_kb"]) == (6, 4, 48)
    assert half["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS | pkg.HARRIS_TUNE_ALIGNED_STORES
    wide, _ = pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_BF16, 1, 8192, 8192)
    assert (wide["rows"], wide["waves_per_block"], wide["lds_kb"]) == (6, 5, 64)
    # an explicit shape gets no reservation beyond the tile's own rows (4 KB per wavefront); an explicit one is kept
    assert pkg.harris_plan(pkg.HARRIS_F32, 64, 1080, 1920, tuning=dict(rows=5, waves_per_block=5))[0]["lds_kb"] == 20
    assert pkg.harris_plan(pkg.HARRIS_F32, 64, 1080, 1920, tuning=dict(rows=5, waves_per_block=5, lds_kb=40))[0]["lds_kb"] == 40
    assert pkg.harris_plan(pkg.HARRIS_F32, 64, 1080, 1920, tuning=dict(lds_kb=28))[0]["lds_kb"] == 28
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560)[0]["lds_kb"] == 36            # one tile per CU: 9 wavefronts, no more
    # 8-bit input takes every wavefront that fits
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 8192, 8192)[0]["lds_kb"] == 16
    # many tiles below 128 MB as well (32 images of 512x512 cannot be one tile per CU): shared rows kept
    many, blocks = pkg.harris_plan(pkg.HARRIS_F32, 32, 512, 512)
    assert (many["rows"], many["waves_per_block"], many["lds_kb"]) == (4, 4, 36) and blocks > 256
    assert many["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS | pkg.HARRIS_TUNE_ALIGNED_STORES
    # lanes narrower than 16 bytes have no mixed policy: default-policy loads from 128 MB on
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 2832, 4258, tuning=dict(px=2))[0]["flags"] == pkg.HARRIS_TUNE_CACHED_LOADS | pkg.HARRIS_TUNE_PLAIN_STORES
    # a width that is no multiple of 4 keeps the 16-byte lanes and their policy, with fixed strip borders
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 2832, 4258)[0]["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS | pkg.HARRIS_TUNE_PLAIN_STORES
    # 8-bit input: non-temporal loads; 35 strips of at most 240 columns cover 8188
    u8, blocks = pkg.harris_plan(pkg.HARRIS_U8, 1, 8192, 8192)
    assert u8["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_KEEP_SHARED_ROWS | pkg.HARRIS_TUNE_ALIGNED_STORES and blocks == 35 * 683
    assert (u8["rows"], u8["waves_per_block"]) == (4, 4)
    assert pkg.harris_plan(pkg.HARRIS_U8, 1, 64, 98, rgb_align=1)[0]["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_PLAIN_STORES
    # narrower lanes and bands never move strip borders
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 64, 98)[0]["flags"] & pkg.HARRIS_TUNE_PLAIN_STORES
    assert pkg.harris_plan(pkg.HARRIS_F32, 1, 64, 96, tuning=dict(schedule=1))[0]["flags"] & pkg.HARRIS_TUNE_PLAIN_STORES
    # an explicit policy is kept
    kept, _ = pkg.harris_plan(pkg.HARRIS_F32, 64, 1080, 1920, tuning=dict(flags=pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_PLAIN_STORES))
    assert kept["flags"] == pkg.HARRIS_TUNE_STREAM_LOADS | pkg.HARRIS_TUNE_PLAIN_STORES
    # asking for bands gives bands: one wavefront per SIMD for small problems, four-wavefront groups for large
    bands, blocks = pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560, tuning=dict(schedule=1))
    assert (bands["rows"], bands["prefetch"], bands["waves_per_block"]) == (17, 3, 1) and blocks == 1001
    bands, blocks = pkg.harris_plan(pkg.HARRIS_F32, 64, 1080, 1920, tuning=dict(schedule=1))
    assert (bands["rows"], bands["prefetch"], bands["waves_per_block"]) == (32, 3, 4) and blocks == 64 * 17 * 4


def test_plan_rejects_bad_arguments(pkg):
    E = pkg.HarrisError
    for args, status in [
        ((7, 1, 64, 64), -3),                       # unknown dtype
        ((0, -1, 64, 64), -2), ((0, 1, 3, 64), -2), ((0, 1, 64, 3), -2),
        ((0, 2 ** 31 - 1, 4096, 4096), -2),         # more tiles than a grid can hold
        ((0, 1, 8, 2 ** 28 + 4), -2),               # row offsets would not fit 32 bits
        ((0, 1, 2 ** 30 + 1, 8), -2),               # row indices would not fit int
        ((0, 2 ** 31 - 1, 2 ** 30, 2 ** 28), -2),   # byte counts would not fit 64 bits
        ((1, 2 ** 20, 2 ** 30, 2 ** 28), -2),
    ]:
        with pytest.raises(E) as e:
            pkg.harris_plan(*args)
        assert e.value.status == status
    for bad in (dict(px=3), dict(px=4, prefetch=5), dict(schedule=1, px=4, waves_per_block=3), dict(waves_per_block=1), dict(flags=256), dict(flags=12), dict(flags=48), dict(flags=64), dict(flags=64 | 4), dict(schedule=1, flags=64 | 8), dict(px=2, flags=64 | 8),
                dict(flags=128 | 4), dict(flags=128 | 64 | 8), dict(schedule=1, flags=128), dict(px=2, flags=128), dict(schedule=1, flags=16), dict(px=2, flags=16), dict(rows=-1),
                dict(schedule=3), dict(schedule=2, rows=7), dict(schedule=2, px=2, rows=5), dict(schedule=2, waves_per_block=1), dict(schedule=2, waves_per_block=17),
                dict(schedule=2, prefetch=3), dict(schedule=2, px=8), dict(px=8), dict(prefetch=2), dict(schedule=1, prefetch=6), dict(schedule=2, px=2, rows=8),
                dict(lds_kb=65), dict(lds_kb=-1), dict(schedule=1, lds_kb=16)):
        with pytest.raises(E) as e:
            pkg.harris_plan(0, 1, 64, 64, tuning=bad)
        assert e.value.status == -3
    with pytest.raises(E):                          # px = 4 in the band schedule needs W % 4 == 0
        pkg.harris_plan(0, 1, 64, 98, tuning=dict(schedule=1, px=4))
    with pytest.raises(E) as e:                     # ready flags: float32 input only
        pkg.harris_plan(pkg.HARRIS_U8, 1, 64, 64, tuning=dict(flags=pkg.HARRIS_TUNE_FLAG_HANDOFF))
    assert e.value.status == -3


def test_plan_for_16_bit_results(pkg):
    # 16-bit results: tile kernel only; moved strip borders reach up to 28 columns (64 bytes),
    # so strips are at most 224 columns; the widest lanes need 8-byte aligned result rows.
    F16, BF16 = pkg.HARRIS_OUT_F16, pkg.HARRIS_OUT_BF16
    shape, blocks = pkg.harris_plan_typed(pkg.HARRIS_F32, F16, 64, 1080, 1920)
    assert shape["schedule"] == pkg.HARRIS_SCHEDULE_TILES and shape["px"] == 4 and shape["flags"] & pkg.HARRIS_TUNE_ALIGNED_STORES
    assert blocks == 64 * 54 * 9                                # ceil(1916 / 224) = 9 strips (8 for float32 results); tiles of 20 result rows
    # small problems and 8-bit input keep the wider strips with fixed borders
    small, blocks = pkg.harris_plan_typed(pkg.HARRIS_F32, F16, 1, 1536, 2560)
    assert small["flags"] & pkg.HARRIS_TUNE_PLAIN_STORES and (small["rows"], small["waves_per_block"]) == (8, 9) and blocks == 253
    assert pkg.harris_plan_typed(pkg.HARRIS_U8, BF16, 1, 8192, 8192)[0]["flags"] & pkg.HARRIS_TUNE_PLAIN_STORES
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, F16, 1, 1536, 2560, tuning=dict(flags=pkg.HARRIS_TUNE_ALIGNED_STORES))[1] % 12 == 0
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, BF16, 1, 64, 96, out_align=4)[0]["px"] == 4      # word-aligned 8-byte stores
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, BF16, 1, 64, 96, out_align=2)[0]["px"] == 1
    # rows with an odd number of 16-bit results: the last column would share a 32-bit word with what lies behind the row
    for odd in (97, 131, 1001):
        assert pkg.harris_plan_typed(pkg.HARRIS_F32, F16, 2, 64, odd, out_align=4)[0]["px"] == 1
        assert pkg.harris_plan_typed(pkg.HARRIS_U8, BF16, 2, 64, odd, rgb_align=1, out_align=4)[0]["px"] == 1
        assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_F32, 2, 64, odd, out_align=4)[0]["px"] == 4
        with pytest.raises(pkg.HarrisError):
            pkg.harris_plan_typed(pkg.HARRIS_F32, F16, 2, 64, odd, out_align=4, tuning=dict(px=4))
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_F32, 1, 1536, 2560) == pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560)
    for bad in (dict(out_dtype=4), dict(out_dtype=F16, tuning=dict(schedule=1)), dict(out_dtype=F16, tuning=dict(prefetch=3)),
                dict(out_dtype=F16, out_align=1), dict(out_dtype=F16, tuning=dict(px=8))):
        with pytest.raises(pkg.HarrisError) as e:
            pkg.harris_plan_typed(pkg.HARRIS_F32, bad["out_dtype"], 1, 64, 96, out_align=bad.get("out_align", 16), tuning=bad.get("tuning"))
        assert e.value.status == -3
    # 8-bit results: plain strips by default, at most 192 columns with moved borders, byte-aligned rows allowed
    u8out, blocks = pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_U8, 64, 1080, 1920)
    assert u8out["flags"] & pkg.HARRIS_TUNE_PLAIN_STORES and blocks == 64 * 54 * 8
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_U8, 64, 1080, 1920, tuning=dict(flags=pkg.HARRIS_TUNE_ALIGNED_STORES))[1] == 64 * 54 * 10
    assert pkg.harris_plan_typed(pkg.HARRIS_F32, pkg.HARRIS_OUT_U8, 1, 64, 96, out_align=1)[0]["px"] == 1
    lib = pkg.load_library()
    one = ctypes.c_void_p(4096)
    assert lib.harris_coarsity_typed(one, 0, 1, 64, 64, None, 0.04, 1.0, 0, one, 7, None, None) == -3
    assert lib.harris_coarsity_typed(one, 0, 1, 64, 64, None, 0.04, 1.0, 0, one, pkg.HARRIS_OUT_U8, None, None) == -3   # 8-bit codes need a scale
    assert lib.harris_coarsity_quantized(one, 0, 1, 64, 64, None, 0.04, 1.0, 0, float("nan"), 0.0, one, None, None) == -3
    assert lib.harris_coarsity_quantized(one, 0, 1, 64, 64, None, 0.04, 1.0, 0, 1.0, float("inf"), one, None, None) == -3
    assert lib.harris_coarsity_quantized(None, 0, 1, 64, 64, None, 0.04, 1.0, 0, 1.0, 0.0, one, None, None) == -1
    assert lib.harris_coarsity_quantized(None, 0, 0, 64, 64, None, 0.04, 1.0, 0, 1.0, 0.0, None, None, None) == 0
    assert lib.harris_coarsity_typed(one, 0, 1, 64, 64, None, 0.04, 1.0, 0, ctypes.c_void_p(4097), 1, None, None) == -3
    assert lib.harris_coarsity_typed(None, 0, 0, 64, 64, None, 0.04, 1.0, 0, None, 2, None, None) == 0


def test_copy_probe_validates_its_arguments(pkg):
    lib = pkg.load_library()
    one = ctypes.c_void_p(4096)
    assert lib.harris_probe_copy(None, 0, 1, 64, 64, one, None) == -1
    assert lib.harris_probe_copy(one, 2, 1, 64, 64, one, None) == -3
    assert lib.harris_probe_copy(one, 0, 1, 3, 64, one, None) == -2
    assert lib.harris_probe_copy(ctypes.c_void_p(4100), 0, 1, 64, 64, one, None) == -3      # rgb not 16-byte aligned
    assert lib.harris_probe_copy(one, 1, 1, 5, 7, one, None) == -3                           # planes of 35 bytes
    assert lib.harris_probe_copy(one, 0, 1, 9, 11, one, None) == -3                          # 35 results: rows of images not 16-byte multiples
    assert lib.harris_probe_copy(None, 0, 0, 64, 64, None, None) == 0


def test_stream_probe_validates_its_arguments(pkg):
    lib = pkg.load_library()
    one = ctypes.c_void_p(4096)
    assert lib.harris_probe_stream(0, one, one, 1024, None) == -3                      # unknown kind
    assert lib.harris_probe_stream(4, one, one, 1024, None) == -3
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_NONE, None, None, -1, None) == -2     # the idle launch ignores all but the sign
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_READ, None, one, 1024, None) == -1
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_READ, one, None, 1024, None) == -1
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_WRITE, None, None, 1024, None) == -1
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_WRITE, None, one, 1000, None) == -3     # not a multiple of 16
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_WRITE, None, ctypes.c_void_p(4100), 1024, None) == -3
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_READ, ctypes.c_void_p(4104), one, 1024, None) == -3
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_WRITE, None, one, -16, None) == -2
    assert lib.harris_probe_stream(pkg.HARRIS_PROBE_READ, None, None, 0, None) == 0          # nothing to move


def test_index_division_by_multiplication_is_exact(tmp_path):
    # The tile kernel splits its workgroup index with a multiply-high division whose constants
    # the host computes; the same header functions are checked here against the hardware division.
    import subprocess
    exe = str(tmp_path / "fastdiv_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
                    "-I" + os.path.join(ROOT, "paper_2212_12035_amd", "csrc"),
                    os.path.join(ROOT, "tests", "fastdiv_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.startswith("ok "), out.stdout


def test_entry_points_validate_before_touching_the_device(pkg):
    # None of these reaches a kernel launch, so they are safe without a GPU.
    lib = pkg.load_library()
    nan = float("nan")
    one = ctypes.c_void_p(4096)
    assert lib.harris_coarsity(None, 1, 64, 64, 0.04, one, None) == -1
    assert lib.harris_coarsity(one, 1, 64, 64, 0.04, None, None) == -1
    assert lib.harris_coarsity(one, 1, 3, 64, 0.04, one, None) == -2
    assert lib.harris_coarsity(one, -1, 64, 64, 0.04, one, None) == -2
    assert lib.harris_coarsity(one, 1, 64, 64, nan, one, None) == -3
    assert lib.harris_coarsity_u8(one, 1, 64, 64, float("inf"), one, None) == -3
    assert lib.harris_coarsity_ex(one, 0, 1, 64, 64, 0.04, nan, 0, one, None, None) == -3
    assert lib.harris_coarsity_ex(one, 0, 1, 64, 64, 0.04, 1.0, 2, one, None, None) == -3
    assert lib.harris_coarsity_ex(one, 5, 1, 64, 64, 0.04, 1.0, 0, one, None, None) == -3
    assert lib.harris_coarsity_ex(one, 0, 1, 64, 64, 0.04, 1.0, 0, ctypes.c_void_p(4098), None, None) == -3  # out not 4-byte aligned
    # empty results succeed without looking at the pointers
    assert lib.harris_coarsity(None, 0, 64, 64, 0.04, None, None) == 0
    assert lib.harris_coarsity(None, 3, 4, 64, 0.04, None, None) == 0
    assert lib.harris_coarsity_u8(None, 3, 64, 4, 0.04, None, None) == 0


def test_grouped_workspace_sizes_and_validation(pkg):
    lib = pkg.load_library()
    H, W = 10, 12
    n0, n2, n4 = H * W, (H - 2) * (W - 2), (H - 4) * (W - 4)
    assert pkg.harris_grouped_workspace_bytes(1, 2, H, W) == 4 * 2 * (n0 + 5 * n2 + 3 * n4)
    assert pkg.harris_grouped_workspace_bytes(2, 2, H, W) == 4 * 2 * (n0 + 3 * n2)
    assert pkg.harris_grouped_workspace_bytes(3, 2, H, W) == 4 * 2 * (n0 + 2 * n2)
    assert pkg.harris_grouped_workspace_bytes(4, 2, H, W) == 0
    assert pkg.harris_grouped_workspace_bytes(5, 2, H, W) == -1 and pkg.harris_grouped_workspace_bytes(1, 2, 3, W) == -1
    one = ctypes.c_void_p(4096)
    need = pkg.harris_grouped_workspace_bytes(1, 1, H, W)
    assert lib.harris_coarsity_grouped(one, 0, 1, H, W, 0.04, 1.0, 0, 0, one, need, one, None) == -3      # grouping 0
    assert lib.harris_coarsity_grouped(one, 0, 1, H, W, 0.04, 1.0, 0, 1, one, need - 4, one, None) == -3  # workspace too small
    assert lib.harris_coarsity_grouped(one, 0, 1, H, W, 0.04, 1.0, 0, 1, None, need, one, None) == -1
    assert lib.harris_coarsity_grouped(one, 0, 1, 3, W, 0.04, 1.0, 0, 2, one, need, one, None) == -2
    assert lib.harris_coarsity_grouped(None, 0, 0, H, W, 0.04, 1.0, 0, 3, None, 0, None, None) == 0


def test_static_scratch_entry_rejects_what_does_not_fit(pkg):
    # Checked on the host before anything touches a device.
    lib = pkg.load_library()
    one = ctypes.c_void_p(4096)
    cap = pkg.HARRIS_GROUPED_SCRATCH_BYTES
    assert cap == 64 << 20
    assert pkg.harris_grouped_workspace_bytes(2, 1, 1536, 2560) <= cap < pkg.harris_grouped_workspace_bytes(1, 1, 1536, 2560)
    assert lib.harris_coarsity_grouped_static(one, 0, 1, 1536, 2560, 0.04, 1.0, 0, 1, one, None) == -5
    assert lib.harris_coarsity_grouped_static(one, 0, 64, 1080, 1920, 0.04, 1.0, 0, 3, one, None) == -5
    assert lib.harris_coarsity_grouped_static(one, 0, 2 ** 31 - 1, 2 ** 30, 2 ** 28, 0.04, 1.0, 0, 2, one, None) == -5
    assert lib.harris_coarsity_grouped_static(one, 0, 1, 64, 64, 0.04, 1.0, 0, 0, one, None) == -3      # grouping 0
    assert lib.harris_coarsity_grouped_static(one, 0, 1, 64, 64, 0.04, 1.0, 0, 5, one, None) == -3
    assert lib.harris_coarsity_grouped_static(one, 0, 1, 3, 64, 0.04, 1.0, 0, 1, one, None) == -2
    assert lib.harris_coarsity_grouped_static(None, 0, 1, 64, 64, 0.04, 1.0, 0, 1, one, None) == -1
    assert lib.harris_coarsity_grouped_static(None, 0, 0, 64, 64, 0.04, 1.0, 0, 2, None, None) == 0       # empty: no work, no scratch
    assert lib.harris_coarsity_grouped_static(None, 0, 3, 4, 64, 0.04, 1.0, 0, 3, None, None) == 0
    assert "scratch" in pkg.harris_strerror(-5)


def test_pitched_entry_validates_the_layout(pkg):
    lib = pkg.load_library()
    one = ctypes.c_void_p(4096)
    H, W = 10, 12

    def call(**kw):
        lay = dict(rgb_row_pitch=W, rgb_plane_pitch=H * W, rgb_image_pitch=3 * H * W, out_row_pitch=W - 4, out_image_pitch=(H - 4) * (W - 4))
        lay.update(kw)
        return lib.harris_coarsity_pitched(one, 0, 2, H, W, ctypes.byref(pkg.HarrisLayout(**lay)), 0.04, 1.0, 0, one, None, None)

    assert call(rgb_row_pitch=W - 1) == -2
    assert call(rgb_plane_pitch=H * W - 1) == -2
    assert call(rgb_image_pitch=3 * H * W - 1) == -2
    assert call(out_row_pitch=W - 5) == -2
    assert call(out_image_pitch=(H - 4) * (W - 4) - 1) == -2
    # padded rows need matching plane pitch
    assert call(rgb_row_pitch=W + 4) == -2
    # NULL layout means dense: same checks as harris_coarsity_ex
    assert lib.harris_coarsity_pitched(None, 0, 1, H, W, None, 0.04, 1.0, 0, one, None, None) == -1
    assert lib.harris_coarsity_pitched(None, 0, 0, H, W, None, 0.04, 1.0, 0, None, None, None) == 0


def test_product_sources_never_reach_for_the_oracle():
    # The oracle is test infrastructure: nothing under the package (or the headers) may name it.
    pkg_dir = os.path.join(ROOT, "paper_2212_12035_amd")
    for base, _, files in os.walk(pkg_dir):
        for name in files:
            if name.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(base, name)).read()
                assert "oracle" not in text.lower(), os.path.join(base, name)
    for name in os.listdir(os.path.join(ROOT, "include")):
        assert "oracle" not in open(os.path.join(ROOT, "include", name)).read().lower()
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert "__graft_entry__" not in bench              # the benchmark builds the library by the package's own build step
    assert "paper_2212_12035_amd" not in open(os.path.join(ROOT, "oracle", "harris_oracle.py")).read()
    assert "harris.h" not in open(os.path.join(ROOT, "oracle", "harris_ref.cpp")).read()


def test_binding_refuses_host_tensors(pkg):
    import torch
    with pytest.raises(TypeError):
        pkg.harris_coarsity(torch.zeros(1, 3, 8, 8))


def test_sweep_candidates_are_launch_shapes_the_library_knows(pkg):
    # The launch-shape sweep times the planner's choice against candidates; every candidate must be a
    # shape harris_plan accepts or cleanly refuses (never one that would only fail at launch), the
    # default must come first, and for a one-tile-per-CU size the planner's own choice must be among them.
    from paper_2212_12035_amd import sweep
    for dtype in (pkg.HARRIS_F32, pkg.HARRIS_U8):
        for B, H, W in ((1, 1536, 2560), (1, 900, 1600), (4, 480, 640), (64, 1080, 1920), (1, 8192, 8192)):
            cands = sweep.candidates(pkg, dtype, B, H, W)
            assert cands[0][0] == "default" and len({name for name, _ in cands}) == len(cands)
            accepted = []
            for name, t in cands:
                try:
                    shape, blocks = pkg.harris_plan(dtype, B, H, W, tuning=t)
                    assert blocks > 0 and shape["schedule"] == pkg.HARRIS_SCHEDULE_TILES and shape["px"] == 4
                    accepted.append((shape["rows"], shape["waves_per_block"]))
                except pkg.HarrisError as e:
                    assert e.status == -3, name
            assert len(accepted) >= 8
    chosen = pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560)[0]
    shapes = [pkg.harris_plan(pkg.HARRIS_F32, 1, 1536, 2560, tuning=t)[0] for _, t in sweep.candidates(pkg, pkg.HARRIS_F32, 1, 1536, 2560)[1:]]
    assert any((s["rows"], s["waves_per_block"], s["flags"] & pkg.HARRIS_TUNE_FLAG_HANDOFF) == (chosen["rows"], chosen["waves_per_block"], chosen["flags"] & pkg.HARRIS_TUNE_FLAG_HANDOFF) for s in shapes)


def test_benchmark_refuses_more_than_one_gpu():
    # The benchmark measures one GPU; asked for more it says so and exits before touching a device.
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr) and "{" not in r.stdout


def test_traffic_figures_belong_to_the_kernels_in_the_tree():
    # roofline.traffic is reported only while the kernel sources hash to the value recorded with
    # the counters; after a change to the kernels the figure must be re-measured, not carried over.
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    assert set(bench.TRAFFIC_BYTES) == {"noise_f32_1536x2560", "rects_f32_64x1080x1920", "blobs_f32_2832x4256", "noise_u8_8192x8192"}
    assert len(bench.TRAFFIC_SOURCES_SHA256) == 64 and len(bench.kernel_sources_sha256()) == 64
    for name, traffic in bench.TRAFFIC_BYTES.items():
        # measured HBM bytes lie between the algorithmic bytes and 1.15 times them
        import harris_inputs
        gen, seed, B, H, W, dt = harris_inputs.WORKLOADS[name]
        algo = B * (3 * H * W * (1 if dt == "u8" else 4) + 4 * (H - 4) * (W - 4))
        assert algo <= traffic <= 1.15 * algo, name
