"""Launch geometry of the MFMA GEMM, checked on the host through the functions the kernel and its launcher call
(radix_debug_gemm_tile / radix_debug_gemm_band): every output tile is computed by exactly one workgroup, whatever the
tile counts and band width - a hole would leave rows of a position-wise projection (Algorithm 1, "QKVProj",
"OProj", "MLP") unwritten, a tile index out of range would write outside the output."""
import ctypes as C
import os

import numpy as np
import pytest

from paper_2601_15013_amd import binding


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2601_15013_amd import build
        build.build()
    return binding.load_library()


def tiles(lib, tiles_m, tiles_n, band):
    tm, tn = C.c_int32(-1), C.c_int32(-1)
    out = np.empty((tiles_m * tiles_n, 2), dtype=np.int64)
    for bid in range(tiles_m * tiles_n):
        assert lib.radix_debug_gemm_tile(bid, tiles_m, tiles_n, band, C.byref(tm), C.byref(tn)) == 0
        out[bid] = (tm.value, tn.value)
    return out


@pytest.mark.parametrize("band", [1, 2, 4, 8])
def test_every_tile_exactly_once(lib, band):
    shapes = [(m, n) for m in (1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 33, 62, 63, 64, 65, 66, 100, 176, 177)
              for n in (1, 2, 3, 4, 10, 16, 24, 76, 96)]
    for tiles_m, tiles_n in shapes:
        t = tiles(lib, tiles_m, tiles_n, band)
        assert t[:, 0].min() >= 0 and t[:, 0].max() < tiles_m and t[:, 1].min() >= 0 and t[:, 1].max() < tiles_n
        flat = t[:, 0] * tiles_n + t[:, 1]
        assert len(np.unique(flat)) == tiles_m * tiles_n, (tiles_m, tiles_n, band)


def test_xcds_sweep_the_columns_in_step(lib):
    # 8 whole bands: workgroups with the same position in their XCD's queue (ids 8 q + x) work on the same column
    # tile, each on its own band of rows; the second sweep runs backwards
    tiles_m, tiles_n, band = 64, 24, 4
    t = tiles(lib, tiles_m, tiles_n, band)
    for q in range(tiles_m * tiles_n // 8):
        group = t[8 * q:8 * q + 8]
        assert len(set(group[:, 1])) == 1
        assert sorted(group[:, 0] // band % 8) == list(range(8))
    first_sweep = t[0:8 * band * tiles_n:8, 1]
    second_sweep = t[8 * band * tiles_n:16 * band * tiles_n:8, 1]
    assert list(first_sweep) == sorted(first_sweep) and list(second_sweep) == sorted(second_sweep, reverse=True)
    assert second_sweep[0] == first_sweep[-1]          # the next sweep starts on the weight strip used last


def test_band_width_follows_the_row_length(lib):
    # (tile rows, K, column tiles) of the named shapes -> band
    assert lib.radix_debug_gemm_band(256, 1024, 16) == 8       # 0.6B QKV
    assert lib.radix_debug_gemm_band(256, 4096, 96) == 4       # 8B gate/up
    assert lib.radix_debug_gemm_band(256, 4096, 24) == 4       # 8B QKV
    assert lib.radix_debug_gemm_band(256, 12288, 16) == 1      # 8B down: all 16 column tiles with 2 row tiles
    assert lib.radix_debug_gemm_band(256, 12288, 96) == 2      # many column tiles: never a single row
    assert lib.radix_debug_gemm_band(128, 3072, 4) == 8        # 0.6B down, 128-row tiles
    widths = [lib.radix_debug_gemm_band(256, k, 16) for k in (64, 512, 2048, 4096, 8192, 16384, 65536)]
    assert widths == sorted(widths, reverse=True) and widths[0] == 8 and widths[-1] == 1


def test_debug_views_reject_bad_arguments(lib):
    tm, tn = C.c_int32(), C.c_int32()
    assert lib.radix_debug_gemm_tile(0, 4, 4, 2, None, C.byref(tn)) == -1
    assert lib.radix_debug_gemm_tile(16, 4, 4, 2, C.byref(tm), C.byref(tn)) == -2
    assert lib.radix_debug_gemm_tile(-1, 4, 4, 2, C.byref(tm), C.byref(tn)) == -2
    assert lib.radix_debug_gemm_tile(0, 4, 4, 0, C.byref(tm), C.byref(tn)) == -2
    assert lib.radix_debug_gemm_band(0, 4096, 4) == -2
