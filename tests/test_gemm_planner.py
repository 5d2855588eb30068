"""Host logic of the GEMM launch planner (no GPU): its choices respect the contract of the kernels
for every shape of the workloads."""
import ctypes as C

import pytest


@pytest.fixture(scope="module")
def lib():
    import os
    from paper_2503_18989_amd.binding import lib_path, load_library
    if not os.path.exists(lib_path()):
        from paper_2503_18989_amd.build import build
        build(verbose=False)
    return load_library()


def plan(lib, T, Nw, Nout, K, epi, part_rows):
    t, k = C.c_int32(-7), C.c_int32(-7)
    assert lib.hat_mid_debug_gemm_plan(T, Nw, Nout, K, epi, part_rows, C.byref(t), C.byref(k)) == 0
    return t.value, k.value


SHAPES = {   # name: (Nw, Nout, K, epilogue)   7B- and 13B-shaped layers, tiny
    "qkv7": (12288, 12288, 4096, 0), "o7": (4096, 4096, 4096, 2), "gu7": (22016, 11008, 4096, 1), "down7": (4096, 4096, 11008, 2),
    "qkv13": (15360, 15360, 5120, 0), "o13": (5120, 5120, 5120, 2), "gu13": (27648, 13824, 5120, 1), "down13": (5120, 5120, 13824, 2),
    "qkvT": (768, 768, 256, 0), "oT": (256, 256, 256, 2), "guT": (1536, 704, 256, 1), "downT": (256, 256, 704, 2),
}


@pytest.mark.parametrize("T", [1, 5, 32, 150, 256, 700, 1380, 3556, 5220, 8192])
def test_choices_are_launchable(lib, T):
    n_tiles = lib.hat_mid_debug_gemm_tile_count()
    for name, (Nw, Nout, K, epi) in SHAPES.items():
        for part_rows in (0, 4096):
            tile, ks = plan(lib, T, Nw, Nout, K, epi, part_rows)
            assert 0 <= tile < n_tiles, name
            assert ks >= 1
            if epi != 2 or part_rows == 0:
                assert ks == 1, "only the accumulating epilogue with a partial-sum buffer may split K (%s)" % name
            else:
                assert ks * T <= part_rows or ks == 1
                assert K // 64 // ks >= 1


def test_small_batches_split_k_and_large_ones_do_not(lib):
    # few token rows: the 4096 x 4096 projection has 16-32 feature tiles, so K is split to fill the CUs;
    # thousands of rows give enough tiles by themselves
    assert plan(lib, 256, 4096, 4096, 4096, 2, 4096)[1] > 1
    assert plan(lib, 3556, 4096, 4096, 4096, 2, 4096)[1] == 1
    assert plan(lib, 256, 4096, 4096, 4096, 2, 0)[1] == 1


def test_null_outputs_are_refused(lib):
    assert lib.hat_mid_debug_gemm_plan(256, 4096, 4096, 4096, 2, 4096, None, None) == -1


def tile_info(lib, tile):
    v = [C.c_int32(-1) for _ in range(5)]
    rc = lib.hat_mid_debug_gemm_tile_info(tile, *[C.byref(x) for x in v])
    return rc, tuple(x.value for x in v)


def test_tile_table_fits_the_hardware(lib):
    n = lib.hat_mid_debug_gemm_tile_count()
    assert n >= 20
    for t in range(n):
        rc, (bf, bt, waves, bk, ns) = tile_info(lib, t)
        assert rc == 0
        assert bf % 32 == 0 and bt % 32 == 0 and bk % 16 == 0 and 2 <= ns <= 4
        assert waves in (2, 4, 8)
        assert ns * (bf + bt) * bk * 2 <= 160 * 1024, "ring of tile %d exceeds the LDS of a CU" % t
        # accumulators (fp32, 64 lanes per wave) + operands must fit the register file of the waves' SIMDs
        acc_regs = bf * bt // (waves * 64)
        assert acc_regs <= (256 if waves == 8 else 512) - 56, "tile %d: %d accumulator registers per lane" % (t, acc_regs)
    assert tile_info(lib, n)[0] == -1 and tile_info(lib, -1)[0] == -1
    assert lib.hat_mid_debug_gemm_tile_info(0, None, None, None, None, None) == 0


def test_small_batches_keep_power_of_two_token_tiles_and_large_ones_use_the_big_tile(lib):
    for T in (1, 32, 128, 150, 161, 256, 384):
        for name, (Nw, Nout, K, epi) in SHAPES.items():
            tile, _ = plan(lib, T, Nw, Nout, K, epi, 4096)
            bt = tile_info(lib, tile)[1][1]
            # the one exception: 129 .. 160 rows may take the 160-row token tile (one token tile instead of two)
            assert bt & (bt - 1) == 0 or (bt == 160 and 128 < T <= 160), "%s at T=%d took a %d-row token tile" % (name, T, bt)
    for name in ("o7", "gu7", "down7", "o13", "gu13", "down13"):     # 30 devices x 5 draft rows: the verify-heavy batch
        Nw, Nout, K, epi = SHAPES[name]
        tile, _ = plan(lib, 150, Nw, Nout, K, epi, 4096)
        assert tile_info(lib, tile)[1][:2] == (128, 160), name
    for name in ("qkv7", "gu7", "qkv13", "gu13"):
        Nw, Nout, K, epi = SHAPES[name]
        tile, ks = plan(lib, 8192, Nw, Nout, K, epi, 4096)
        bf, bt, waves = tile_info(lib, tile)[1][:3]
        assert (bf, bt, waves, ks) == (256, 256, 8, 1), name
    # 2200 rows: 8.6 tiles of 256 rows; the 160-row tile (13.75 -> 14 tiles, 2 % padding instead of 5 %, and a tile count
    # that packs the 256 CUs better) measured 21-23 % faster on the O and down projections
    for name in ("o7", "down7"):
        Nw, Nout, K, epi = SHAPES[name]
        tile, ks = plan(lib, 2200, Nw, Nout, K, epi, 4096)
        assert tile_info(lib, tile)[1][1] in (160, 192)
