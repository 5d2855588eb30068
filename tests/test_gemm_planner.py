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
