"""The C-ABI library loads and exports every symbol include/*.h declares
(no compute: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        txt = open(os.path.join(ROOT, "include", header)).read()
        txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
        names |= set(re.findall(r"\b(hat_(?:mid|sched)_\w+)\s*\(", txt))
    return sorted(names)


def test_header_declares_the_three_named_calls():
    names = declared_functions()
    for n in ("hat_mid_create", "hat_mid_forward", "hat_mid_release"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2503_18989_amd.binding import lib_path, EXPORTED_SYMBOLS
    if not os.path.exists(lib_path()):
        from paper_2503_18989_amd.build import build
        build(verbose=False)
    lib = ctypes.CDLL(lib_path())
    names = declared_functions()
    assert sorted(EXPORTED_SYMBOLS) == names
    for n in names:
        assert getattr(lib, n) is not None


def test_size_queries_reject_bad_configs_and_scale():
    from paper_2503_18989_amd.binding import load_library, Config
    lib = load_library()
    good = Config(2, 256, 4, 64, 688, 1e-6, 1e4, 16, 10, 4, 64, 256, 0, 0)
    kv = lib.hat_mid_kv_bytes(ctypes.byref(good))
    assert kv == 2 * 10 * 4 * 2 * 16 * 64 * 2
    assert lib.hat_mid_workspace_bytes(ctypes.byref(good)) > 0
    for field, val in (("head_dim", 32), ("d_model", 250), ("page_size", 8), ("n_pages", 0), ("io_dtype", 7), ("kv_dtype", 2)):
        bad = Config(2, 256, 4, 64, 688, 1e-6, 1e4, 16, 10, 4, 64, 256, 0, 0)
        setattr(bad, field, val)
        assert lib.hat_mid_kv_bytes(ctypes.byref(bad)) == 0
        assert lib.hat_mid_workspace_bytes(ctypes.byref(bad)) == 0


def test_binding_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from paper_2503_18989_amd import HatMid
    import hat_inputs as hi
    with pytest.raises(RuntimeError):
        HatMid(hi.TINY, [], n_pages=4)


def test_headers_compile_as_plain_c99(tmp_path):
    """The boundary is a C ABI: both headers must be usable from a plain C99 translation unit, and the
    segment struct must have the layout the Python binding marshals (4 x int32 + 3 pointers)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    src = tmp_path / "abi.c"
    src.write_text('#include "hat_mid.h"\n#include "hat_sched.h"\n'
                   'int main(void) { return (sizeof(hat_mid_segment_t) == 40 && sizeof(hat_mid_config_t) == 56) ? 0 : 1; }\n')
    exe = tmp_path / "abi"
    b = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", str(exe)], capture_output=True, text=True)
    assert b.returncode == 0, b.stderr
    assert subprocess.run([str(exe)]).returncode == 0
    from paper_2503_18989_amd.binding import CSegment, Config
    import ctypes
    assert ctypes.sizeof(CSegment) == 40 and ctypes.sizeof(Config) == 56
