"""The C-ABI library builds, loads, and exports every symbol ``include/hylra.h`` declares.
No compute call is made here (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2602_00777_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_00777_amd import build

        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hylra.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hylra_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_agree(lib):
    names = declared_functions()
    assert len(names) >= 10
    assert set(names) == set(binding.EXPORTS)


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = set()
    for code in range(6):
        s = lib.hylra_status_str(code)
        assert s and s not in seen
        seen.add(s)
    assert lib.hylra_status_str(0) == b"ok"


def test_shape_struct_layout_matches_header():
    # int32 x5, padding to 8, int64 x3, float, padding to 8
    assert ctypes.sizeof(binding.Shape) == 56
    assert binding.Shape.kv_stride_b.offset == 24
    assert binding.Shape.scale.offset == 48


def test_null_arguments_are_rejected_without_touching_a_gpu(lib):
    assert lib.hylra_destroy(None) == 0
    assert lib.hylra_set_option(None, b"full_split_rows", 1) == 1
    assert lib.hylra_profile_reset(None) == 1
    assert lib.hylra_create(None, None, 1, 0) == 1
    h = ctypes.c_void_p()
    assert lib.hylra_create(ctypes.byref(h), None, 1, 0) == 1
    assert h.value is None
    assert b"NULL" in lib.hylra_last_error(None)
    bad = binding.Shape(1, 6, 4, 128, 64, 0, 0, 0, 0.0)      # 6 heads over 4 KV heads
    assert lib.hylra_create(ctypes.byref(h), ctypes.byref(bad), 1, 0) == 1
    bad = binding.Shape(1, 8, 2, 96, 64, 0, 0, 0, 0.0)       # head_dim 96
    assert lib.hylra_create(ctypes.byref(h), ctypes.byref(bad), 1, 0) == 2


@pytest.mark.parametrize("compiler,std,ext", [("gcc", "-std=c99", ".c"), ("g++", "-std=c++17", ".cpp")])
def test_header_is_plain_c_and_cxx(tmp_path, compiler, std, ext):
    """include/hylra.h must be usable from C and from C++ with nothing but the standard headers."""
    import shutil
    import subprocess
    if shutil.which(compiler) is None:
        pytest.skip(compiler + " is not installed")
    src = tmp_path / ("use_header" + ext)
    src.write_text('#include "hylra.h"\n'
                   "int main(void) { hylra_shape s; hylra_paged p; (void)s; (void)p; return (int)HYLRA_OK; }\n")
    inc = os.path.join(ROOT, "include")
    r = subprocess.run([compiler, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-c", str(src),
                        "-o", str(tmp_path / "use_header.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
