"""The C-ABI library loads, exports every symbol include/svgd.h declares, and rejects bad
arguments before touching a device.  No GPU needed (no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "svgd.h")
LIB = os.path.join(ROOT, "paper_2306_06528_amd", "libsvgd.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:svgd|swag)_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = declared_functions()
    for f in ("svgd_create", "svgd_bandwidth", "svgd_step", "svgd_destroy", "swag_update_moments"):
        assert f in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in svgd.h but not exported"


def test_status_strings(lib):
    lib.svgd_status_string.restype = ctypes.c_char_p
    want = {0: "SVGD_OK", -1: "SVGD_ERR_INVALID_ARG", -2: "SVGD_ERR_BAD_HANDLE",
            -3: "SVGD_ERR_TOO_LARGE", -4: "SVGD_ERR_ALLOC", -5: "SVGD_ERR_DEVICE"}
    for code, name in want.items():
        assert lib.svgd_status_string(code).decode() == name
    assert lib.svgd_status_string(-99).decode() == "SVGD_ERR_UNKNOWN"


def test_create_rejects_bad_arguments(lib):
    lib.svgd_create.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32]
    h = ctypes.c_void_p()
    assert lib.svgd_create(None, 4, 100, 0, 0) == -1
    assert lib.svgd_create(ctypes.byref(h), 0, 100, 0, 0) == -1
    assert lib.svgd_create(ctypes.byref(h), 4, 0, 0, 0) == -1
    assert lib.svgd_create(ctypes.byref(h), 4, 100, 0, 4) == -1      # unknown flag bit
    assert lib.svgd_create(ctypes.byref(h), 4, 100, -2, 0) == -1
    assert lib.svgd_create(ctypes.byref(h), 65, 100, 0, 0) == -3     # beyond SVGD_MAX_PARTICLES
    assert lib.svgd_create(ctypes.byref(h), 4, (1 << 36) + 1, 0, 0) == -3     # beyond SVGD_MAX_D
    assert not h.value


def test_null_and_stale_handles_are_rejected(lib):
    vp = ctypes.c_void_p
    lib.svgd_step.argtypes = [vp, vp, vp, ctypes.c_int, ctypes.c_int64, ctypes.c_float, vp]
    lib.svgd_phi.argtypes = [vp, vp, vp, ctypes.c_int, ctypes.c_int64, vp, vp]
    lib.svgd_bandwidth.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int64, vp, vp]
    lib.svgd_get_last.argtypes = [vp, vp, vp, vp]
    lib.svgd_destroy.argtypes = [vp]
    lib.svgd_set_bandwidth.argtypes = [vp, ctypes.c_double]
    lib.svgd_last_device_error.argtypes = [vp]
    bogus = ctypes.create_string_buffer(256)          # not a handle this library made
    for h in (None, ctypes.addressof(bogus)):
        assert lib.svgd_step(h, 16, 32, 1, 1, 0.1, None) == -2
        assert lib.svgd_phi(h, 16, 32, 1, 1, 48, None) == -2
        assert lib.svgd_bandwidth(h, 16, 1, 1, None, None) == -2
        assert lib.svgd_get_last(h, None, None, None) == -2
        assert lib.svgd_set_bandwidth(h, 1.0) == -2
        assert lib.svgd_destroy(h) == -2
        assert lib.svgd_last_device_error(h) == 0


def test_binding_has_the_same_names():
    import paper_2306_06528_amd.svgd as b
    for m in ("step", "bandwidth", "phi", "get_last", "set_bandwidth", "close"):
        assert hasattr(b.Svgd, m)


@pytest.mark.parametrize("compiler,std,suffix", [("gcc", "-std=c99", ".c"), ("g++", "-std=c++11", ".cpp")])
def test_header_is_plain_c_and_cpp(tmp_path, compiler, std, suffix):
    """The boundary is usable from C as well as C++: no torch or HIP types, nothing but <stdint.h>."""
    import shutil
    import subprocess
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not installed")
    src = tmp_path / ("use_header" + suffix)
    src.write_text('#include "svgd.h"\n'
                   "int main(void) { svgd_handle_t h = 0; (void)h; return SVGD_OK + SVGD_MAX_PARTICLES * 0; }\n")
    r = subprocess.run([compiler, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
