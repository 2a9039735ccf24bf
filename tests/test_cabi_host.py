"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and validates arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2512_07710_amd as moe
from paper_2512_07710_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(moe.LIB_PATH):
        from paper_2512_07710_amd.build import build
        build()
    return moe.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "moe355.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_and_version(lib):
    assert lib.moe_strerror(0) == b"ok"
    assert b"invalid" in lib.moe_strerror(-1)
    assert b"id" in lib.moe_strerror(-3)
    assert b"gfx950" in lib.moe_version()


@pytest.mark.parametrize("dims", [
    (64, 100, 8, 2, 256),     # d not a multiple of 128
    (64, 128, 8, 2, 200),     # F not a multiple of 128
    (64, 128, 8, 9, 256),     # k > E
    (64, 128, 0, 1, 256),     # no experts
    (64, 128, 300, 2, 256),   # more experts than supported
    (-1, 128, 8, 2, 256),     # negative token count
    (64, 128, 32, 17, 256),   # k beyond the supported maximum
    (1 << 20, 2048, 8, 2, 256),        # T*d = 2^31: the router's 32-bit byte offsets into x would wrap
    (16, 1 << 16, 8, 2, 1 << 16),      # F*d = 2^32: byte offsets inside one expert's weight matrix would wrap
    ((1 << 27) + 1, 128, 16, 8, 128),  # T*k beyond 2^30
])
def test_create_rejects_bad_dims_without_a_device(lib, dims):
    d = binding._Dims(*dims)
    h = ctypes.c_void_p()
    assert lib.moe_create(ctypes.byref(h), ctypes.byref(d), None) == -1
    assert h.value is None


def test_null_arguments_are_rejected(lib):
    assert lib.moe_create(None, None, None) == -1
    assert lib.moe_destroy(None) == -1
    assert lib.moe_route(None, None, None, None, 2, None, None, None, None, None) == -1
    assert lib.moe_route_replay(None, None, None, None, None, None, None, None, None) == -1
    assert lib.moe_quantize_fp8(None, None, 4, 128, 128, None, 1, None, None) == -1
    assert lib.moe_route_replay_ids(None, None, None, None, None, None, None, None, None) == -1
    assert lib.moe_quantize_weights_fp8(None, None, 128, 128, None, None) == -1
    assert lib.moe_linear_fp8(None, None, None, 4, 128, None, None, 128, None) == -1
    assert lib.moe_expert_ffn_fp8_gather(*([None] * 12)) == -1
    assert lib.moe_expert_ffn_fp8(*([None] * 11)) == -1
    assert lib.moe_combine(*([None] * 6)) == -1
    assert lib.moe_debug_copy_hidden(None, None, None) == -1
    assert lib.moe_check_ids(None) == -1
    assert lib.moe_probe_copy(None, None, None, 1024) == -1
    assert lib.moe_probe_fp8_mfma(None, 1, 1, 0, None) == -1


def test_noalloc_replay_validates_before_touching_a_device(lib):
    n = [None] * 8
    assert lib.moe_route_replay_noalloc(None, 65537, 256, 16, *n) == -1     # T*k beyond the static scratch array
    assert lib.moe_route_replay_noalloc(None, 10, 300, 2, *n) == -1         # more experts than supported
    assert lib.moe_route_replay_noalloc(None, 10, 8, 9, *n) == -1           # k > E
    assert lib.moe_route_replay_noalloc(None, -1, 8, 2, *n) == -1
    assert lib.moe_route_replay_noalloc(None, 10, 8, 2, *n) == -1           # null arrays


def test_binding_fails_loudly_without_library(tmp_path):
    with pytest.raises(moe.MoEError):
        moe.load_library(str(tmp_path / "missing.so"))


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 with nothing but <stdint.h>, and every entry point it
    declares must be usable from C (a translation unit that takes each one's address)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    header = open(os.path.join(ROOT, "include", "moe355.h")).read()
    names = sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", re.sub(r"/\*.*?\*/", "", header, flags=re.S))))
    src = tmp_path / "use.c"
    src.write_text('#include "moe355.h"\ntypedef void (*fn)(void);\nfn table[] = {' + ", ".join(f"(fn){n}" for n in names) + "};\n")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
