"""The C-ABI library loads and exports every entry point the header declares.
No compute call is made here (there is no GPU on the build host)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "comet_ring.h")
LIB = os.path.join(ROOT, "paper_2505_07239_amd", "libcomet_ring.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(comet_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2505_07239_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for must in ("comet_mask_share", "comet_mask_share_gather", "comet_open", "comet_compact_mask",
                 "comet_somm_share", "comet_simm_share", "comet_workspace_bytes", "comet_create"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), "missing export: " + name


def test_binding_lists_the_same_symbols():
    from paper_2505_07239_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()


def test_workspace_query_is_host_only(lib):
    lib.comet_workspace_bytes.restype = ctypes.c_size_t
    lib.comet_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_int]
    # SOMM, m = 256 (already a multiple of 128), k = 4096: 256 * 2 * 128 steps * 256 bytes of
    # digit planes, then the tile lists of the result-block form: a selector and twice
    # (count + 4 x 26 tiles of 64 x 64) int32, rounded up to 256 bytes, then the step lists of
    # the row-set form: per 32-row tile a count, an offset and up to 128 steps, plus one offset
    planes = 256 * 2 * 128 * 256
    lists = ((2 * (4 * 26 + 1) + 1) * 4 + 255) // 256 * 256
    steps = ((8 * (128 + 2) + 1) * 4 + 255) // 256 * 256
    assert lib.comet_workspace_bytes(1, 256, 4096, 1664, 32) == planes + lists + steps
    # small masks need no scratch, large ones do
    assert lib.comet_workspace_bytes(0, 1, 0, 344, 0) == 0
    assert lib.comet_workspace_bytes(0, 1, 0, 1 << 20, 0) > 0
    assert lib.comet_workspace_bytes(99, 1, 1, 1, 1) == 0


def test_version_string(lib):
    lib.comet_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.comet_version()


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_07239_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, "%s mentions the oracle" % f
