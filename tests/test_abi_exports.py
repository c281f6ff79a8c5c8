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


def test_share_group_member_struct_matches_the_header():
    """The ctypes image of comet_share_operands: field order, types and size as the header
    declares them (two int32, then six pointers), and the group limit."""
    from paper_2505_07239_amd import binding
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    body = re.search(r"typedef struct comet_share_operands \{(.*?)\} comet_share_operands;", text, flags=re.S).group(1)
    fields = [re.sub(r"\s+", " ", f.strip()) for f in body.split(";") if f.strip()]
    names = [f.split()[-1].lstrip("*") for f in fields]
    assert names == [n for n, _ in binding.ShareOperands._fields_]
    assert [("*" in f) for f in fields] == [False, False] + [True] * 6
    assert ctypes.sizeof(binding.ShareOperands) == 2 * 4 + 6 * ctypes.sizeof(ctypes.c_void_p)
    limit = int(re.search(r"COMET_SHARE_GROUP_MAX = (\d+)", text).group(1))
    assert limit == binding.SHARE_GROUP_MAX


def test_host_side_checks_of_the_group_call_need_no_gpu(lib):
    """Argument errors of comet_share_group are found before anything touches a device."""
    from paper_2505_07239_amd import binding
    lib.comet_share_group.restype = ctypes.c_int
    lib.comet_share_group.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.POINTER(binding.ShareOperands),
                                      ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t]
    arr = (binding.ShareOperands * 1)()
    # a null context is refused first
    assert lib.comet_share_group(None, 1, 1, arr, 8, 8, 8, 8, None, None, 1, 0, None, 0) != 0
