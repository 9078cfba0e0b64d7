"""The C-ABI library loads and exports every function include/px.h declares (no GPU calls)."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "px.h")
LIBRARY = os.path.join(ROOT, "paper_1808_02621_amd", "libpx.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(px_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def library():
    if not os.path.exists(LIBRARY):
        from paper_1808_02621_amd import build
        build.build_library()
    return ctypes.CDLL(LIBRARY)


def test_header_declares_the_hot_path_calls():
    names = declared_functions()
    for required in ("px_sparse_coalesce", "px_partition_rows", "px_sparse_apply_sgd",
                     "px_sparse_apply_adagrad", "px_dense_average"):
        assert required in names


def test_every_declared_function_is_exported(library):
    for name in declared_functions():
        assert hasattr(library, name), "%s declared in px.h but not exported" % name


def test_binding_lists_the_same_functions(library):
    from paper_1808_02621_amd import px
    assert sorted(px.EXPORTS) == declared_functions()


def test_host_only_calls(library):
    library.px_status_string.restype = ctypes.c_char_p
    assert library.px_status_string(0) == b"ok"
    assert b"scratch" in library.px_status_string(3)
    library.px_coalesce_scratch_bytes.restype = ctypes.c_size_t
    library.px_coalesce_scratch_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    small = library.px_coalesce_scratch_bytes(1024, 64)
    large = library.px_coalesce_scratch_bytes(1 << 20, 128)
    assert 0 < small < large
    assert library.px_coalesce_scratch_bytes(0, 64) > 0
    # sort buffers (16 B/row) plus partial rows: well under the size of the input itself
    assert large < (1 << 20) * 128 * 4
    library.px_partition_scratch_bytes.restype = ctypes.c_size_t
    library.px_partition_scratch_bytes.argtypes = [ctypes.c_int64]
    assert library.px_partition_scratch_bytes(1000) > 0


def test_dense_launch_count_is_host_arithmetic(library):
    """2^19 16-byte pieces per launch, more for few buffers, at most 16 MiB of output."""
    f = library.px_dense_average_launches
    f.restype = ctypes.c_int64
    f.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
    F32, BF16 = 0, 1
    assert f(48, 1 << 26, BF16, F32) == 16          # the headline workload: 2^23 pieces
    assert f(48, 1 << 23, F32, F32) == 4            # 2^21 pieces
    assert f(8, 1 << 22, F32, F32) == 1             # few buffers: one launch of 16 MiB of output
    assert f(2, 6_300_003, F32, F32) == 2 and f(2, 6_300_003, BF16, F32) == 2
    assert f(4, 65_536, F32, F32) == 1
    assert f(4, 3, F32, F32) == 0 and f(0, 100, F32, F32) == 0 and f(4, 0, F32, F32) == 0
