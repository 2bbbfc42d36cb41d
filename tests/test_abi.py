"""The C-ABI library loads and exports every symbol include/minf.h declares;
host-side helpers of the binding (no GPU compute)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2407_02490_amd", "libminf.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "minf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(minf_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"minf_build_vs_index", "minf_build_bs_index", "minf_ashape_attn", "minf_vs_attn",
            "minf_bs_attn", "minf_dense_attn"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in minf.h but not exported"


def test_status_strings_and_cover_words(lib):
    lib.minf_status_string.restype = ctypes.c_char_p
    assert lib.minf_status_string(0) == b"ok"
    assert all(len(lib.minf_status_string(i)) > 0 for i in range(7))
    lib.minf_vs_cover_words.restype = ctypes.c_int32
    for N in (64, 4096, 131072, 1048576):
        assert lib.minf_vs_cover_words(N) * 32 >= N + 64 + 1


def test_null_arguments_are_rejected_on_the_host(lib):
    # validation happens before any HIP call, so this runs without a GPU
    assert lib.minf_ashape_attn(None, None, 0, 0, 1, None) == 1
    assert lib.minf_dense_attn(None, None, 0, None) == 1
    assert lib.minf_vs_attn(None, None, 0, None, None) == 1
    assert lib.minf_bs_attn(None, None, 0, None, None) == 1


def test_vs_index_from_lines_rejects_bad_arguments_on_the_host(lib):
    from paper_2407_02490_amd.binding import _VSIndex
    idx = _VSIndex()
    assert lib.minf_vs_index_from_lines(1024, 1, None, None) == 1
    assert lib.minf_vs_index_from_lines(1024, 1, ctypes.byref(idx), None) == 1          # NULL buffers
    for name in ("v_idx", "s_idx", "cover", "cover_bits", "counts"):
        setattr(idx, name, 256)                                                         # never dereferenced
    idx.nv, idx.ns, idx.block, idx.cover_words = 4, 4, 64, 64
    assert lib.minf_vs_index_from_lines(1000, 1, ctypes.byref(idx), None) == 2          # seq_len % 64
    assert lib.minf_vs_index_from_lines(1024, 0, ctypes.byref(idx), None) == 2          # no rows
    idx.cover_words = 3
    assert lib.minf_vs_index_from_lines(1024, 1, ctypes.byref(idx), None) == 2          # bitmap too small
    idx.cover_words, idx.block = 64, 32
    assert lib.minf_vs_index_from_lines(1024, 1, ctypes.byref(idx), None) == 5
    idx.block, idx.ns = 64, 0
    assert lib.minf_vs_index_from_lines(1024, 1, ctypes.byref(idx), None) == 3
