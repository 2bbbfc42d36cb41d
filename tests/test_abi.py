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
    assert lib.minf_vs_bs_attn(None, None, 0, None, None, 0, None, None) == 1


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


def _qkv(N, n_q=32, n_kv=8):
    from paper_2407_02490_amd.binding import _QKV
    x = _QKV()
    x.q = x.k = x.v = x.o = 4096                                                        # never dereferenced
    for name, h in (("q_stride", n_q), ("k_stride", n_kv), ("v_stride", n_kv), ("o_stride", n_q)):
        st = getattr(x, name)
        st[0], st[1], st[2] = h * N * 128, N * 128, 128
    x.batch, x.n_q_heads, x.n_kv_heads, x.seq_len, x.head_dim, x.softmax_scale = 1, n_q, n_kv, N, 128, 0.0
    return x


def test_workspace_sizes(lib):
    """Host arithmetic only.  Up to a budget of 112 blocks the Block-Sparse build stores neither block logits
    nor the pooled Q (Alg. 3's pooling of Q and its top-k are then fused with the logits): the pooled K alone,
    512 bytes per head and block."""
    lib.minf_bs_index_workspace_bytes.restype = ctypes.c_size_t
    lib.minf_vs_index_workspace_bytes.restype = ctypes.c_size_t
    x = _qkv(1 << 20)
    NB = (1 << 20) // 64
    fused = lib.minf_bs_index_workspace_bytes(ctypes.byref(x), 6, 100)
    assert fused == 6 * NB * 512
    assert lib.minf_bs_index_workspace_bytes(ctypes.byref(x), 6, 112) == fused
    staged = lib.minf_bs_index_workspace_bytes(ctypes.byref(x), 6, 113)
    assert staged >= 2 * fused + 2 * NB * NB * 4                                        # pooled Q too, and at least two heads' logits
    assert lib.minf_bs_index_workspace_bytes(ctypes.byref(x), 6, 0) == 0
    assert lib.minf_bs_index_workspace_bytes(ctypes.byref(x), 0, 100) == 0
    # ragged number of blocks: pooled K is padded to whole 32-row tiles
    y = _qkv(64 * 33)
    assert lib.minf_bs_index_workspace_bytes(ctypes.byref(y), 1, 8) == 64 * 512
    # Vertical-Slash: grows with heads x tokens, within 16 .. 24 bytes per head and token
    per = lib.minf_vs_index_workspace_bytes(ctypes.byref(x), 24, 64) / (24 * (1 << 20))
    assert 16 <= per <= 24
