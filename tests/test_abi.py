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


def test_host_run_merge_matches_oracle_cover():
    """binding.vs_index_from_host merges slash tiles into offset runs on the
    host; compare with the oracle's offset-space cover (CPU tensors only)."""
    import torch
    from oracle import minference_oracle as O
    from paper_2407_02490_amd import binding as B
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    N = 2048
    rng = np.random.default_rng(3)
    S = np.sort(rng.choice(N, 40, replace=False))
    idx = B.vs_index_from_host([[1, 5]], [S.tolist()], N, device="cpu")
    n_c = int(idx.counts[0, 2])
    runs = idx.cover[0, :n_c].numpy()
    cover = O.slash_cover(S, N, 64)
    mine = np.zeros_like(cover)
    for t0, t1 in runs:
        mine[t0 + 64:t1 + 64] = True
    assert np.array_equal(mine, cover)
    bits = np.unpackbits(idx.cover_bits[0].numpy().view(np.uint8), bitorder="little")
    assert np.array_equal(bits[:N + 64].astype(bool), cover)
