"""Vertical-Slash budgets beyond the default: the head-pattern search space
(App. C.2, search-space table) and the "only vertical" / "only slash"
ablation limits (App. D.3), on a reduced layer of the 128K recipe.

For every setting the index is built on the GPU and compared with the
oracle's exact top-k (tie rule of the benchmark contract); attention runs
from the GPU's own index and is compared with the oracle on sampled 64-row
query blocks; the tile count derived from the GPU index equals the oracle's.
The settings span the column-dominated and the slash-dominated extremes of
the sparse kernel (3000 columns in three LDS rounds; 2048 slashes and one
column).
"""
import numpy as np
import pytest
import torch

from oracle import minference_oracle as O
from paper_2407_02490_amd import costmodel as C
from paper_2407_02490_amd import workloads as W
from tests.helpers import assert_close_rows, check_topk

pytestmark = pytest.mark.gpu

N = 8192


@pytest.fixture(scope="module")
def B():
    from paper_2407_02490_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def layer():
    return W.make_config("c2", device="cuda", N=N, n_q_heads=2, n_kv_heads=1)


@pytest.mark.parametrize("label,nv,ns", W.VS_BUDGET_SWEEP)
def test_budget_setting_matches_oracle(B, layer, label, nv, ns):
    x = layer
    heads = [0, 1]
    idx = B.alloc_vs_index(len(heads), nv, ns, N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(x.q, x.k, len(heads), 64), dtype=torch.uint8, device="cuda")
    o = torch.full_like(x.q, float("nan"))
    B.minf_build_vs_index(x.q, x.k, heads, 64, nv, ns, idx, ws)
    B.minf_vs_attn(x.q, x.k, x.v, o, heads, idx)
    torch.cuda.synchronize()
    tiles_gpu = C.vs_index_tiles(idx, N)
    NB = N // 64
    blocks = sorted({0, 1, 2, NB // 2, NB - 2, NB - 1, *np.random.default_rng(nv + ns).integers(0, NB, 6).tolist()})
    for r, h in enumerate(heads):
        Qh, Kh, Vh = x.head_f64(h)
        _, _, col, diag = O.vs_index(Qh, Kh, 64, nv, ns)
        counts = idx.counts[r].cpu().numpy()
        assert counts[0] == min(nv, N) and counts[1] == min(ns, N)
        Vg = idx.v_idx[r, :counts[0]].cpu().numpy()
        Sg = idx.s_idx[r, :counts[1]].cpu().numpy()
        check_topk(Vg, col, nv)
        check_topk(Sg, diag, ns)
        assert np.array_equal(tiles_gpu[r], O.tiles_vs(N, Vg, Sg)), f"{label}: tile count of head {h}"
        for b in blocks:
            want = O.vs_attention(Qh, Kh, Vh, Vg, Sg, 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"{label} head {h} block {b}")
