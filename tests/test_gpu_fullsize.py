"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times: the 128K single-pattern layers (c1, c2, c3) and the mixed 1M layer (c4).

The oracle cannot do a whole layer in fp64 in reasonable time, so outputs are
checked on sampled 64-row query blocks (rows are independent given the
indices): block 0, the last block, the blocks that straddle the A-shape sink
and window edges, the first block with a full Block-Sparse budget, plus at least twelve
seeded random blocks per sampled head; three heads per pattern from different
K/V groups.  Index sets are checked in full for the sampled heads (at 1M
tokens every Block-Sparse index row of one head, sampled rows of the others).
Next to the absolute bar every block must be close in relative L2 norm
(tests/helpers.py), which a dropped tile or a dropped gathered step fails.
"""
import numpy as np
import pytest
import torch

from oracle import minference_oracle as O
from paper_2407_02490_amd import workloads as W
from tests.helpers import assert_close_rows, check_topk, observed_errors

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2407_02490_amd import binding
    binding.lib()
    return binding


def sample_blocks(NB, extra, n_random, seed):
    rng = np.random.default_rng(seed)
    s = {0, NB - 1, *[b for b in extra if 0 <= b < NB]}
    s.update(int(b) for b in rng.integers(0, NB, size=n_random))
    return sorted(s)


def test_c1_ashape_128k(B):
    x = W.make_config("c1", device="cuda")
    c = x.meta
    o = torch.empty_like(x.q)
    B.minf_ashape_attn(x.q, x.k, x.v, o, list(range(x.n_q_heads)), c["n_init"], c["n_local"])
    torch.cuda.synchronize()
    NB = x.seq_len // 64
    blocks = sample_blocks(NB, [15, 16, 17, 63, 64, 65, 79, 80, 81], 12, 1)
    for h in (0, 13, 31):
        Qh, Kh, Vh = x.head_f64(h)
        for b in blocks:
            want = O.ashape_attention(Qh, Kh, Vh, c["n_init"], c["n_local"], 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"c1 head {h} block {b}")


def test_c2_vertical_slash_128k(B):
    x = W.make_config("c2", device="cuda")
    c, N = x.meta, x.seq_len
    heads = list(range(x.n_q_heads))
    idx = B.alloc_vs_index(len(heads), c["nv"], c["ns"], N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(x.q, x.k, len(heads), c["last_q"]), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(x.q)
    B.minf_build_vs_index(x.q, x.k, heads, c["last_q"], c["nv"], c["ns"], idx, ws)
    B.minf_vs_attn(x.q, x.k, x.v, o, heads, idx)
    torch.cuda.synchronize()
    NB = N // 64
    swaps = 0
    for n, h in enumerate((0, 17, 30)):                         # three K/V groups
        blocks = sample_blocks(NB, [1, 2, 100, NB - 2], 12, 20 + n)
        Qh, Kh, Vh = x.head_f64(h)
        Vo, So, col, diag = O.vs_index(Qh, Kh, c["last_q"], c["nv"], c["ns"])
        Vg = idx.v_idx[h].cpu().numpy()
        Sg = idx.s_idx[h].cpu().numpy()
        swaps += check_topk(Vg, col, c["nv"], max_swaps=4) + check_topk(Sg, diag, c["ns"], max_swaps=4)
        assert np.isin(x.sinks[h // 4].numpy(), Vg).mean() >= 0.9      # planted sinks are found
        for b in blocks:
            want = O.vs_attention(Qh, Kh, Vh, Vg, Sg, 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"c2 head {h} block {b}")
    print("c2 tolerated index swaps:", swaps, "observed errors:", observed_errors())


def bs_row_check(idx_row, cnt, Qp, Kp, b, topk, tau):
    row = (Qp[b] @ Kp[:b + 1].T) * tau          # Alg. 3: block logits of query block b
    assert cnt == min(topk, b + 1)
    return check_topk(idx_row[:cnt], row, topk, relative=False)


def test_c3_block_sparse_128k(B):
    x = W.make_config("c3", device="cuda")
    c, N = x.meta, x.seq_len
    heads = list(range(x.n_q_heads))
    idx = B.alloc_bs_index(len(heads), N, c["topk"])
    ws = torch.empty(B.minf_bs_index_workspace_bytes(x.q, x.k, len(heads), c["topk"]), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(x.q)
    B.minf_build_bs_index(x.q, x.k, heads, c["topk"], idx, ws)
    B.minf_bs_attn(x.q, x.k, x.v, o, heads, idx)
    torch.cuda.synchronize()
    NB = N // 64
    for n, h in enumerate((0, 13, 21)):                         # three K/V groups
        blocks = sample_blocks(NB, [98, 99, 100, 101], 12, 30 + n)
        Qh, Kh, Vh = x.head_f64(h)
        io, co, s = O.bs_index(Qh, Kh, 64, c["topk"])
        got = idx.blk_idx[h].cpu().numpy()
        cnt = idx.blk_cnt[h].cpu().numpy()
        assert np.array_equal(cnt, co)
        # every row of the index
        swaps = sum(check_topk(got[b, :cnt[b]], s[b, :b + 1], c["topk"], relative=False, max_swaps=2) for b in range(NB))
        assert swaps <= 8
        print(f"c3 head {h} tolerated index swaps:", swaps)
        for b in blocks:
            want = O.bs_attention(Qh, Kh, Vh, got, cnt, 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"c3 head {h} block {b}")
    print("c3 observed errors:", observed_errors())


def test_c4_mixed_1m(B):
    x = W.make_config("c4", device="cuda")
    c, N = x.meta, x.seq_len
    vs_h, bs_h, a_h = W.head_assignment(x.n_q_heads, c["n_vs"], c["n_bs"], c["n_ashape"])
    vsi = B.alloc_vs_index(len(vs_h), c["nv"], c["ns"], N)
    vws = torch.empty(B.minf_vs_index_workspace_bytes(x.q, x.k, len(vs_h), c["last_q"]), dtype=torch.uint8, device="cuda")
    bsi = B.alloc_bs_index(len(bs_h), N, c["topk"])
    bws = torch.empty(B.minf_bs_index_workspace_bytes(x.q, x.k, len(bs_h), c["topk"]), dtype=torch.uint8, device="cuda")
    o = torch.full_like(x.q, float("nan"))
    B.minf_build_vs_index(x.q, x.k, vs_h, c["last_q"], c["nv"], c["ns"], vsi, vws)
    B.minf_build_bs_index(x.q, x.k, bs_h, c["topk"], bsi, bws)
    B.minf_ashape_attn(x.q, x.k, x.v, o, a_h, c["n_init"], c["n_local"])
    B.minf_vs_attn(x.q, x.k, x.v, o, vs_h, vsi)
    B.minf_bs_attn(x.q, x.k, x.v, o, bs_h, bsi)
    torch.cuda.synchronize()
    assert not torch.isnan(o[:, -1].float()).any()            # every head was written by some call
    NB = N // 64
    tau = 1.0 / np.sqrt(128.0)
    g = x.n_q_heads // x.n_kv_heads

    def pick(heads, n):
        """n positions of a head list whose heads read different K/V heads (as far as there are)."""
        out, seen = [], set()
        for r, h in enumerate(heads):
            if h // g not in seen:
                seen.add(h // g)
                out.append(r)
        out += [r for r in range(len(heads)) if r not in out]
        return out[:n]

    # Vertical-Slash: three heads of different K/V groups; edge blocks + 12 random ones each
    swaps = 0
    for n, r in enumerate(pick(vs_h, 3)):
        h = vs_h[r]
        Qh, Kh, Vh = x.head_f64(h)
        Vo, So, col, diag = O.vs_index(Qh, Kh, c["last_q"], c["nv"], c["ns"])
        Vg, Sg = vsi.v_idx[r].cpu().numpy(), vsi.s_idx[r].cpu().numpy()
        swaps += check_topk(Vg, col, c["nv"], max_swaps=4) + check_topk(Sg, diag, c["ns"], max_swaps=4)
        for b in sample_blocks(NB, [1, 3, NB - 2], 12, 40 + n):
            want = O.vs_attention(Qh, Kh, Vh, Vg, Sg, 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"c4 VS head {h} block {b}")
        del Qh, Kh, Vh
    print("c4 VS tolerated index swaps:", swaps)
    # Block-Sparse: three heads; every row of the index for the first of them
    for n, r in enumerate(pick(bs_h, 3)):
        h = bs_h[r]
        Qh, Kh, Vh = x.head_f64(h)
        Qp, Kp = O.bs_pool(Qh), O.bs_pool(Kh)
        got, cnt = bsi.blk_idx[r].cpu().numpy(), bsi.blk_cnt[r].cpu().numpy()
        assert np.array_equal(cnt, np.minimum(c["topk"], np.arange(1, NB + 1)))
        blocks = sample_blocks(NB, [98, 99, 100, 101], 12, 50 + n)
        rows = range(NB) if n == 0 else blocks
        bs_swaps = 0
        for b0 in range(0, NB, 2048):                          # block logits of 2048 rows at a time
            sc = (Qp[b0:b0 + 2048] @ Kp.T) * tau               # Alg. 3: block logits
            for b in rows:
                if b0 <= b < b0 + 2048:
                    assert cnt[b] == min(c["topk"], b + 1)
                    bs_swaps += check_topk(got[b, :cnt[b]], sc[b - b0, :b + 1], c["topk"], relative=False, max_swaps=2)
        print(f"c4 BS head {h}: {len(rows)} index rows checked, tolerated swaps {bs_swaps}")
        assert bs_swaps <= 16
        for b in blocks:
            want = O.bs_attention(Qh, Kh, Vh, got, cnt, 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"c4 BS head {h} block {b}")
        del Qh, Kh, Vh
    # A-shape: both heads
    for n, h in enumerate(a_h):
        Qh, Kh, Vh = x.head_f64(h)
        for b in sample_blocks(NB, [15, 16, 17, 63, 64, 65, 79, 80, 81], 12, 60 + n):
            want = O.ashape_attention(Qh, Kh, Vh, c["n_init"], c["n_local"], 64 * b, 64 * b + 64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"c4 A-shape head {h} block {b}")
        del Qh, Kh, Vh
    print("c4 observed errors:", observed_errors())


def test_ragged_medium_length_mixed(B):
    """A length that is a multiple of 64 and of nothing larger (1025 blocks): the last
    1024-key chunk of the score kernels holds one tile, rows of block logits are not 16-byte
    aligned (general selection path), the last shared-tile workgroup has three idle waves."""
    N = 64 * 1025
    x = W.make_config("c4", device="cuda", N=N, n_q_heads=8, n_kv_heads=2)
    heads_vs, heads_bs, heads_a = [0, 1, 5], [2, 6, 7], [3, 4]
    nv, ns, topk = 300, 2000, 40
    vsi = B.alloc_vs_index(len(heads_vs), nv, ns, N)
    vws = torch.empty(B.minf_vs_index_workspace_bytes(x.q, x.k, len(heads_vs), 64), dtype=torch.uint8, device="cuda")
    bsi = B.alloc_bs_index(len(heads_bs), N, topk)
    bws = torch.empty(B.minf_bs_index_workspace_bytes(x.q, x.k, len(heads_bs), topk), dtype=torch.uint8, device="cuda")
    o = torch.full_like(x.q, float("nan"))
    B.minf_build_vs_index(x.q, x.k, heads_vs, 64, nv, ns, vsi, vws)
    B.minf_build_bs_index(x.q, x.k, heads_bs, topk, bsi, bws)
    B.minf_ashape_attn(x.q, x.k, x.v, o, heads_a, 1024, 4096)
    B.minf_vs_attn(x.q, x.k, x.v, o, heads_vs, vsi)
    B.minf_bs_attn(x.q, x.k, x.v, o, heads_bs, bsi)
    torch.cuda.synchronize()
    assert not torch.isnan(o.float()).any()
    NB = N // 64
    blocks = sample_blocks(NB, [15, 16, 17, 63, 64, 65, 80, 81, NB - 2], 4, 5)
    r, h = 1, heads_vs[1]
    Qh, Kh, Vh = x.head_f64(h)
    Vo, So, col, diag = O.vs_index(Qh, Kh, 64, nv, ns)
    Vg, Sg = vsi.v_idx[r].cpu().numpy(), vsi.s_idx[r].cpu().numpy()
    check_topk(Vg, col, nv)
    check_topk(Sg, diag, ns)
    for b in blocks:
        assert_close_rows(o[h, 64 * b:64 * b + 64], O.vs_attention(Qh, Kh, Vh, Vg, Sg, 64 * b, 64 * b + 64), f"ragged VS block {b}")
    r, h = 2, heads_bs[2]
    Qh, Kh, Vh = x.head_f64(h)
    io, co, s = O.bs_index(Qh, Kh, 64, topk)
    got, cnt = bsi.blk_idx[r].cpu().numpy(), bsi.blk_cnt[r].cpu().numpy()
    assert np.array_equal(cnt, co)
    for b in range(NB):
        check_topk(got[b, :cnt[b]], s[b, :b + 1], topk, relative=False)
    assert np.array_equal(bsi.order[r].cpu().numpy(), np.lexsort((np.arange(NB), got[:, 0])))
    for b in blocks:
        assert_close_rows(o[h, 64 * b:64 * b + 64], O.bs_attention(Qh, Kh, Vh, got, cnt, 64 * b, 64 * b + 64), f"ragged BS block {b}")
    h = heads_a[0]
    Qh, Kh, Vh = x.head_f64(h)
    for b in blocks:
        assert_close_rows(o[h, 64 * b:64 * b + 64], O.ashape_attention(Qh, Kh, Vh, 1024, 4096, 64 * b, 64 * b + 64), f"ragged A-shape block {b}")


def test_two_million_tokens_one_head(B):
    """Beyond the benchmark sizes: 2M tokens (32768 blocks), one head per pattern on one K/V
    head.  Rows of block logits are longer than the selection kernel holds in registers, the
    sort of the processing order fills 128 KiB of LDS, row offsets pass 2^29 bytes."""
    N = 1 << 21
    x = W.make_config("c4", device="cuda", N=N, n_q_heads=3, n_kv_heads=1)
    NB = N // 64
    nv, ns, topk = 1000, 6096, 100
    vsi = B.alloc_vs_index(1, nv, ns, N)
    vws = torch.empty(B.minf_vs_index_workspace_bytes(x.q, x.k, 1, 64), dtype=torch.uint8, device="cuda")
    bsi = B.alloc_bs_index(1, N, topk)
    bws = torch.empty(B.minf_bs_index_workspace_bytes(x.q, x.k, 1, topk), dtype=torch.uint8, device="cuda")
    o = torch.full_like(x.q, float("nan"))
    B.minf_build_vs_index(x.q, x.k, [0], 64, nv, ns, vsi, vws)
    B.minf_build_bs_index(x.q, x.k, [1], topk, bsi, bws)
    B.minf_vs_attn(x.q, x.k, x.v, o, [0], vsi)
    B.minf_bs_attn(x.q, x.k, x.v, o, [1], bsi)
    B.minf_ashape_attn(x.q, x.k, x.v, o, [2], 1024, 4096)
    torch.cuda.synchronize()
    del vws, bws
    torch.cuda.empty_cache()
    assert not torch.isnan(o[:, -1].float()).any()
    tau = 1.0 / np.sqrt(128.0)
    blocks = sample_blocks(NB, [16383, 16384, 16385], 2, 8)
    Qh, Kh, Vh = x.head_f64(0)
    Vo, So, col, diag = O.vs_index(Qh, Kh, 64, nv, ns)
    Vg, Sg = vsi.v_idx[0].cpu().numpy(), vsi.s_idx[0].cpu().numpy()
    print("2M VS tolerated index swaps:", check_topk(Vg, col, nv, max_swaps=4) + check_topk(Sg, diag, ns, max_swaps=4))
    for b in blocks:
        want = O.vs_attention(Qh, Kh, Vh, Vg, Sg, 64 * b, 64 * b + 64)
        assert_close_rows(o[0, 64 * b:64 * b + 64], want, f"2M VS block {b}")
    Qh, Kh, Vh = x.head_f64(1)
    Qp, Kp = O.bs_pool(Qh), O.bs_pool(Kh)
    got, cnt = bsi.blk_idx[0].cpu().numpy(), bsi.blk_cnt[0].cpu().numpy()
    assert np.array_equal(cnt, np.minimum(topk, np.arange(1, NB + 1)))
    assert np.array_equal(bsi.order[0].cpu().numpy(), np.lexsort((np.arange(NB), got[:, 0])))
    for b in blocks + [99, 100, 16500, 30000]:
        bs_row_check(got[b], cnt[b], Qp, Kp, b, topk, tau)
    for b in blocks:
        want = O.bs_attention(Qh, Kh, Vh, got, cnt, 64 * b, 64 * b + 64)
        assert_close_rows(o[1, 64 * b:64 * b + 64], want, f"2M BS block {b}")
    Qh, Kh, Vh = x.head_f64(2)
    for b in blocks:
        want = O.ashape_attention(Qh, Kh, Vh, 1024, 4096, 64 * b, 64 * b + 64)
        assert_close_rows(o[2, 64 * b:64 * b + 64], want, f"2M A-shape block {b}")
