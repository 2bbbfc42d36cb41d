"""Parity of the HIP index builders with the CPU oracle, through the C ABI.

Index sets must equal the oracle's exact top-k except for swaps among scores
that tie within 1e-3 of the k-th score (tests/helpers.check_topk); the merged
slash runs and the run bitmap are integer work and must be exact functions of
the kept offsets.
"""
import numpy as np
import pytest
import torch

from oracle import minference_oracle as O
from paper_2407_02490_amd import workloads as W
from tests.helpers import assert_close_rows, check_topk, random_qkv, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2407_02490_amd import binding
    binding.lib()
    return binding


def build_vs(B, q, k, heads, last_q, nv, ns):
    N = q.shape[-2]
    idx = B.alloc_vs_index(len(heads), nv, ns, N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, len(heads), last_q), dtype=torch.uint8, device="cuda")
    B.minf_build_vs_index(q, k, heads, last_q, nv, ns, idx, ws)
    torch.cuda.synchronize()
    return idx


def check_vs_index(idx, r, N, Qh, Kh, last_q, nv, ns):
    Vo, So, col, diag = O.vs_index(Qh, Kh, last_q, nv, ns)
    n_v, n_s, n_c, _ = idx.counts[r].cpu().tolist()
    assert n_v == min(nv, N) and n_s == min(ns, N)
    Vg = idx.v_idx[r, :n_v].cpu().numpy()
    Sg = idx.s_idx[r, :n_s].cpu().numpy()
    swaps = check_topk(Vg, col, nv) + check_topk(Sg, diag, ns)
    # runs and bitmap: exact functions of the kept offsets (compared with the
    # oracle's cover of the GPU's own offsets)
    cover = O.slash_cover(Sg, N, 64)                       # index t + 64, t in [-64, N)
    runs = idx.cover[r, :n_c].cpu().numpy()
    c8 = cover.astype(np.int8)
    edges = np.diff(np.concatenate([[0], c8, [0]]))
    t0 = np.flatnonzero(edges == 1) - 64
    t1 = np.flatnonzero(edges == -1) - 64
    assert n_c == t0.size
    assert np.array_equal(runs[:, 0], t0) and np.array_equal(runs[:, 1], t1)
    bits = idx.cover_bits[r].cpu().numpy().view(np.uint32)
    flat = np.unpackbits(bits.view(np.uint8), bitorder="little")
    assert np.array_equal(flat[:N + 64].astype(bool), cover)
    assert not flat[N + 64:].any()
    return Vg, Sg, swaps


@pytest.mark.parametrize("N,last_q,nv,ns", [(1024, 64, 30, 50), (4096, 64, 256, 512), (2112, 17, 100, 3000),
                                             (64, 64, 5, 5), (1088, 1, 7, 9)])
def test_vs_index_random_inputs(B, N, last_q, nv, ns):
    q, k, v = random_qkv(11, 4, 2, N)
    heads = [2, 0, 3]
    idx = build_vs(B, q, k, heads, last_q, nv, ns)
    for r, h in enumerate(heads):
        check_vs_index(idx, r, N, to_f64(q[h]), to_f64(k[h // 2]), last_q, nv, ns)


@pytest.mark.parametrize("N,n_s", [(2048, 40), (4096, 1), (131072, 3000), (1024, 1024)])
def test_vs_index_from_lines_matches_oracle_cover(B, rng, N, n_s):
    """Runs, bitmap and counts built on the device from caller-supplied lines (the static-index
    use) equal the oracle's offset-space cover of the same slashes, bit for bit."""
    lists = [np.sort(rng.choice(N, n_s, replace=False)), np.sort(rng.choice(N, max(1, n_s // 2), replace=False))]
    if n_s >= 40:
        lists[1][:20] = np.arange(20)                       # a contiguous stretch: one wide run
        lists[1] = np.unique(lists[1])
    Vl = [[1, 5], list(range(0, N, 97))]
    idx = B.vs_index_from_host(Vl, [l.tolist() for l in lists], N)
    torch.cuda.synchronize()
    for r, S in enumerate(lists):
        n_v, n_sg, n_c, zero = idx.counts[r].cpu().tolist()
        assert (n_v, n_sg, zero) == (len(Vl[r]), S.size, 0)
        assert np.array_equal(idx.s_idx[r, :S.size].cpu().numpy(), S)
        cover = O.slash_cover(S, N, 64)
        edges = np.diff(np.concatenate([[0], cover.astype(np.int8), [0]]))
        t0, t1 = np.flatnonzero(edges == 1) - 64, np.flatnonzero(edges == -1) - 64
        runs = idx.cover[r, :n_c].cpu().numpy()
        assert n_c == t0.size and np.array_equal(runs[:, 0], t0) and np.array_equal(runs[:, 1], t1)
        flat = np.unpackbits(idx.cover_bits[r].cpu().numpy().view(np.uint8), bitorder="little")
        assert np.array_equal(flat[:N + 64].astype(bool), cover) and not flat[N + 64:].any()


def test_vs_index_from_lines_clamps_offsets_outside_the_sequence(B):
    N = 1024
    idx = B.vs_index_from_host([[0]], [[5, 700, N + 4000]], N)       # the last offset is not a valid line
    torch.cuda.synchronize()
    n_c = int(idx.counts[0, 2])
    runs = idx.cover[0, :n_c].cpu().numpy()
    assert runs.min() >= -63 and runs.max() <= N
    flat = np.unpackbits(idx.cover_bits[0].cpu().numpy().view(np.uint8), bitorder="little")
    assert np.array_equal(flat[:N + 64].astype(bool), O.slash_cover(np.array([5, 700, N - 1]), N, 64))


def test_vs_attn_refuses_rows_too_far_apart_for_the_gather(B):
    """seq_len * row pitch >= 2^32 bytes: refused with a shape status before any launch."""
    N = 128
    q, k, v = random_qkv(15, 1, 1, N)
    big = torch.empty(1 << 31, dtype=torch.bfloat16, device="cuda")   # 4 GiB, never read
    kk = torch.as_strided(big, (1, N, 128), (0, 1 << 24, 1))          # the largest row pitch accepted: 32 MiB
    idx = B.vs_index_from_host([[0]], [[0]], N)
    o = torch.zeros_like(q)
    with pytest.raises(B.MinfError) as e:
        B.minf_vs_attn(q, kk, v, o, [0], idx)
    assert e.value.status == 2
    torch.cuda.synchronize()
    assert (o == 0).all()


def test_last_q_17_index_then_attention(B):
    """Fewer estimating rows than a block (last_q = 17), then attention with that index."""
    N, nv, ns = 2112, 60, 150
    q, k, v = random_qkv(13, 2, 1, N)
    idx = build_vs(B, q, k, [1, 0], 17, nv, ns)
    o = torch.full_like(q, float("nan"))
    B.minf_vs_attn(q, k, v, o, [1, 0], idx)
    torch.cuda.synchronize()
    for r, h in enumerate([1, 0]):
        Qh, Kh, Vh = to_f64(q[h]), to_f64(k[0]), to_f64(v[0])
        Vg, Sg, swaps = check_vs_index(idx, r, N, Qh, Kh, 17, nv, ns)
        assert swaps == 0
        assert_close_rows(o[h], O.vs_attention(Qh, Kh, Vh, Vg, Sg, Bm=64), f"last_q=17 head {h}")


def test_scale_other_than_default_through_both_builders(B):
    """softmax_scale != 1/sqrt(d) through minf_build_vs_index / minf_build_bs_index and on into
    attention: the estimate's softmax sharpens with the scale, so the kept lines change."""
    N, scale = 2048, 0.2
    q, k, v = random_qkv(14, 2, 1, N)
    heads = [0, 1]
    idx = B.alloc_vs_index(2, 40, 90, N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, 2, 64), dtype=torch.uint8, device="cuda")
    B.minf_build_vs_index(q, k, heads, 64, 40, 90, idx, ws, scale=scale)
    bidx = B.alloc_bs_index(2, N, 6)
    ws2 = torch.empty(B.minf_bs_index_workspace_bytes(q, k, 2), dtype=torch.uint8, device="cuda")
    B.minf_build_bs_index(q, k, heads, 6, bidx, ws2, scale=scale)
    o = torch.full_like(q, float("nan"))
    ob = torch.full_like(q, float("nan"))
    B.minf_vs_attn(q, k, v, o, heads, idx, scale=scale)
    B.minf_bs_attn(q, k, v, ob, heads, bidx, scale=scale)
    torch.cuda.synchronize()
    changed = 0
    for r, h in enumerate(heads):
        Qh, Kh, Vh = to_f64(q[h]), to_f64(k[0]), to_f64(v[0])
        Vo, So, col, diag = O.vs_index(Qh, Kh, 64, 40, 90, scale=scale)
        Vg, Sg = idx.v_idx[r].cpu().numpy(), idx.s_idx[r].cpu().numpy()
        assert check_topk(Vg, col, 40) + check_topk(Sg, diag, 90) == 0
        Vd, Sd, _, _ = O.vs_index(Qh, Kh, 64, 40, 90)
        changed += int(not np.array_equal(Vd, Vo)) + int(not np.array_equal(Sd, So))
        assert_close_rows(o[h], O.vs_attention(Qh, Kh, Vh, Vg, Sg, Bm=64, scale=scale), f"vs scale head {h}")
        io, co, s = O.bs_index(Qh, Kh, 64, 6, scale=scale)
        got, cnt = bidx.blk_idx[r].cpu().numpy(), bidx.blk_cnt[r].cpu().numpy()
        assert np.array_equal(cnt, co)
        for b in range(N // 64):
            assert check_topk(got[b, :cnt[b]], s[b, :b + 1], 6, relative=False) == 0
        assert_close_rows(ob[h], O.bs_attention(Qh, Kh, Vh, got, cnt, scale=scale), f"bs scale head {h}")
    assert changed > 0          # the case can tell the scales apart


def test_vs_index_is_bit_reproducible(B):
    q, k, v = random_qkv(12, 2, 1, 2048)
    a = build_vs(B, q, k, [0, 1], 64, 100, 200)
    b = build_vs(B, q, k, [0, 1], 64, 100, 200)
    for name in ("v_idx", "s_idx", "cover_bits", "counts"):
        assert torch.equal(getattr(a, name), getattr(b, name))


def test_c0_vertical_slash_layer_end_to_end(B):
    """Workload c0 in full: index build + attention on all rows of all heads."""
    x = W.make_config("c0")
    q, k, v = x.q.cuda(), x.k.cuda(), x.v.cuda()
    N, heads = x.seq_len, [0, 1, 2, 3]
    idx = build_vs(B, q, k, heads, 64, 256, 512)
    o = torch.zeros_like(q)
    B.minf_vs_attn(q, k, v, o, heads, idx)
    torch.cuda.synchronize()
    total_swaps = 0
    for r, h in enumerate(heads):
        Qh, Kh, Vh = x.head_f64(h)
        Vg, Sg, swaps = check_vs_index(idx, r, N, Qh, Kh, 64, 256, 512)
        total_swaps += swaps
        # planted sinks are found as verticals
        assert np.isin(x.sinks[h].numpy(), Vg).mean() >= 0.9
        want = O.vs_attention(Qh, Kh, Vh, Vg, Sg, Bm=64)
        assert_close_rows(o[h], want, f"c0 head {h}")
    assert total_swaps == 0


def build_bs(B, q, k, heads, topk):
    N = q.shape[-2]
    idx = B.alloc_bs_index(len(heads), N, topk)
    ws = torch.empty(B.minf_bs_index_workspace_bytes(q, k, len(heads)), dtype=torch.uint8, device="cuda")
    B.minf_build_bs_index(q, k, heads, topk, idx, ws)
    torch.cuda.synchronize()
    return idx


def check_bs_index(idx, r, Qh, Kh, topk):
    _, cnt_o, s = O.bs_index(Qh, Kh, 64, topk)
    NB = s.shape[0]
    got = idx.blk_idx[r].cpu().numpy()
    cnt = idx.blk_cnt[r].cpu().numpy()
    assert np.array_equal(cnt, cnt_o)
    swaps = 0
    for b in range(NB):
        assert np.all(got[b, cnt[b]:] == -1)
        swaps += check_topk(got[b, :cnt[b]], s[b, :b + 1], topk, relative=False)
    # processing order: the query blocks sorted by (first kept key block, block id) -- integer work, exact
    order = idx.order[r].cpu().numpy()
    want = np.lexsort((np.arange(NB), got[:, 0]))
    assert np.array_equal(order, want)
    return got, cnt, swaps


@pytest.mark.parametrize("N,topk", [(1024, 4), (4096, 16), (1344, 100), (64, 3)])
def test_bs_index_random_inputs(B, N, topk):
    q, k, v = random_qkv(13, 4, 2, N)
    heads = [1, 2, 0]
    idx = build_bs(B, q, k, heads, topk)
    for r, h in enumerate(heads):
        check_bs_index(idx, r, to_f64(q[h]), to_f64(k[h // 2]), topk)


@pytest.mark.parametrize("NB,topk", [(64, 7), (2304, 100)])
def test_bs_index_equal_logits_keep_the_lowest_blocks(B, NB, topk):
    """Every key block is the same 64 rows, so all logits of a row are exactly equal:
    the kept blocks are the first min(topk, b+1) ones.  NB = 2304 has rows with more
    equal candidates than the selection kernel stages on chip (its general path)."""
    N = 64 * NB
    g = torch.Generator().manual_seed(21)
    q = torch.randn(1, N, 128, generator=g).to(torch.bfloat16).cuda()
    k = torch.randn(1, 64, 128, generator=g).to(torch.bfloat16).repeat(1, NB, 1).cuda()
    idx = build_bs(B, q, k, [0], topk)
    got = idx.blk_idx[0].cpu().numpy()
    cnt = idx.blk_cnt[0].cpu().numpy()
    want_cnt = np.minimum(topk, np.arange(NB) + 1)
    assert np.array_equal(cnt, want_cnt)
    want = np.where(np.arange(topk)[None, :] < want_cnt[:, None], np.arange(topk)[None, :], -1)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("topk", [100, 112, 113])
def test_bs_index_several_workgroups_ragged_tail(B, topk):
    """421 query blocks: four workgroups of the fused logits + top-k kernel, the last one ragged, rows long
    enough for many cuts of their candidate lists; 112 is the largest budget that kernel takes, 113 goes
    through the stored logits."""
    q, k, v = random_qkv(17, 2, 1, 64 * 421)
    idx = build_bs(B, q, k, [1, 0], topk)
    check_bs_index(idx, 0, to_f64(q[1]), to_f64(k[0]), topk)
    check_bs_index(idx, 1, to_f64(q[0]), to_f64(k[0]), topk)


def test_bs_index_few_distinct_logits(B):
    """Key blocks drawn from five distinct ones: every row sees five logit values, each many times over, so
    every cut of a candidate list lands on a value with far more equal entries than it may keep, and the
    kept ones must be the lowest blocks.  Equal blocks give bit-equal logits: the result is the oracle's."""
    NB, topk = 700, 100
    g = torch.Generator().manual_seed(23)
    q = torch.randn(1, 64 * NB, 128, generator=g).to(torch.bfloat16)
    proto = torch.randn(5, 64, 128, generator=g).to(torch.bfloat16)
    pick = torch.randint(0, 5, (NB,), generator=g)
    k = proto[pick].reshape(1, 64 * NB, 128)
    idx = build_bs(B, q.cuda(), k.cuda(), [0], topk)
    io, co, _ = O.bs_index(to_f64(q[0]), to_f64(k[0]), 64, topk)
    assert np.array_equal(idx.blk_cnt[0].cpu().numpy(), co)
    got = idx.blk_idx[0].cpu().numpy()
    for b in range(NB):
        assert np.array_equal(got[b, :co[b]], np.sort(io[b, :co[b]])), b


def test_bs_index_budget_above_256_blocks(B):
    """A budget larger than the number of threads of the selection workgroup."""
    q, k, v = random_qkv(15, 2, 1, 64 * 400)
    idx = build_bs(B, q, k, [1], 300)
    check_bs_index(idx, 0, to_f64(q[1]), to_f64(k[0]), 300)


def test_bs_clustered_layer_end_to_end(B):
    """Workload c3's recipe at a reduced length: index build + attention."""
    x = W.make_config("c3", N=8192, n_q_heads=4, n_kv_heads=2)
    q, k, v = x.q.cuda(), x.k.cuda(), x.v.cuda()
    heads = [0, 1, 2, 3]
    idx = build_bs(B, q, k, heads, 20)
    o = torch.zeros_like(q)
    B.minf_bs_attn(q, k, v, o, heads, idx)
    torch.cuda.synchronize()
    for r, h in enumerate(heads):
        Qh, Kh, Vh = x.head_f64(h)
        got, cnt, swaps = check_bs_index(idx, r, Qh, Kh, 20)
        want = O.bs_attention(Qh, Kh, Vh, got, cnt)
        assert_close_rows(o[h], want, f"clustered bs head {h}")


def test_index_argument_errors(B):
    q, k, v = random_qkv(14, 2, 1, 256)
    idx = B.alloc_vs_index(1, 10, 10, 256)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.MinfError) as e:
        B.minf_build_vs_index(q, k, [0], 64, 10, 10, idx, small)
    assert e.value.status == 4
    ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, 1, 64), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.MinfError) as e:
        B.minf_build_vs_index(q, k, [0], 65, 10, 10, idx, ws)       # last_q > 64
    assert e.value.status == 3
    with pytest.raises(B.MinfError) as e:
        B.minf_build_vs_index(q, k, [0], 64, 10, 0, idx, ws)        # needs at least one slash
    assert e.value.status == 3
    bidx = B.alloc_bs_index(1, 256, 4)
    with pytest.raises(B.MinfError) as e:
        B.minf_build_bs_index(q, k, [0], 4, bidx, ws, block=32)
    assert e.value.status == 5


def test_index_builders_token_major_layout(B):
    """K and Q rows n_heads * 256 bytes apart (the [token][head][128] layout)."""
    N = 2048
    q0, k0, v0 = random_qkv(23, 4, 2, N)
    q = q0.transpose(0, 1).contiguous().transpose(0, 1)
    k = k0.transpose(0, 1).contiguous().transpose(0, 1)
    heads = [3, 0]
    idx = build_vs(B, q, k, heads, 64, 30, 50)
    for r, h in enumerate(heads):
        check_vs_index(idx, r, N, to_f64(q0[h]), to_f64(k0[h // 2]), 64, 30, 50)
    bidx = build_bs(B, q, k, heads, 8)
    for r, h in enumerate(heads):
        check_bs_index(bidx, r, to_f64(q0[h]), to_f64(k0[h // 2]), 8)


def test_batch_of_two_all_calls(B):
    """[batch, heads, N, d] tensors: every entry point loops over the batch; index rows are
    batch-major (row = batch index * n_heads + position in the head list)."""
    N, nb = 1024, 2
    g = torch.Generator().manual_seed(31)
    q = torch.randn(nb, 4, N, 128, generator=g).to(torch.bfloat16).cuda()
    k = torch.randn(nb, 2, N, 128, generator=g).to(torch.bfloat16).cuda()
    v = torch.randn(nb, 2, N, 128, generator=g).to(torch.bfloat16).cuda()
    heads = [1, 2]
    # Vertical-Slash
    nv, ns = 20, 40
    idx = B.alloc_vs_index(nb * len(heads), nv, ns, N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, len(heads), 64), dtype=torch.uint8, device="cuda")
    B.minf_build_vs_index(q, k, heads, 64, nv, ns, idx, ws)
    o = torch.full_like(q, float("nan"))
    B.minf_vs_attn(q, k, v, o, heads, idx)
    torch.cuda.synchronize()
    for b in range(nb):
        for j, h in enumerate(heads):
            Qh, Kh, Vh = to_f64(q[b, h]), to_f64(k[b, h // 2]), to_f64(v[b, h // 2])
            Vg, Sg, _ = check_vs_index(idx, b * len(heads) + j, N, Qh, Kh, 64, nv, ns)
            assert_close_rows(o[b, h], O.vs_attention(Qh, Kh, Vh, Vg, Sg), f"batch {b} vs head {h}")
        assert torch.isnan(o[b, 0].float()).all() and torch.isnan(o[b, 3].float()).all()   # heads not named stay untouched
    # Block-Sparse
    topk = 5
    bidx = B.alloc_bs_index(nb * len(heads), N, topk)
    ws = torch.empty(B.minf_bs_index_workspace_bytes(q, k, len(heads)), dtype=torch.uint8, device="cuda")
    B.minf_build_bs_index(q, k, heads, topk, bidx, ws)
    o = torch.full_like(q, float("nan"))
    B.minf_bs_attn(q, k, v, o, heads, bidx)
    torch.cuda.synchronize()
    for b in range(nb):
        for j, h in enumerate(heads):
            Qh, Kh, Vh = to_f64(q[b, h]), to_f64(k[b, h // 2]), to_f64(v[b, h // 2])
            got, cnt, _ = check_bs_index(bidx, b * len(heads) + j, Qh, Kh, topk)
            assert_close_rows(o[b, h], O.bs_attention(Qh, Kh, Vh, got, cnt), f"batch {b} bs head {h}")
    # both patterns in one launch: Vertical-Slash on head 1 (rows 0 and 2 of idx), Block-Sparse on head 2
    # (rows 1 and 3 of bidx) would not line up with two-head indices, so build one-head indices
    vidx1 = B.alloc_vs_index(nb, nv, ns, N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, 1, 64), dtype=torch.uint8, device="cuda")
    B.minf_build_vs_index(q, k, [1], 64, nv, ns, vidx1, ws)
    bidx1 = B.alloc_bs_index(nb, N, topk)
    ws = torch.empty(B.minf_bs_index_workspace_bytes(q, k, 1, topk), dtype=torch.uint8, device="cuda")
    B.minf_build_bs_index(q, k, [2], topk, bidx1, ws)
    o_two = torch.full_like(q, float("nan"))
    o_one = torch.full_like(q, float("nan"))
    B.minf_vs_attn(q, k, v, o_two, [1], vidx1)
    B.minf_bs_attn(q, k, v, o_two, [2], bidx1)
    B.minf_vs_bs_attn(q, k, v, o_one, [1], vidx1, [2], bidx1)
    torch.cuda.synchronize()
    assert torch.equal(o_one[:, 1:3], o_two[:, 1:3])
    assert torch.isnan(o_one[:, 0].float()).all() and torch.isnan(o_one[:, 3].float()).all()
    # A-shape and dense
    o = torch.full_like(q, float("nan"))
    B.minf_ashape_attn(q, k, v, o, [0], 64, 200)
    B.minf_dense_attn(q, k, v, o, [3])
    torch.cuda.synchronize()
    for b in range(nb):
        assert_close_rows(o[b, 0], O.ashape_attention(to_f64(q[b, 0]), to_f64(k[b, 0]), to_f64(v[b, 0]), 64, 200), f"batch {b} a-shape")
        assert_close_rows(o[b, 3], O.dense_attention(to_f64(q[b, 3]), to_f64(k[b, 1]), to_f64(v[b, 1])), f"batch {b} dense")
