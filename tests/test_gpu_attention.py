"""Parity of the HIP attention kernels with the CPU oracle, through the C ABI.

Sizes span several 64-key tiles, several 4-block workgroups, ragged mask edges
(window and sink sizes that are not multiples of 64) and the degenerate cases.
Bar: 2e-2 max-abs, 5e-3 mean-abs on bf16 outputs (tests/helpers.py).
"""
import numpy as np
import pytest
import torch

from oracle import minference_oracle as O
from paper_2407_02490_amd import workloads as W
from tests.helpers import assert_close_rows, random_qkv, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2407_02490_amd import binding
    binding.lib()
    return binding


def run_heads(fn, q, k, v, heads, *args):
    o = torch.full_like(q, float("nan"))
    fn(q, k, v, o, heads, *args)
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("N,nq,nkv", [(64, 1, 1), (320, 2, 1), (1024, 4, 2)])
def test_dense_matches_oracle(B, N, nq, nkv):
    q, k, v = random_qkv(1, nq, nkv, N)
    o = run_heads(B.minf_dense_attn, q, k, v, list(range(nq)))
    g = nq // nkv
    for h in range(nq):
        want = O.dense_attention(to_f64(q[h]), to_f64(k[h // g]), to_f64(v[h // g]))
        assert_close_rows(o[h], want, f"dense N={N} head {h}")


@pytest.mark.parametrize("heads", [[0, 1, 2, 3, 4, 5, 6, 7, 8], [5, 1, 12, 3], [9, 10, 11, 15, 2, 3],
                                   list(range(16))])
def test_head_lists_of_mixed_kv_groups(B, rng, heads):
    """Work items are scheduled in chunks of consecutive list entries that share a K/V head
    (here 8 query heads per K/V head): full and partial groups, a group longer than one chunk
    would be, unsorted lists.  Every listed (head, block) must be computed exactly once, by
    all three kernels' mappings, and no other head touched."""
    N, nq, nkv = 704, 16, 2            # 11 blocks
    q, k, v = random_qkv(5, nq, nkv, N)
    NB = N // 64
    o = run_heads(B.minf_dense_attn, q, k, v, heads)
    idxs = [random_bs_index(rng, NB, 3) for _ in heads]
    dev = B.bs_index_from_host(np.stack([i for i, _ in idxs]), np.stack([c for _, c in idxs]))
    ob = run_heads(B.minf_bs_attn, q, k, v, heads, dev)
    Vl, Sl = [0, 100, 333], [0, 1, 200]
    ov = run_heads(B.minf_vs_attn, q, k, v, heads, B.vs_index_from_host([Vl] * len(heads), [Sl] * len(heads), N))
    for r, h in enumerate(heads):
        Qh, Kh, Vh = to_f64(q[h]), to_f64(k[h // 8]), to_f64(v[h // 8])
        assert_close_rows(o[h], O.dense_attention(Qh, Kh, Vh), f"dense head {h}")
        assert_close_rows(ob[h], O.bs_attention(Qh, Kh, Vh, idxs[r][0], idxs[r][1]), f"bs head {h}")
        assert_close_rows(ov[h], O.vs_attention(Qh, Kh, Vh, Vl, Sl, Bm=64), f"vs head {h}")
    for h in set(range(nq)) - set(heads):
        assert torch.isnan(o[h].float()).all() and torch.isnan(ob[h].float()).all() and torch.isnan(ov[h].float()).all()


@pytest.mark.parametrize("n_init,n_local", [(64, 128), (100, 200), (0, 65), (5, 1), (1024, 4096), (130, 64)])
def test_ashape_matches_oracle(B, n_init, n_local):
    N, nq, nkv = 1344, 4, 2          # 21 blocks: last workgroup has one idle wave slot
    q, k, v = random_qkv(2, nq, nkv, N)
    heads = [3, 0, 2]
    o = run_heads(B.minf_ashape_attn, q, k, v, heads, n_init, n_local)
    for h in heads:
        want = O.ashape_attention(to_f64(q[h]), to_f64(k[h // 2]), to_f64(v[h // 2]), n_init, n_local)
        assert_close_rows(o[h], want, f"ashape ({n_init},{n_local}) head {h}")
    assert torch.isnan(o[1].float()).all()       # heads not listed are left untouched


def test_ashape_strided_views_and_scale(B):
    # q/k/v as slices of a fused [N, H, d] projection output (token-major)
    N, nq, nkv = 512, 4, 4
    g = torch.Generator().manual_seed(5)
    fused = torch.randn(N, 3 * nq, 128, generator=g).to(torch.bfloat16).cuda()
    q = fused[:, 0:nq].transpose(0, 1)
    k = fused[:, nq:2 * nq].transpose(0, 1)
    v = fused[:, 2 * nq:].transpose(0, 1)
    o = torch.zeros(nq, N, 128, dtype=torch.bfloat16, device="cuda")
    B.minf_ashape_attn(q, k, v, o, [1, 2], 64, 128, scale=0.05)
    torch.cuda.synchronize()
    for h in (1, 2):
        want = O.ashape_attention(to_f64(q[h]), to_f64(k[h]), to_f64(v[h]), 64, 128, scale=0.05)
        assert_close_rows(o[h], want, f"strided head {h}")


def random_bs_index(rng, NB, topk, dense_diag=True):
    idx = -np.ones((NB, topk), np.int64)
    cnt = np.zeros(NB, np.int64)
    for b in range(NB):
        c = min(topk, b + 1)
        sel = np.sort(rng.choice(b + 1, c, replace=False))
        idx[b, :c], cnt[b] = sel, c
    return idx, cnt


def test_bs_matches_oracle(B, rng):
    N, nq, nkv, topk = 1024, 4, 2, 5
    NB = N // 64
    q, k, v = random_qkv(3, nq, nkv, N)
    heads = [0, 3]
    idxs = [random_bs_index(rng, NB, topk) for _ in heads]
    dev = B.bs_index_from_host(np.stack([i for i, _ in idxs]), np.stack([c for _, c in idxs]))
    o = run_heads(B.minf_bs_attn, q, k, v, heads, dev)
    for r, h in enumerate(heads):
        want = O.bs_attention(to_f64(q[h]), to_f64(k[h // 2]), to_f64(v[h // 2]), idxs[r][0], idxs[r][1])
        assert_close_rows(o[h], want, f"bs head {h}")


def test_bs_list_longer_than_one_lane_chunk(B, rng):
    """More than 64 listed blocks per query block: the list is walked in chunks of 64 ids."""
    N, topk = 8192, 100
    NB = N // 64
    q, k, v = random_qkv(22, 1, 1, N)
    idx, cnt = random_bs_index(rng, NB, topk)
    dev = B.bs_index_from_host(idx[None], cnt[None])
    o = run_heads(B.minf_bs_attn, q, k, v, [0], dev)
    want = O.bs_attention(to_f64(q[0]), to_f64(k[0]), to_f64(v[0]), idx, cnt)
    assert_close_rows(o[0], want, "bs topk=100")


def test_bs_processing_order_does_not_change_the_result(B, rng):
    """The index may carry an order in which the query blocks are taken (any permutation):
    the output is bit-identical to the natural order's."""
    N, topk = 1344, 4                   # 21 blocks
    NB = N // 64
    q, k, v = random_qkv(6, 2, 1, N)
    idxs = [random_bs_index(rng, NB, topk) for _ in range(2)]
    bi, bc = np.stack([i for i, _ in idxs]), np.stack([c for _, c in idxs])
    o_nat = run_heads(B.minf_bs_attn, q, k, v, [0, 1], B.bs_index_from_host(bi, bc))
    order = np.stack([rng.permutation(NB), np.arange(NB)[::-1]])
    o_perm = run_heads(B.minf_bs_attn, q, k, v, [0, 1], B.bs_index_from_host(bi, bc, order=order))
    assert torch.equal(o_nat, o_perm)
    for h in (0, 1):
        want = O.bs_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]), idxs[h][0], idxs[h][1])
        assert_close_rows(o_perm[h], want, f"bs with order, head {h}")


def test_bs_full_index_is_dense(B):
    N = 512
    NB = N // 64
    q, k, v = random_qkv(4, 1, 1, N)
    idx = np.tile(np.arange(NB), (NB, 1))
    cnt = np.arange(1, NB + 1)
    idx = np.where(idx < cnt[:, None], idx, -1)
    dev = B.bs_index_from_host(idx[None], cnt[None])
    o = run_heads(B.minf_bs_attn, q, k, v, [0], dev)
    assert_close_rows(o[0], O.dense_attention(to_f64(q[0]), to_f64(k[0]), to_f64(v[0])), "bs dense limit")


def test_bs_ignores_bad_block_ids(B):
    N = 256
    q, k, v = random_qkv(6, 1, 1, N)
    idx = np.array([[[0, -1, 99], [0, 1, 4], [7, 1, 2], [0, 3, -5]]])
    cnt = np.array([[3, 3, 3, 3]])
    dev = B.bs_index_from_host(idx, cnt)
    o = run_heads(B.minf_bs_attn, q, k, v, [0], dev)
    clean_idx = np.array([[0, -1, -1], [0, 1, -1], [1, 2, -1], [0, 3, -1]])
    want = O.bs_attention(to_f64(q[0]), to_f64(k[0]), to_f64(v[0]), clean_idx, np.array([1, 2, 2, 2]))
    assert_close_rows(o[0], want, "bs bad ids")


def token_major(t):
    """The same values in a [token][head][128] buffer, viewed as [head][token][128]:
    rows of one head are then n_heads * 256 bytes apart (the kernels' general-stride path)."""
    return t.transpose(0, 1).contiguous().transpose(0, 1)


def test_token_major_layout_bs_vs_dense(B, rng):
    N, nq, nkv = 1024, 4, 2
    NB = N // 64
    q0, k0, v0 = random_qkv(21, nq, nkv, N)
    q, k, v = token_major(q0), token_major(k0), token_major(v0)
    assert k.stride(1) == nkv * 128 and q.stride(1) == nq * 128
    # Block-Sparse
    heads = [1, 2]
    idxs = [random_bs_index(rng, NB, 5) for _ in heads]
    dev = B.bs_index_from_host(np.stack([i for i, _ in idxs]), np.stack([c for _, c in idxs]))
    o = token_major(torch.full_like(q0, float("nan")))
    B.minf_bs_attn(q, k, v, o, heads, dev)
    torch.cuda.synchronize()
    for r, h in enumerate(heads):
        want = O.bs_attention(to_f64(q0[h]), to_f64(k0[h // 2]), to_f64(v0[h // 2]), idxs[r][0], idxs[r][1])
        assert_close_rows(o[h], want, f"token-major bs head {h}")
    # Vertical-Slash: runs, verticals and a run that ends at the end of the sequence
    Vl, Sl = list(range(0, N, 37)), [0, 1, 2, 3, 130, 131, 400, 1000]
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    o = token_major(torch.full_like(q0, float("nan")))
    B.minf_vs_attn(q, k, v, o, [0, 3], dev)
    torch.cuda.synchronize()
    for h in (0, 3):
        want = O.vs_attention(to_f64(q0[h]), to_f64(k0[h // 2]), to_f64(v0[h // 2]), Vl, Sl, Bm=64)
        assert_close_rows(o[h], want, f"token-major vs head {h}")
    # dense
    o = token_major(torch.full_like(q0, float("nan")))
    B.minf_dense_attn(q, k, v, o, [2])
    torch.cuda.synchronize()
    assert_close_rows(o[2], O.dense_attention(to_f64(q0[2]), to_f64(k0[1]), to_f64(v0[1])), "token-major dense")


VS_CASES = [
    # (N, verticals, slashes)
    (512, [3, 70, 71, 300, 511], [0, 5, 64, 200, 201, 450]),
    (1024, list(range(0, 1024, 37)), [0, 1, 2, 3, 130, 131, 400, 1000]),
    (1024, [0], [0]),                                   # only-slash / only-vertical limits
    (768, list(range(768)), [0]),                       # every vertical: dense
    (768, [5], list(range(768))),                       # every slash: dense
    (640, [600, 601], [500]),                           # early blocks have no permitted key
]


@pytest.mark.parametrize("N,Vl,Sl", VS_CASES)
def test_vs_matches_oracle(B, N, Vl, Sl):
    q, k, v = random_qkv(7, 2, 1, N)
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    o = run_heads(B.minf_vs_attn, q, k, v, [0, 1], dev)
    for h in (0, 1):
        want = O.vs_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]), Vl, Sl, Bm=64)
        assert_close_rows(o[h], want, f"vs N={N} head {h}")


@pytest.fixture
def ring_engine():
    """Selects the shared-tile Vertical-Slash engine (four waves per workgroup) for one test."""
    import os
    old = os.environ.get("MINF_VS_ENGINE")
    os.environ["MINF_VS_ENGINE"] = "ring"
    yield
    if old is None:
        del os.environ["MINF_VS_ENGINE"]
    else:
        os.environ["MINF_VS_ENGINE"] = old


RING_CASES = VS_CASES + [
    # 21 and 13 blocks: the last workgroup has idle waves; narrow, wide and neighbouring runs,
    # runs that start before key 0 for some of the four blocks of a workgroup only
    (1344, [0, 7, 640, 1300], [0, 1, 2, 3, 64, 130, 131, 400, 401, 402, 700, 1000, 1343]),
    (832, list(range(0, 832, 5)), list(range(0, 200)) + [300, 301, 302, 500, 831]),
    (64, [3], [0]),
]


@pytest.mark.parametrize("N,Vl,Sl", RING_CASES)
def test_vs_ring_engine_matches_oracle(B, ring_engine, N, Vl, Sl):
    q, k, v = random_qkv(7, 2, 1, N)
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    o = run_heads(B.minf_vs_attn, q, k, v, [0, 1], dev)
    for h in (0, 1):
        want = O.vs_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]), Vl, Sl, Bm=64)
        assert_close_rows(o[h], want, f"vs ring N={N} head {h}")


def test_vs_ring_engine_many_runs_token_major_and_fallback(B, ring_engine, rng):
    """More than 64 runs (the run list is taken 64 at a time), the general-stride tile fetch, and
    the exact two-pass fallback, all through the shared-tile engine."""
    N = 32768
    q0, k0, v0 = random_qkv(23, 2, 1, N)
    Sl = sorted(set(rng.choice(N, 150, replace=False).tolist()) | set(range(0, 100)))
    Vl = sorted(rng.choice(N, 300, replace=False).tolist())
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    assert int(dev.counts[0, 2]) > 64
    q, k, v = token_major(q0), token_major(k0), token_major(v0)
    o = token_major(torch.full_like(q0, float("nan")))
    B.minf_vs_attn(q, k, v, o, [0, 1], dev)
    torch.cuda.synchronize()
    blocks = [0, 1, 2, 3, 4, 63, 64, 100, 255, 256, 257, 510, 511]
    for h in (0, 1):
        Qh, Kh, Vh = to_f64(q0[h]), to_f64(k0[0]), to_f64(v0[0])
        for b in blocks:
            want = O.vs_attention(Qh, Kh, Vh, Vl, Sl, 64 * b, 64 * b + 64, Bm=64)
            assert_close_rows(o[h, 64 * b:64 * b + 64], want, f"ring token-major head {h} block {b}")
    k1 = k0.clone()
    k1[:, 20000:] *= 60.0
    o = run_heads(B.minf_vs_attn, q0, k1, v0, [0, 1], dev)
    for b in (300, 400, 511):
        want = O.vs_attention(to_f64(q0[1]), to_f64(k1[0]), to_f64(v0[0]), Vl, Sl, 64 * b, 64 * b + 64, Bm=64)
        assert_close_rows(o[1, 64 * b:64 * b + 64], want, f"ring fallback block {b}")


def test_scale_other_than_default_through_vs_and_bs(B, rng):
    """softmax_scale != 1/sqrt(d) through both sparse attention calls (caller-filled indices)."""
    N, NB, scale = 1024, 16, 0.21
    q, k, v = random_qkv(31, 2, 1, N)
    Vl, Sl = [0, 5, 300, 777], [0, 1, 2, 200, 201, 640]
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    o = torch.full_like(q, float("nan"))
    B.minf_vs_attn(q, k, v, o, [0, 1], dev, scale=scale)
    idxs = [random_bs_index(rng, NB, 4) for _ in range(2)]
    devb = B.bs_index_from_host(np.stack([i for i, _ in idxs]), np.stack([c for _, c in idxs]))
    ob = torch.full_like(q, float("nan"))
    B.minf_bs_attn(q, k, v, ob, [0, 1], devb, scale=scale)
    torch.cuda.synchronize()
    for h in (0, 1):
        Qh, Kh, Vh = to_f64(q[h]), to_f64(k[0]), to_f64(v[0])
        assert_close_rows(o[h], O.vs_attention(Qh, Kh, Vh, Vl, Sl, Bm=64, scale=scale), f"vs scale head {h}")
        assert_close_rows(ob[h], O.bs_attention(Qh, Kh, Vh, idxs[h][0], idxs[h][1], scale=scale), f"bs scale head {h}")
        # the scale matters: the default-scale result is far outside the bar
        assert np.abs(O.vs_attention(Qh, Kh, Vh, Vl, Sl, Bm=64) - o[h].double().cpu().numpy()).max() > 5e-2


def test_vs_many_columns_more_than_one_round(B, rng):
    # more kept verticals than one LDS round holds (1024): the column phase runs twice
    N = 2048
    q, k, v = random_qkv(8, 1, 1, N)
    Vl = sorted(rng.choice(N, 1500, replace=False).tolist())
    Sl = [0, 777]
    dev = B.vs_index_from_host([Vl], [Sl], N)
    o = run_heads(B.minf_vs_attn, q, k, v, [0], dev)
    want = O.vs_attention(to_f64(q[0]), to_f64(k[0]), to_f64(v[0]), Vl, Sl, Bm=64)
    assert_close_rows(o[0], want, "vs 1500 columns")


def test_outputs_are_bit_reproducible(B, rng):
    """No kernel of the path accumulates through atomics or in a timing-dependent order: two runs
    on the same inputs give identical bits (all four attention calls, index from the GPU)."""
    N = 4096
    x = W.make_config("c4", device="cuda", N=N, n_q_heads=8, n_kv_heads=2)
    heads = list(range(8))
    outs = []
    for _ in range(2):
        vi = B.alloc_vs_index(8, 100, 300, N)
        ws = torch.empty(B.minf_vs_index_workspace_bytes(x.q, x.k, 8, 64), dtype=torch.uint8, device="cuda")
        B.minf_build_vs_index(x.q, x.k, heads, 64, 100, 300, vi, ws)
        bi = B.alloc_bs_index(8, N, 9)
        ws2 = torch.empty(B.minf_bs_index_workspace_bytes(x.q, x.k, 8), dtype=torch.uint8, device="cuda")
        B.minf_build_bs_index(x.q, x.k, heads, 9, bi, ws2)
        o = [torch.empty_like(x.q) for _ in range(4)]
        B.minf_vs_attn(x.q, x.k, x.v, o[0], heads, vi)
        B.minf_bs_attn(x.q, x.k, x.v, o[1], heads, bi)
        B.minf_ashape_attn(x.q, x.k, x.v, o[2], heads, 128, 512)
        B.minf_dense_attn(x.q, x.k, x.v, o[3], heads)
        torch.cuda.synchronize()
        outs.append(o + [vi.v_idx.clone(), vi.s_idx.clone(), vi.cover_bits.clone(), bi.blk_idx.clone(), bi.order.clone()])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_bad_arguments_are_rejected_before_launch(B):
    q, k, v = random_qkv(9, 2, 1, 128)
    o = torch.zeros_like(q)
    with pytest.raises(B.MinfError) as e:
        B.minf_ashape_attn(q, k, v, o, [5], 64, 64)           # head id out of range
    assert e.value.status == 2
    with pytest.raises(B.MinfError) as e:
        B.minf_ashape_attn(q, k, v, o, [0], 64, 0)            # n_local < 1
    assert e.value.status == 3
    with pytest.raises(B.MinfError) as e:
        B.minf_dense_attn(q[:, :100], k[:, :100], v[:, :100], o[:, :100], [0])   # N % 64 != 0
    assert e.value.status == 2
    assert (o == 0).all()


def test_exact_two_pass_fallback(B):
    """Logits that outgrow the first step's row max by far more than 2^100
    overflow the optimistic fixed-reference pass; the kernels must detect it
    and redo the query block with the exact two-pass scheme."""
    N = 1024
    q, k, v = random_qkv(21, 2, 1, N)
    k = k.clone()
    k[:, 700:] *= 60.0                      # late keys: logits of +-100s of nats
    # dense / A-shape
    o = run_heads(B.minf_dense_attn, q, k, v, [0, 1])
    for h in (0, 1):
        want = O.dense_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]))
        assert_close_rows(o[h], want, f"fallback dense head {h}")
    # Block-Sparse with every block kept
    NB = N // 64
    idx = np.tile(np.arange(NB), (NB, 1))
    cnt = np.arange(1, NB + 1)
    idx = np.where(idx < cnt[:, None], idx, -1)
    dev = B.bs_index_from_host(np.stack([idx, idx]), np.stack([cnt, cnt]))
    o = run_heads(B.minf_bs_attn, q, k, v, [0, 1], dev)
    assert_close_rows(o[1], O.dense_attention(to_f64(q[1]), to_f64(k[0]), to_f64(v[0])), "fallback bs")
    # Vertical-Slash: a local band plus verticals inside the scaled region
    Vl, Sl = [5, 710, 800, 1000], list(range(0, 96)) + [300]
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    o = run_heads(B.minf_vs_attn, q, k, v, [0, 1], dev)
    for h in (0, 1):
        want = O.vs_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]), Vl, Sl, Bm=64)
        assert_close_rows(o[h], want, f"fallback vs head {h}")


def test_exact_fallback_on_underflow(B):
    """Strongly negative logits (every key nearly opposite to every query): a row whose exponent
    reference is the neutral 0 -- no permitted key in the first step its wave computes -- would
    flush every term to zero; the kernels must notice the vanishing row sum and redo the block
    exactly.  That is A-shape without sink and with a window shorter than a workgroup's rows (the
    last wave's rows see nothing in the workgroup's first tile); Vertical-Slash and Block-Sparse
    rows always find a key in their first step and are checked here for the extreme logits only."""
    N = 1024
    g = torch.Generator().manual_seed(77)
    u = torch.randn(128, generator=g)
    u = u / u.norm() * (128 ** 0.5)
    q = (u + 0.3 * torch.randn(2, N, 128, generator=g)).to(torch.bfloat16).cuda()
    k = (-14.0 * u + 0.3 * torch.randn(1, N, 128, generator=g)).to(torch.bfloat16).cuda()
    v = torch.randn(1, N, 128, generator=g).to(torch.bfloat16).cuda()
    # logits are about -14 * 128 / sqrt(128) = -158 nats = -228 in the base-2 domain
    assert float((q[0, 100].float() @ k[0, 50].float()) / 128 ** 0.5) < -120
    o = run_heads(B.minf_ashape_attn, q, k, v, [0, 1], 0, 65)
    for h in (0, 1):
        want = O.ashape_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]), 0, 65)
        assert np.abs(want).max() > 0.1
        assert_close_rows(o[h], want, f"underflow A-shape head {h}")
    Vl, Sl = [3, 500], [0, 200, 201, 700]
    dev = B.vs_index_from_host([Vl, Vl], [Sl, Sl], N)
    o = run_heads(B.minf_vs_attn, q, k, v, [0, 1], dev)
    for h in (0, 1):
        want = O.vs_attention(to_f64(q[h]), to_f64(k[0]), to_f64(v[0]), Vl, Sl, Bm=64)
        assert_close_rows(o[h], want, f"underflow VS head {h}")
    idx, cnt = np.array([[[0, -1]] + [[0, b] for b in range(1, 16)]]), np.array([[1] + [2] * 15])
    devb = B.bs_index_from_host(idx, cnt)
    o = run_heads(B.minf_bs_attn, q, k, v, [0], devb)
    assert_close_rows(o[0], O.bs_attention(to_f64(q[0]), to_f64(k[0]), to_f64(v[0]), idx[0], cnt[0]), "underflow BS")


def test_vs_and_bs_heads_in_one_launch_match_the_two_calls_bit_for_bit(B):
    """minf_vs_bs_attn (Section 3.2 / App. E: a layer mixes the patterns): the interleaved launch gives what
    minf_vs_attn followed by minf_bs_attn give, and leaves the other heads alone; token-major layout too."""
    N = 4096
    for layout in ("head", "token"):
        q, k, v = random_qkv(71, 8, 2, N)
        if layout == "token":
            def tm(t):
                return t.transpose(0, 1).contiguous().transpose(0, 1)
            q, k, v = tm(q), tm(k), tm(v)
        vs_heads, bs_heads = [0, 1, 5], [2, 7]
        vidx = B.alloc_vs_index(len(vs_heads), 48, 100, N)
        ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, len(vs_heads), 64), dtype=torch.uint8, device="cuda")
        B.minf_build_vs_index(q, k, vs_heads, 64, 48, 100, vidx, ws)
        bidx = B.alloc_bs_index(len(bs_heads), N, 9)
        ws2 = torch.empty(B.minf_bs_index_workspace_bytes(q, k, len(bs_heads), 9), dtype=torch.uint8, device="cuda")
        B.minf_build_bs_index(q, k, bs_heads, 9, bidx, ws2)
        o1 = torch.full_like(q, 7.0)
        o2 = torch.full_like(q, 7.0)
        B.minf_vs_attn(q, k, v, o1, vs_heads, vidx)
        B.minf_bs_attn(q, k, v, o1, bs_heads, bidx)
        B.minf_vs_bs_attn(q, k, v, o2, vs_heads, vidx, bs_heads, bidx)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2), layout
        assert bool((o2[[3, 4, 6]] == 7.0).all())
        # against the oracle, one head of each kind
        Vg, Sg = vidx.v_idx[1].cpu().numpy(), vidx.s_idx[1].cpu().numpy()
        cnt = vidx.counts[1].cpu().numpy()
        Qh, Kh, Vh = to_f64(q[1]), to_f64(k[0]), to_f64(v[0])
        assert_close_rows(o2[1], O.vs_attention(Qh, Kh, Vh, Vg[:cnt[0]], Sg[:cnt[1]], Bm=64), f"one launch VS {layout}")
        Qh, Kh, Vh = to_f64(q[7]), to_f64(k[1]), to_f64(v[1])
        bi, bc = bidx.blk_idx[1].cpu().numpy(), bidx.blk_cnt[1].cpu().numpy()
        assert_close_rows(o2[7], O.bs_attention(Qh, Kh, Vh, bi, bc, B=64), f"one launch BS {layout}")
    with pytest.raises(B.MinfError) as e:
        B.minf_vs_bs_attn(q, k, v, o2, [0, 1], vidx, [1], bidx)      # head 1 in both lists
    assert e.value.status == 2
