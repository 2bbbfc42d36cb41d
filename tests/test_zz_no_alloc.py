"""minf_build_vs_index_noalloc (the entry point that allocates nothing) against
minf_build_vs_index, through the C ABI: two calls in a row, the second with a
smaller input; then a size beyond the scratch array's is refused."""
import pytest
import torch

from tests.helpers import random_qkv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2407_02490_amd import binding
    binding.lib()
    return binding


def both(B, q, k, heads, last_q, nv, ns):
    N = q.shape[-2]
    ref = B.alloc_vs_index(len(heads), nv, ns, N)
    ws = torch.empty(B.minf_vs_index_workspace_bytes(q, k, len(heads), last_q), dtype=torch.uint8, device="cuda")
    B.minf_build_vs_index(q, k, heads, last_q, nv, ns, ref, ws)
    got = B.alloc_vs_index(len(heads), nv, ns, N)
    for t in (got.v_idx, got.s_idx, got.cover, got.cover_bits, got.counts):
        t.fill_(-7)
    B.minf_build_vs_index_noalloc(q, k, heads, last_q, nv, ns, got)
    torch.cuda.synchronize()
    return ref, got


def same(ref, got):
    # index work: bit-exact
    assert torch.equal(ref.counts, got.counts)
    assert torch.equal(ref.v_idx, got.v_idx) and torch.equal(ref.s_idx, got.s_idx)
    assert torch.equal(ref.cover_bits, got.cover_bits)
    for r in range(ref.rows):
        n_c = int(ref.counts[r, 2])
        assert torch.equal(ref.cover[r, :n_c], got.cover[r, :n_c])


def test_noalloc_entry_matches_the_workspace_entry_twice_in_a_row(B):
    q, k, v = random_qkv(41, 4, 2, 8192)
    ref, got = both(B, q, k, [0, 1, 2, 3], 64, 200, 700)
    same(ref, got)
    # second call: a smaller input (fewer heads, shorter sequence, fewer estimating rows);
    # whatever the first call left in the scratch array must not matter
    q2, k2, v2 = random_qkv(42, 2, 1, 2112)
    ref2, got2 = both(B, q2, k2, [1, 0], 17, 50, 90)
    same(ref2, got2)


def test_noalloc_entry_refuses_sizes_beyond_its_scratch_array(B):
    N = 1 << 20                                  # 16 heads x 1M tokens need 296 MiB of workspace, the array holds 96
    q = torch.empty(16, N, 128, dtype=torch.bfloat16, device="cuda")
    k = torch.empty(4, N, 128, dtype=torch.bfloat16, device="cuda")
    idx = B.alloc_vs_index(16, 8, 8, N)
    idx.counts.fill_(-7)
    with pytest.raises(B.MinfError) as e:
        B.minf_build_vs_index_noalloc(q, k, list(range(16)), 64, 8, 8, idx)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert (idx.counts == -7).all()              # nothing was launched
