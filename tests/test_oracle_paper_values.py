"""The oracle's tile counters against the figures the paper itself prints
(tests/golden/paper_values.txt, each with its place in the paper): the
block-sparse speedup formula of App. C.4.1 and the "sparsity in kernel"
thresholds of App. F, at the budgets of Section 4 / App. C.2."""
import os

import numpy as np

from oracle import minference_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def paper_values():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, value, _where = [f.strip() for f in line.split(";", 2)]
        out[name] = [float(v) for v in value.split()]
    return out


def bs_counts(N, B, k):
    return np.minimum(k, np.arange(N // B) + 1)


def test_block_sparse_speedup_formula():
    """App. C.4.1: dense tiles / block-sparse tiles is about S / (2 B k_b) once S >> B k_b."""
    P = paper_values()
    B, k, div = int(P["block_size"][0]), int(P["bs_topk"][0]), P["bs_speedup_divisor"][0]
    for N in (131072, 262144, 1048576):
        ratio = O.tiles_dense(N, B).sum() / O.tiles_bs(bs_counts(N, B, k)).sum()
        want = N / (div * B * k)
        # the formula ignores the diagonal (+1 block per row) and the short first rows
        assert abs(ratio / want - 1) < 0.03, (N, ratio, want)


def ashape_total(N, n_init, n_local, B):
    """Sum of the oracle's A-shape tile counts over all query blocks.  Masking every block of a
    200k-token sequence takes too long; past the blocks that still see the sink and the window
    grow, the count is the same for every block (checked on samples), so those are taken once."""
    NB = N // B
    head = (n_init + n_local) // B + 4
    first = O.tiles_ashape(N, n_init, n_local, B, blocks=list(range(head)))
    probe = sorted({head, head + 1, (head + NB) // 2, NB - 2, NB - 1})
    rest = O.tiles_ashape(N, n_init, n_local, B, blocks=probe)
    assert np.all(rest == rest[0])
    return first.sum() + rest[0] * (NB - head)


def test_sparsity_in_kernel_thresholds():
    """App. F: beyond 200k tokens more than 90 % of the causal tile triangle is skipped, beyond
    500k more than 95 % -- checked for the two patterns whose tile counts do not depend on data."""
    P = paper_values()
    B, k = int(P["block_size"][0]), int(P["bs_topk"][0])
    n_init, n_local = (int(v) for v in P["ashape_budget"])
    for N, key in ((204800, "sparsity_beyond_200k"), (512000, "sparsity_beyond_500k")):
        dense = O.tiles_dense(N, B).sum()
        assert 1.0 - ashape_total(N, n_init, n_local, B) / dense > P[key][0]
        assert 1.0 - O.tiles_bs(bs_counts(N, B, k)).sum() / dense > P[key][0]
    # and the statement is not vacuous: at 32k tokens neither pattern reaches 90 %
    N = 32768
    dense = O.tiles_dense(N, B).sum()
    assert 1.0 - O.tiles_ashape(N, n_init, n_local, B).sum() / dense < 0.90
    assert 1.0 - O.tiles_bs(bs_counts(N, B, k)).sum() / dense < 0.90
