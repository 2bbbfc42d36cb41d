"""The seeded input generator: shapes, determinism, RoPE is a rotation."""
import numpy as np
import torch

from paper_2407_02490_amd import workloads as W


def test_shapes_dtype_and_determinism():
    a = W.make_config("c0", N=512)
    b = W.make_config("c0", N=512)
    assert a.q.shape == (4, 512, 128) and a.k.shape == (4, 512, 128)
    assert a.q.dtype == torch.bfloat16
    assert torch.equal(a.q, b.q) and torch.equal(a.k, b.k) and torch.equal(a.v, b.v)
    assert a.sinks.shape == (4, 16)


def test_rope_preserves_pair_norms():
    x = torch.randn(300, 128)
    y = W._rope(x.clone(), 1.0e4)
    n0 = x[:, :64] ** 2 + x[:, 64:] ** 2
    n1 = y[:, :64] ** 2 + y[:, 64:] ** 2
    assert torch.allclose(n0, n1, atol=1e-4)
    assert torch.allclose(y[0], x[0])            # position 0 is not rotated
    # relative property: <R_i a, R_j b> depends on i - j only
    a, b = torch.randn(128), torch.randn(128)
    A = W._rope(a.repeat(64, 1), 5.0e5)
    Bm = W._rope(b.repeat(64, 1), 5.0e5)
    assert abs(float(A[10] @ Bm[3]) - float(A[40] @ Bm[33])) < 1e-3


def test_gqa_layout_and_clusters():
    x = W.make_config("c3", N=1024, n_q_heads=4, n_kv_heads=2)
    assert x.q.shape[0] == 4 and x.k.shape[0] == 2
    Q, K, V = x.head_f64(3)
    assert np.array_equal(K, x.k[1].double().numpy())


def test_head_assignment_partition():
    vs, bs, a = W.head_assignment(32, 24, 6, 2)
    assert sorted(vs + bs + a) == list(range(32))
    assert (len(vs), len(bs), len(a)) == (24, 6, 2)
    assert W.head_assignment(32, 24, 6, 2) == (vs, bs, a)
