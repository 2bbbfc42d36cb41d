"""The parity bar of the GPU tests can fail where it must (CPU only).

With thousands of attended keys per row an output element is ~0.02 in
magnitude, so the absolute bar (2e-2 max, 5e-3 mean) alone would accept an
output that lost a whole 64-key tile.  The mistake is planted in the oracle's
mask; the relative-L2 criterion of tests/helpers.assert_close_rows must catch
it while plain bf16 rounding of the right answer passes."""
import numpy as np
import pytest
import torch

from oracle import minference_oracle as O
from tests.helpers import MAX_ABS, MEAN_ABS, REL_L2, assert_close_rows, error_norms


def to_bf16(a):
    return torch.from_numpy(a).to(torch.bfloat16)


def test_a_dropped_tile_fails_the_relative_criterion_only(rng):
    N, d, n_init, n_local = 8192, 128, 1024, 4096
    Q = to_bf16(rng.normal(size=(N, d))).double().numpy()
    K = to_bf16(rng.normal(size=(N, d))).double().numpy()
    V = to_bf16(rng.normal(size=(N, d))).double().numpy()
    i0 = 64 * 100
    mask = O.ashape_rows(i0, i0 + 64, N, n_init, n_local)
    want = O.attend(Q[i0:i0 + 64], K, V, mask)
    assert_close_rows(to_bf16(want), want, "bf16 rounding of the right answer")
    bad_mask = mask.copy()
    bad_mask[:, 4096:4160] = False                       # one 64-key tile of the window is lost
    bad = O.attend(Q[i0:i0 + 64], K, V, bad_mask)
    mx, mean, rel = error_norms(to_bf16(bad).double().numpy(), want)
    # the absolute bar hardly sees it (the mean is far inside, the maximum sits at the bar) ...
    assert mean <= MEAN_ABS / 2 and mx <= 1.5 * MAX_ABS
    # ... the relative one does, by a wide margin
    assert rel > 4 * REL_L2
    with pytest.raises(AssertionError):
        assert_close_rows(to_bf16(bad), want, "one tile dropped")


def test_dropped_verticals_fail_the_relative_criterion(rng):
    N, d = 16384, 128
    Q = to_bf16(rng.normal(size=(N, d))).double().numpy()
    K = to_bf16(rng.normal(size=(N, d))).double().numpy()
    V = to_bf16(rng.normal(size=(N, d))).double().numpy()
    Vl = np.sort(rng.choice(N, 1000, replace=False))
    Sl = np.arange(0, 12000)                                   # a wide band: 12000 keys per row
    i0 = 64 * 250
    want = O.vs_attention(Q, K, V, Vl, Sl, i0, i0 + 64)
    assert_close_rows(to_bf16(want), want, "bf16 rounding of the right answer")
    # the whole gathered phase lost: every vertical outside the band (about 250 of 12250 keys)
    bad = O.vs_attention(Q, K, V, Vl[Vl > i0 - 12000], Sl, i0, i0 + 64)
    mx, mean, rel = error_norms(to_bf16(bad).double().numpy(), want)
    assert mx <= MAX_ABS and mean <= MEAN_ABS                  # inside the absolute bar
    assert rel > 2 * REL_L2
    with pytest.raises(AssertionError, match="relative L2"):
        assert_close_rows(to_bf16(bad), want, "verticals dropped")
