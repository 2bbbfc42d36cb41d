"""Host-side tile counter of the product against the oracle's independent counts."""
import numpy as np
import pytest

from oracle import minference_oracle as O
from paper_2407_02490_amd import costmodel as C


@pytest.mark.parametrize("n_init,n_local", [(1024, 4096), (100, 200), (0, 65), (64, 64), (5, 1), (4096, 1)])
def test_ashape_tiles(n_init, n_local):
    N = 8192
    assert np.array_equal(C.tiles_ashape(N, n_init, n_local), O.tiles_ashape(N, n_init, n_local))


def test_dense_and_ashape_limits():
    N = 4096
    assert np.array_equal(C.tiles_dense(N), O.tiles_dense(N))
    assert np.array_equal(C.tiles_ashape(N, 0, N), C.tiles_dense(N))
    assert C.tile_flops() == 2097152


def runs_of(S, N):
    cover = O.slash_cover(S, N, 64).astype(np.int8)
    e = np.diff(np.concatenate([[0], cover, [0]]))
    return np.stack([np.flatnonzero(e == 1) - 64, np.flatnonzero(e == -1) - 64], axis=1)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_vs_tiles_match_oracle(seed):
    rng = np.random.default_rng(seed)
    N = 4096
    V = np.sort(rng.choice(N, 300, replace=False))
    S = np.sort(np.concatenate([np.arange(0, 200), rng.choice(np.arange(200, N), 60, replace=False)]))
    assert np.array_equal(C.tiles_vs(N, V, runs_of(S, N)), O.tiles_vs(N, V, S))


@pytest.mark.parametrize("seed", [3, 4])
def test_vs_executed_steps_match_oracle(seed):
    """The 64 x 32 steps the Vertical-Slash kernel executes (what its FLOP rate is computed from):
    never more than two per canonical tile, fewer whenever a run's length mod 64 is in 1 .. 32."""
    rng = np.random.default_rng(seed)
    N = 4096
    V = np.sort(rng.choice(N, 300, replace=False))
    S = np.sort(np.concatenate([np.arange(0, 90), rng.choice(np.arange(200, N), 60, replace=False)]))
    steps = C.tiles_vs(N, V, runs_of(S, N), width=C.STEP)
    assert np.array_equal(steps, O.tiles_vs(N, V, S, 64, 32))
    tiles = C.tiles_vs(N, V, runs_of(S, N))
    assert np.all(steps <= 2 * tiles) and steps.sum() < 2 * tiles.sum()


def test_vs_tiles_edge_cases():
    N = 1024
    assert np.array_equal(C.tiles_vs(N, [], runs_of(np.array([0]), N)), O.tiles_vs(N, [], [0]))
    assert np.array_equal(C.tiles_vs(N, [5, 700], np.zeros((0, 2))), O.tiles_vs(N, [5, 700], []))
    # every slash kept: dense
    assert np.array_equal(C.tiles_vs(N, [3], runs_of(np.arange(N), N)), C.tiles_dense(N))


def test_bs_speedup_closed_form():
    # App. C.4.1: speedup over dense ~ S / (2 B k_b) once the sequence is long
    N, kb = 131072, 100
    NB = N // 64
    cnt = np.minimum(kb, np.arange(1, NB + 1))
    ratio = C.tiles_dense(N).sum() / C.tiles_bs(cnt).sum()
    assert abs(ratio - N / (2 * 64 * kb)) / ratio < 0.03


def block_sums(mask_rows):
    return mask_rows.sum(axis=1).reshape(-1, 64).sum(axis=1)


def test_permitted_pair_counts_match_the_oracle_masks(rng=np.random.default_rng(5)):
    """The useful-work counters against explicit masks of the oracle on a short sequence."""
    N = 1024
    NB = N // 64
    assert np.array_equal(C.nnz_dense(N), block_sums(O.causal_rows(0, N, N)))
    for n_init, n_local in [(64, 128), (100, 200), (0, 65), (5, 1), (2000, 3)]:
        assert np.array_equal(C.nnz_ashape(N, n_init, n_local), block_sums(O.ashape_rows(0, N, N, n_init, n_local)))
    idx = -np.ones((NB, 5), np.int64)
    cnt = np.zeros(NB, np.int64)
    for b in range(NB):
        c = min(5, b + 1)
        idx[b, :c], cnt[b] = np.sort(rng.choice(b + 1, c, replace=False)), c
    assert np.array_equal(C.nnz_bs(idx, cnt), block_sums(O.bs_rows(0, N, N, idx, cnt)))
    for V, S in [([3, 70, 71, 300, 1023], [0, 5, 64, 200, 201, 450]), ([], [0]), ([5], list(range(N))),
                 (list(range(0, N, 37)), [0, 1, 2, 3, 130, 131, 400, 1000]), ([600, 601], [500])]:
        want = block_sums(O.vs_rows(0, N, N, np.asarray(V, dtype=np.int64), np.asarray(S, dtype=np.int64), 64))
        assert np.array_equal(C.nnz_vs(N, V, runs_of(np.asarray(S, dtype=np.int64), N)), want), (V[:3], S[:3])
