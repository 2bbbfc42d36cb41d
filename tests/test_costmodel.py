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
