"""Pins for the oracle's index builders and the Vertical-Slash / Block-Sparse
masks (CPU only): brute force on tiny inputs, invariants, planted structure,
special cases that reduce to dense attention, closed-form counts."""
import math

import numpy as np
import pytest

from oracle import minference_oracle as O


# ------------------------------------------------------------ exact top-k
def test_topk_bruteforce_and_tie_rule():
    s = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.5, 3.0])
    # sorted by (-score, index): 6, 1, 2, 4, 0, 5, 3
    assert list(O.topk_indices(s, 1)) == [6]
    assert list(O.topk_indices(s, 3)) == [1, 2, 6]
    assert list(O.topk_indices(s, 5)) == [0, 1, 2, 4, 6]
    assert list(O.topk_indices(s, 99)) == list(range(7))


def test_topk_random_against_python_sort(rng):
    for _ in range(20):
        n = int(rng.integers(1, 60))
        s = rng.integers(0, 8, size=n).astype(float)      # many ties
        k = int(rng.integers(1, n + 1))
        want = sorted(sorted(range(n), key=lambda i: (-s[i], i))[:k])
        assert list(O.topk_indices(s, k)) == want


# --------------------------------------------------- Alg. 2: VS estimate
def brute_vs_scores(Q, K, last_q, tau=None):
    """Explicit loops over (r, j): softmax rows of the last queries, column
    sums and diagonal sums."""
    N, d = K.shape
    R = min(last_q, N)
    tau = 1.0 / math.sqrt(d) if tau is None else tau
    A = np.zeros((R, N))
    for r in range(R):
        p = N - R + r
        logits = [sum(Q[p, c] * K[j, c] for c in range(d)) * tau for j in range(p + 1)]
        mx = max(logits)
        e = [math.exp(x - mx) for x in logits]
        z = sum(e)
        for j in range(p + 1):
            A[r, j] = e[j] / z
    col = np.zeros(N)
    diag = np.zeros(N)
    for r in range(R):
        p = N - R + r
        for j in range(p + 1):
            col[j] += A[r, j]
            diag[p - j] += A[r, j]
    return A, col, diag


@pytest.mark.parametrize("N,last_q", [(48, 8), (20, 5), (6, 8)])
def test_vs_scores_bruteforce(rng, N, last_q):
    d = 8
    Q, K = rng.normal(size=(2, N, d))
    A, col, diag = brute_vs_scores(Q, K, last_q)
    A2 = O.vs_estimate(Q, K, last_q)
    col2, diag2 = O.vs_line_scores(A2)
    assert np.allclose(A, A2, atol=1e-14)
    assert np.allclose(col, col2, atol=1e-14)
    assert np.allclose(diag, diag2, atol=1e-14)
    nv, ns = 5, 7
    V, S, _, _ = O.vs_index(Q, K, last_q, nv, ns)
    wantV = sorted(sorted(range(N), key=lambda j: (-col[j], j))[:min(nv, N)])
    wantS = sorted(sorted(range(N), key=lambda o: (-diag[o], o))[:min(ns, N)])
    assert list(V) == wantV and list(S) == wantS


def test_vs_scores_bruteforce_with_a_scale_other_than_the_default(rng):
    """The scale argument multiplies the logits before the softmax (Eq. 1's 1/sqrt(d) replaced):
    a sharper softmax changes the line scores and the kept lines."""
    N, d, last_q, tau = 40, 8, 6, 0.9
    Q, K = rng.normal(size=(2, N, d))
    A, col, diag = brute_vs_scores(Q, K, last_q, tau)
    A2 = O.vs_estimate(Q, K, last_q, scale=tau)
    col2, diag2 = O.vs_line_scores(A2)
    assert np.allclose(A, A2, atol=1e-14) and np.allclose(col, col2, atol=1e-14) and np.allclose(diag, diag2, atol=1e-14)
    assert not np.allclose(A2, O.vs_estimate(Q, K, last_q), atol=1e-3)        # the argument is not ignored
    V, S, c3, d3 = O.vs_index(Q, K, last_q, 4, 6, scale=tau)
    assert np.allclose(c3, col, atol=1e-14) and np.allclose(d3, diag, atol=1e-14)
    assert list(V) == sorted(sorted(range(N), key=lambda j: (-col[j], j))[:4])
    assert list(S) == sorted(sorted(range(N), key=lambda o: (-diag[o], o))[:6])


def test_vs_scores_mass_invariant(rng):
    N, d, R = 256, 16, 64
    Q, K = rng.normal(size=(2, N, d))
    col, diag = O.vs_line_scores(O.vs_estimate(Q, K, R))
    assert abs(col.sum() - R) < 1e-10
    assert abs(diag.sum() - R) < 1e-10
    # offsets that no estimating row reaches carry nothing: o > p_r for all r
    assert np.all(diag >= 0) and np.all(col >= 0)


def test_vs_estimate_is_causal_in_the_corner(rng):
    N, d, R = 64, 8, 16
    Q, K = rng.normal(size=(2, N, d))
    A = O.vs_estimate(Q, K, R)
    for r in range(R):
        assert np.all(A[r, N - R + r + 1:] == 0)


def test_vs_planted_vertical(rng):
    N, d, R = 512, 32, 64
    Q, K = rng.normal(size=(2, N, d))
    u = rng.normal(size=d)
    Q[N - R:] += 2.0 * u            # the estimating queries share a direction
    K[100] += 2.0 * u               # ... and key 100 is aligned with it
    V, S, col, diag = O.vs_index(Q, K, R, 1, 1)
    assert list(V) == [100]


def test_vs_planted_slash(rng):
    N, d, R = 512, 32, 64
    Q, K = rng.normal(size=(2, N, d))
    for i in range(N - R, N):       # k_{i-37} aligned with q_i: diagonal offset 37
        K[i - 37] += 0.8 * Q[i]
    V, S, col, diag = O.vs_index(Q, K, R, 1, 3)
    assert 37 in S
    assert diag[37] == diag.max()


def test_vs_k_equals_n_returns_everything(rng):
    N, d = 40, 8
    Q, K = rng.normal(size=(2, N, d))
    V, S, _, _ = O.vs_index(Q, K, 8, N + 5, N)
    assert list(V) == list(range(N)) and list(S) == list(range(N))


# ------------------------------------------------------ VS mask (tiles)
def test_vs_mask_bm1_is_exact_lines(rng):
    N = 70
    V = np.sort(rng.choice(N, 6, replace=False))
    S = np.sort(rng.choice(N, 9, replace=False))
    m = O.vs_rows(0, N, N, V, S, Bm=1)
    for i in range(N):
        for j in range(N):
            want = j <= i and (j in V or (i - j) in S)
            assert m[i, j] == want


def brute_vs_tile_mask(N, V, S, B):
    """Per query block, per slash: permit the B keys starting at bB - o."""
    m = np.zeros((N, N), dtype=bool)
    for b in range(N // B):
        rows = range(b * B, b * B + B)
        for o in S:
            for j in range(b * B - o, b * B - o + B):
                if 0 <= j < N:
                    for i in rows:
                        m[i, j] = True
        for v in V:
            for i in rows:
                m[i, v] = True
    for i in range(N):
        m[i, i + 1:] = False
    return m


@pytest.mark.parametrize("B", [4, 8])
def test_vs_mask_tile_bruteforce_and_containment(rng, B):
    N = 64
    V = np.sort(rng.choice(N, 5, replace=False))
    S = np.sort(rng.choice(N, 7, replace=False))
    m = O.vs_rows(0, N, N, V, S, Bm=B)
    assert np.array_equal(m, brute_vs_tile_mask(N, V, S, B))
    exact = O.vs_rows(0, N, N, V, S, Bm=1)
    assert np.all(m[exact])                     # exact lines are inside the tile cover
    assert np.array_equal(O.vs_rows(16, 40, N, V, S, Bm=B), m[16:40])


def test_vs_cover_translation_property(rng):
    # merging the per-block key ranges [bB - o, bB - o + B) block by block gives
    # the same key set as shifting one offset-space cover by bB
    N, B = 96, 8
    S = np.sort(rng.choice(N, 11, replace=False))
    cover = O.slash_cover(S, N, B)              # indexed by t + B, t in [-B, N)
    for b in range(N // B):
        keys = set()
        for o in S:
            keys.update(range(b * B - o, b * B - o + B))
        shifted = {b * B - t for t in range(-B, N) if cover[t + B]}
        assert keys == shifted


def test_vs_full_index_is_dense(rng):
    N, d = 64, 8
    Q, K, V = rng.normal(size=(3, N, d))
    dense = O.dense_attention(Q, K, V)
    allidx = np.arange(N)
    assert np.allclose(O.vs_attention(Q, K, V, [], allidx, Bm=8), dense, atol=1e-13)
    assert np.allclose(O.vs_attention(Q, K, V, allidx, [], Bm=8), dense, atol=1e-13)
    assert np.allclose(O.vs_attention(Q, K, V, allidx, allidx, Bm=1), dense, atol=1e-13)


def test_vs_contiguous_slashes_give_band_with_closed_form_count():
    # S = {0..w-1}, no verticals, tile size B: row i (r = i mod B) sees offsets
    # delta in [0, w - 1 + r] -> min(i, w - 1 + r) + 1 keys
    N, B, w = 96, 8, 13
    m = O.vs_rows(0, N, N, [], np.arange(w), Bm=B)
    for i in range(N):
        r = i % B
        assert m[i].sum() == min(i, w - 1 + r) + 1
        assert m[i, max(0, i - (w - 1 + r)): i + 1].all()


def test_vs_double_membership_counts_once(rng):
    # a vertical inside a slash tile must not be weighted twice: P rows sum to 1
    # and equal the set-union mask result
    N, d, B = 64, 8, 8
    Q, K, V = rng.normal(size=(3, N, d))
    Vi, Si = np.array([10, 11, 30]), np.array([0, 3, 20])
    m = O.vs_rows(0, N, N, Vi, Si, Bm=B)
    out, P = O.attend(Q, K, V, m, return_p=True)
    assert np.allclose(P[m.any(axis=1)].sum(axis=1), 1.0)
    assert np.allclose(out, O.vs_attention(Q, K, V, Vi, Si, Bm=B))


def test_vs_empty_rows_when_nothing_selected():
    N, B = 32, 8
    m = O.vs_rows(0, N, N, [20], [9], Bm=B)
    # block 0 (rows 0..7): slash 9 maps to keys [-9, -1) -> nothing; vertical 20 not causal
    assert not m[:8].any()


def test_tiles_vs_bruteforce_per_block_also_in_narrower_key_steps(rng):
    """tiles_vs against sets built slash by slash for every block (pure python), in B x B tiles
    and in B x W steps (W < B: the unit of a kernel that walks a run W keys at a time)."""
    N, B = 96, 8
    for trial in range(6):
        S = sorted(rng.choice(N, int(rng.integers(1, 12)), replace=False).tolist())
        V = sorted(rng.choice(N, int(rng.integers(0, 20)), replace=False).tolist())
        for W in (8, 4, 2):
            want = []
            for b in range(N // B):
                keys = set()
                for o in S:
                    keys |= {j for j in range(b * B - o, b * B - o + B) if 0 <= j < b * B + B}
                n, j = 0, 0
                while j < b * B + B:                       # maximal runs of covered keys
                    if j in keys:
                        e = j
                        while e in keys:
                            e += 1
                        n += -(-(e - j) // W)
                        j = e
                    else:
                        j += 1
                free = sum(1 for v in V if v < b * B + B and v not in keys)
                want.append(n + -(-free // W))
            got = O.tiles_vs(N, V, S, B, W) if W != B else O.tiles_vs(N, V, S, B)
            assert list(got) == want, (trial, W)


def test_tiles_vs_bounds_and_closed_form(rng):
    N, B = 256, 16
    # contiguous slashes 0..w-1: cover (-B, w-1] in offsets -> one run of
    # min(bB + B, w + B - 1) keys per block
    w = 40
    t = O.tiles_vs(N, [], np.arange(w), B)
    for b in range(N // B):
        run = min(b * B + B, w + B - 1)
        assert t[b] == -(-run // B)
    # isolated slashes, far apart: one tile each once causal; verticals add ceil(n/B)
    S = np.array([0, 64, 160])
    Vv = np.arange(0, 200, 8)          # 25 verticals
    t = O.tiles_vs(N, Vv, S, B)
    m = O.vs_rows(0, N, N, Vv, S, Bm=B)
    for b in range(N // B):
        area = m[b * B:(b + 1) * B].any(axis=0).sum()
        assert t[b] * B >= area                   # tiles hold every permitted key
    assert t[-1] == 3 + -(-int(np.sum(~O.slash_cover(S, N, B)[np.clip((N - B) - Vv, -B, N - 1) + B])) // B)


# --------------------------------------------------------- Alg. 3: BS
def brute_bs_index(Q, K, B, k):
    N, d = Q.shape
    NB = N // B
    Qp = [[sum(Q[b * B + t, c] for t in range(B)) / B for c in range(d)] for b in range(NB)]
    Kp = [[sum(K[b * B + t, c] for t in range(B)) / B for c in range(d)] for b in range(NB)]
    out = []
    for b in range(NB):
        sc = [sum(Qp[b][c] * Kp[cb][c] for c in range(d)) / math.sqrt(d) for cb in range(b + 1)]
        out.append(sorted(sorted(range(b + 1), key=lambda cb: (-sc[cb], cb))[:k]))
    return out


def test_bs_index_bruteforce(rng):
    N, d, B, k = 48, 8, 4, 3
    Q, K = rng.normal(size=(2, N, d))
    idx, cnt, s = O.bs_index(Q, K, B, k)
    want = brute_bs_index(Q, K, B, k)
    for b in range(N // B):
        assert cnt[b] == min(k, b + 1)
        assert list(idx[b, :cnt[b]]) == want[b]
        assert np.all(idx[b, cnt[b]:] == -1)


def test_bs_scores_with_a_scale_other_than_the_default(rng):
    """Block logits are tau * <Q_hat_b, K_hat_c>: explicit loops with tau = 0.37."""
    N, d, B, tau = 96, 6, 8, 0.37
    Q, K = rng.normal(size=(2, N, d))
    NB = N // B
    s = O.bs_scores(Q, K, B, scale=tau)
    for b in range(NB):
        for c in range(NB):
            if c > b:
                assert s[b, c] == -np.inf
                continue
            qb = [sum(Q[b * B + t, x] for t in range(B)) / B for x in range(d)]
            kc = [sum(K[c * B + t, x] for t in range(B)) / B for x in range(d)]
            assert abs(s[b, c] - tau * sum(qb[x] * kc[x] for x in range(d))) < 1e-13
    idx, cnt, s2 = O.bs_index(Q, K, B, 3, scale=tau)
    assert np.array_equal(s, s2)
    # a positive scale does not change the selection (Alg. 3 keeps the largest logits per row)
    idx0, cnt0, _ = O.bs_index(Q, K, B, 3)
    assert np.array_equal(idx, idx0) and np.array_equal(cnt, cnt0)


def test_bs_tile_count_is_the_number_of_tiles_the_mask_touches(rng):
    """tiles_bs against the explicit mask: per query block, the number of B x B tiles of the
    Block-Sparse mask that hold a permitted (query, key) pair."""
    N, B, k = 160, 8, 4
    NB = N // B
    idx = -np.ones((NB, k), dtype=np.int64)
    cnt = np.zeros(NB, dtype=np.int64)
    for b in range(NB):
        c = int(rng.integers(1, min(k, b + 1) + 1))
        idx[b, :c] = np.sort(rng.choice(b + 1, c, replace=False))
        cnt[b] = c
    M = O.bs_rows(0, N, N, idx, cnt, B)
    touched = M.reshape(NB, B, NB, B).any(axis=(1, 3)).sum(axis=1)
    assert np.array_equal(O.tiles_bs(cnt), touched)


def test_bs_selection_on_logits_equals_selection_on_softmax(rng):
    N, d, B, k = 128, 16, 8, 4
    Q, K = rng.normal(size=(2, N, d))
    idx, cnt, s = O.bs_index(Q, K, B, k)
    NB = N // B
    for b in range(NB):
        row = s[b, :b + 1]
        p = np.exp(row - row.max())
        p /= p.sum()
        assert list(O.topk_indices(p, k)) == list(idx[b, :cnt[b]])


def test_bs_planted_centroids(rng):
    N, d, B = 256, 32, 16
    NB = N // B
    cent = np.eye(d)[:4] * 10.0
    assign = rng.integers(0, 4, size=NB)
    Q = rng.normal(size=(N, d)) * 0.1 + np.repeat(cent[assign], B, axis=0)
    K = rng.normal(size=(N, d)) * 0.1 + np.repeat(cent[assign], B, axis=0)
    k = 3
    idx, cnt, _ = O.bs_index(Q, K, B, k)
    for b in range(NB):
        same = [c for c in range(b + 1) if assign[c] == assign[b]]
        got = set(idx[b, :cnt[b]])
        if len(same) >= cnt[b]:
            assert got <= set(same)
        else:
            assert set(same) <= got


def test_bs_mask_dense_limit_and_nnz(rng):
    N, d, B = 64, 8, 8
    NB = N // B
    Q, K, V = rng.normal(size=(3, N, d))
    idx, cnt, _ = O.bs_index(Q, K, B, NB)
    assert np.allclose(O.bs_attention(Q, K, V, idx, cnt, B=B), O.dense_attention(Q, K, V), atol=1e-13)
    idx, cnt, _ = O.bs_index(Q, K, B, 3)
    m = O.bs_rows(0, N, N, idx, cnt, B)
    want = 0
    for b in range(NB):
        has_diag = b in idx[b, :cnt[b]]
        want += cnt[b] * B * B - (B * (B - 1) // 2 if has_diag else 0)
    assert m.sum() == want
    assert np.array_equal(O.bs_rows(8, 24, N, idx, cnt, B), m[8:24])
    assert np.array_equal(O.tiles_bs(cnt), np.minimum(3, np.arange(1, NB + 1)))


def test_bs_mask_bruteforce(rng):
    N, B = 32, 4
    NB = N // B
    idx = -np.ones((NB, 2), dtype=np.int64)
    cnt = np.zeros(NB, dtype=np.int64)
    for b in range(NB):
        sel = np.sort(rng.choice(b + 1, min(2, b + 1), replace=False))
        idx[b, :sel.size] = sel
        cnt[b] = sel.size
    m = O.bs_rows(0, N, N, idx, cnt, B)
    for i in range(N):
        for j in range(N):
            want = j <= i and (j // B) in set(idx[i // B, :cnt[i // B]])
            assert m[i, j] == want
