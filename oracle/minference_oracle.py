"""CPU oracle for dynamic sparse prefill attention (MInference 1.0, arXiv 2407.02490).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP library is checked against.  Nothing in the product path may import it;
only tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares
no code, tables or helpers with the GPU path and never receives a value
computed by it.

Everything is numpy in float64 on the (bf16-representable) input values.
Library primitives used as steps: matmul, exp, sort.  No blocking, fusion or
reordering beyond what the definitions state.

Conventions (paper notation): S = N sequence length, d head dimension,
B block size (64), tau = 1/sqrt(d), i query position, j key position,
delta = i - j the diagonal ("slash") offset.  A mask M[i, j] in {0,1} says
whether query i may attend key j.  Every mask is causal (j <= i).

Readings of the paper where it is silent or ambiguous (listed with reasons in
the design document):
  * Eq. 1 uses a finite constant c; here c -> infinity (masked logits are -inf).
  * A row with no permitted key yields a zero output row.
  * Top-k is exact, ties go to the lower index; k is clamped to the number of
    candidates.
  * The Vertical-Slash mask computed by the kernels (App. C.4.2, Alg. 4/5) is a
    mix of B x B slash tiles and single columns.  For the query block that
    holds row i (rows bB .. bB+B-1), slash offset o permits the key range
    [bB - o, bB - o + B) (the tile whose main diagonal is the slash); a
    vertical v permits key v.  The parameter Bm selects the tile size; Bm = 1
    gives the exact lines.
  * Block-Sparse top-k is taken per query-block row (App. C.4.1).
  * A-shape is element exact: key j is permitted iff j < n_init or
    i - j < n_local (Section 4, implementation details: 1k global + 4k local).

Pins: every function here is pinned by tests/test_oracle_*.py (closed forms,
brute force on tiny inputs, invariants, planted structure, special cases that
reduce to dense attention).  The paper prints no numeric example of an index
or an output, so parity with the authors' own implementation is unpinned.
"""
import numpy as np

__all__ = [
    "attend", "causal_rows", "ashape_rows", "vs_rows", "bs_rows",
    "topk_indices", "vs_estimate", "vs_line_scores", "vs_index",
    "slash_cover", "bs_pool", "bs_scores", "bs_index",
    "dense_attention", "ashape_attention", "vs_attention", "bs_attention",
    "tiles_dense", "tiles_ashape", "tiles_bs", "tiles_vs",
]


# --------------------------------------------------------------------------
# Eq. 1: masked softmax attention
# --------------------------------------------------------------------------
def attend(q, K, V, mask, scale=None, return_p=False):
    """Eq. 1 with c -> infinity, for a set of query rows.

    q [R, d], K [N, d], V [N, d] float64; mask [R, N] bool.
    Returns O [R, d] (and P [R, N] if return_p).  Rows whose mask is empty
    give zeros.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    mask = np.asarray(mask, dtype=bool)
    d = q.shape[1]
    tau = 1.0 / np.sqrt(d) if scale is None else float(scale)
    # Keys that no row of this call may attend contribute exactly zero;
    # leaving them out of the matmul changes nothing but the run time.
    used = np.flatnonzero(mask.any(axis=0))
    if return_p or used.size * 2 > K.shape[0]:
        used = np.arange(K.shape[0])
    Ks, Vs, Ms = K[used], V[used], mask[:, used]
    logits = (q @ Ks.T) * tau
    logits = np.where(Ms, logits, -np.inf)
    m = logits.max(axis=1, keepdims=True) if used.size else np.zeros((q.shape[0], 1))
    m = np.where(np.isfinite(m), m, 0.0)
    E = np.where(Ms, np.exp(logits - m), 0.0)
    l = E.sum(axis=1, keepdims=True)
    P = np.divide(E, l, out=np.zeros_like(E), where=l > 0)
    O = P @ Vs
    if return_p:
        return O, P
    return O


# --------------------------------------------------------------------------
# Masks, produced for a range of query rows [i0, i1)
# --------------------------------------------------------------------------
def causal_rows(i0, i1, N):
    """Dense causal mask rows: j <= i."""
    i = np.arange(i0, i1)[:, None]
    j = np.arange(N)[None, :]
    return j <= i


def ashape_rows(i0, i1, N, n_init, n_local):
    """A-shape (Section 2.2 / Section 4): initial tokens plus a local window."""
    i = np.arange(i0, i1)[:, None]
    j = np.arange(N)[None, :]
    return (j <= i) & ((j < n_init) | (i - j < n_local))


def slash_cover(S_idx, N, Bm):
    """cover[t + Bm] for t in [-Bm, N): True iff some o in S has t <= o < t+Bm.

    t = (first row of the query block) - j.  This is the offset-space image of
    "slash o covers the Bm x Bm tile whose main diagonal it is" (App. C.4.2).
    """
    S_idx = np.asarray(S_idx, dtype=np.int64)
    has = np.zeros(N + 2 * Bm + 1, dtype=np.int64)      # has[x + Bm] = [x in S]
    has[S_idx + Bm] = 1
    cnt = np.concatenate([[0], np.cumsum(has)])          # cnt[x + Bm] = #{o in S : o < x}
    t = np.arange(-Bm, N)
    return (cnt[t + Bm + Bm] - cnt[t + Bm]) > 0


def vs_rows(i0, i1, N, V_idx, S_idx, Bm=64):
    """Vertical-Slash mask rows (Alg. 2 step 'sparseformat', App. C.4.2).

    j permitted iff j <= i and ( j in V  or  exists o in S with
    t <= o < t + Bm, t = (i - i mod Bm) - j ).
    """
    i = np.arange(i0, i1)[:, None]
    j = np.arange(N)[None, :]
    vert = np.zeros(N, dtype=bool)
    vert[np.asarray(V_idx, dtype=np.int64)] = True
    cover = slash_cover(S_idx, N, Bm)
    t = (i - i % Bm) - j                                  # > -Bm wherever j <= i
    t_c = np.clip(t, -Bm, N - 1)
    return (j <= i) & (vert[None, :] | cover[t_c + Bm])


def bs_rows(i0, i1, N, blk_idx, blk_cnt, B=64):
    """Block-Sparse mask rows (Alg. 3): key block of j is among the blocks kept
    for the query block of i; causal inside the diagonal block."""
    NB = N // B
    keep = np.zeros((NB, NB), dtype=bool)
    for b in range(NB):
        keep[b, np.asarray(blk_idx[b][: int(blk_cnt[b])], dtype=np.int64)] = True
    i = np.arange(i0, i1)
    j = np.arange(N)
    return (j[None, :] <= i[:, None]) & keep[(i // B)[:, None], (j // B)[None, :]]


# --------------------------------------------------------------------------
# Exact top-k
# --------------------------------------------------------------------------
def topk_indices(scores, k):
    """Indices of the k largest scores, ties to the lower index, returned
    ascending.  Full sort on (-score, index)."""
    scores = np.asarray(scores, dtype=np.float64)
    k = int(min(k, scores.shape[0]))
    order = np.lexsort((np.arange(scores.shape[0]), -scores))
    return np.sort(order[:k])


# --------------------------------------------------------------------------
# Alg. 2: Vertical-Slash index
# --------------------------------------------------------------------------
def vs_estimate(Q, K, last_q=64, scale=None):
    """A_hat = softmax(Q[-last_q:] K^T / sqrt(d) + causal) (Alg. 2, first step).
    Returns A_hat [R, N] with R = min(last_q, N); row r is query N - R + r."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    N, d = K.shape
    R = min(int(last_q), N)
    tau = 1.0 / np.sqrt(d) if scale is None else float(scale)
    logits = (Q[N - R:] @ K.T) * tau
    p = (N - R + np.arange(R))[:, None]
    logits = np.where(np.arange(N)[None, :] <= p, logits, -np.inf)
    logits = logits - logits.max(axis=1, keepdims=True)
    E = np.exp(logits)
    return E / E.sum(axis=1, keepdims=True)


def vs_line_scores(A_hat):
    """Column sums ("sum in vertical") and diagonal sums ("sum in slash") of
    A_hat (Alg. 2).  diagsum[o] adds A_hat[r, p_r - o] over the rows whose
    diagonal o exists (p_r >= o), p_r = N - R + r."""
    R, N = A_hat.shape
    colsum = A_hat.sum(axis=0)
    diagsum = np.zeros(N, dtype=np.float64)
    for r in range(R):
        p = N - R + r
        diagsum[p - np.arange(p + 1)] += A_hat[r, : p + 1]
    return colsum, diagsum


def vs_index(Q, K, last_q, nv, ns, scale=None):
    """Alg. 2: vertical index i_v (key positions) and slash index i_s (offsets),
    both ascending.  Also returns the two score vectors."""
    A_hat = vs_estimate(Q, K, last_q, scale)
    colsum, diagsum = vs_line_scores(A_hat)
    N = K.shape[0]
    return (topk_indices(colsum, min(nv, N)), topk_indices(diagsum, min(ns, N)),
            colsum, diagsum)


# --------------------------------------------------------------------------
# Alg. 3: Block-Sparse index
# --------------------------------------------------------------------------
def bs_pool(X, B=64):
    """MeanPooling(X, block_size) (Alg. 3)."""
    X = np.asarray(X, dtype=np.float64)
    N, d = X.shape
    return X.reshape(N // B, B, d).mean(axis=1)


def bs_scores(Q, K, B=64, scale=None):
    """Block logits Q_hat K_hat^T / sqrt(d) with the block-causal mask
    (Alg. 3).  Softmax is monotone per row, so top-k of these logits equals
    top-k of A_hat."""
    d = np.asarray(Q).shape[1]
    tau = 1.0 / np.sqrt(d) if scale is None else float(scale)
    Qp, Kp = bs_pool(Q, B), bs_pool(K, B)
    s = (Qp @ Kp.T) * tau
    NB = s.shape[0]
    return np.where(np.arange(NB)[None, :] <= np.arange(NB)[:, None], s, -np.inf)


def bs_index(Q, K, B=64, topk=100, scale=None):
    """Alg. 3: for every query block b the min(topk, b+1) key blocks with the
    largest block logit.  Returns (idx [NB, topk] ascending, padded with -1;
    cnt [NB]; scores [NB, NB])."""
    s = bs_scores(Q, K, B, scale)
    NB = s.shape[0]
    idx = -np.ones((NB, topk), dtype=np.int64)
    cnt = np.zeros(NB, dtype=np.int64)
    for b in range(NB):
        sel = topk_indices(s[b, : b + 1], topk)
        cnt[b] = sel.size
        idx[b, : sel.size] = sel
    return idx, cnt, s


# --------------------------------------------------------------------------
# Whole-head attention for the four masks, rows [i0, i1)
# --------------------------------------------------------------------------
def _rows(i0, i1, N):
    return (0 if i0 is None else i0), (N if i1 is None else i1)


def dense_attention(Q, K, V, i0=None, i1=None, scale=None):
    N = K.shape[0]
    i0, i1 = _rows(i0, i1, N)
    return attend(Q[i0:i1], K, V, causal_rows(i0, i1, N), scale)


def ashape_attention(Q, K, V, n_init, n_local, i0=None, i1=None, scale=None):
    N = K.shape[0]
    i0, i1 = _rows(i0, i1, N)
    return attend(Q[i0:i1], K, V, ashape_rows(i0, i1, N, n_init, n_local), scale)


def vs_attention(Q, K, V, V_idx, S_idx, i0=None, i1=None, Bm=64, scale=None):
    N = K.shape[0]
    i0, i1 = _rows(i0, i1, N)
    return attend(Q[i0:i1], K, V, vs_rows(i0, i1, N, V_idx, S_idx, Bm), scale)


def bs_attention(Q, K, V, blk_idx, blk_cnt, i0=None, i1=None, B=64, scale=None):
    N = K.shape[0]
    i0, i1 = _rows(i0, i1, N)
    return attend(Q[i0:i1], K, V, bs_rows(i0, i1, N, blk_idx, blk_cnt, B), scale)


# --------------------------------------------------------------------------
# Tile counts of the masks ("FLOPs in kernel", Alg. 1; App. C.4: latency is
# linear in the number of blocks / the area of blocks and columns).
# One tile = B query rows x B keys.  Per query block b:
# --------------------------------------------------------------------------
def tiles_dense(N, B=64):
    return np.arange(1, N // B + 1, dtype=np.int64)


def tiles_ashape(N, n_init, n_local, B=64, blocks=None):
    """Number of B-aligned key tiles that hold at least one permitted key, per query block
    (all of them, or only the listed ones: a long sequence has too many to mask one by one)."""
    NB = N // B
    blocks = range(NB) if blocks is None else blocks
    out = np.zeros(len(blocks), dtype=np.int64)
    for n, b in enumerate(blocks):
        m = ashape_rows(b * B, (b + 1) * B, N, n_init, n_local).any(axis=0)
        out[n] = m.reshape(NB, B).any(axis=1).sum()
    return out


def tiles_bs(blk_cnt):
    return np.asarray(blk_cnt, dtype=np.int64).copy()


def tiles_vs(N, V_idx, S_idx, B=64, W=None):
    """Slash part: the cover of block b, as maximal runs of permitted keys in
    [0, bB + B), costs ceil(len / B) tiles per run.  Column part: causal
    verticals (v < bB + B) outside that cover, B per gathered tile.
    With W given the unit is a step of B query rows x W keys instead of a
    B x B tile (a kernel that walks runs W keys at a time computes
    ceil(len / W) steps per run, which is less work than ceil(len / B) tiles
    whenever len mod B is in 1 .. B - W)."""
    NB = N // B
    W = B if W is None else W
    cover = slash_cover(S_idx, N, B)
    V_idx = np.asarray(V_idx, dtype=np.int64)
    out = np.zeros(NB, dtype=np.int64)
    for b in range(NB):
        j = np.arange(0, min(N, b * B + B))
        t = b * B - j
        c = cover[np.clip(t, -B, N - 1) + B]
        edges = np.diff(np.concatenate([[0], c.astype(np.int8), [0]]))
        starts, ends = np.flatnonzero(edges == 1), np.flatnonzero(edges == -1)
        n_slash = int(np.sum(-(-(ends - starts) // W)))
        v = V_idx[V_idx < b * B + B]
        free = int(np.sum(~c[v])) if v.size else 0
        out[b] = n_slash + -(-free // W)
    return out
