"""Kernel-aware cost of a set of sparse indices (host logic, numpy).

The paper's pattern search compares candidates by the FLOPs the kernels
really spend (Alg. 1, "FLOPs_in_kernel"), and its kernels' latency is linear in
the number of 64 x 64 blocks / the area of blocks and columns (App. C.4).
This module counts those tiles from the index buffers the library produces or
consumes.  One tile = 64 query rows x 64 keys = 4 * 64 * 64 * d FLOP
(QK^T and PV, multiply + add).

Tile decomposition per 64-row query block b (independent of how a kernel
schedules the work):
  dense        b + 1
  A-shape      64-aligned key tiles holding at least one permitted key
  Block-Sparse number of kept blocks
  Vertical-Slash  sum over slash runs clipped to keys [0, 64b + 64) of
               ceil(len / 64), plus ceil(n_free / 64) where n_free counts the
               kept verticals v < 64b + 64 that lie outside every run
"""
import numpy as np

BLOCK = 64


def tile_flops(d=128, block=BLOCK):
    return 4 * block * block * d


def tiles_dense(N):
    return np.arange(1, N // BLOCK + 1, dtype=np.int64)


def tiles_ashape(N, n_init, n_local):
    NB = N // BLOCK
    b = np.arange(NB, dtype=np.int64)
    n_init, n_local = min(n_init, N), min(n_local, N)
    sink = np.minimum(-(-n_init // BLOCK), b + 1)            # tiles [0, sink)
    w = np.maximum(BLOCK * b - n_local + 1, 0) // BLOCK      # first window tile
    first = np.maximum(w, sink)
    return sink + np.maximum(b - first + 1, 0)


def tiles_bs(blk_cnt):
    return np.asarray(blk_cnt, dtype=np.int64).copy()


STEP = 32     # keys per step of the Vertical-Slash kernel (one step = 64 query rows x 32 keys)


def tiles_vs(N, v_idx, runs, width=BLOCK):
    """v_idx: ascending kept verticals; runs: [n, 2] offset runs [t0, t1).
    width = 64: the canonical 64 x 64 tile count of the index.  width = 32: the 64 x 32 steps
    the kernel executes (it walks a run 32 keys at a time from the run's first key and gathers
    verticals 32 at a time), which is what its FLOP rate is computed from: a run of length len
    costs ceil(len / 32) steps, less than ceil(len / 64) tiles when len mod 64 is in 1 .. 32."""
    NB = N // BLOCK
    q0 = BLOCK * np.arange(NB, dtype=np.int64)[:, None]
    runs = np.asarray(runs, dtype=np.int64).reshape(-1, 2)
    v = np.asarray(v_idx, dtype=np.int64)
    out = np.zeros(NB, dtype=np.int64)
    if runs.size:
        ks = np.maximum(q0 - runs[None, :, 1] + 1, 0)
        ke = np.minimum(q0 - runs[None, :, 0] + 1, N)
        ln = np.maximum(ke - ks, 0)
        out += (-(-ln // width)).sum(axis=1)
    if v.size:
        for lo in range(0, NB, 1024):                       # bounded memory at 1M tokens
            hi = min(NB, lo + 1024)
            t = q0[lo:hi] - v[None, :]                        # offset of vertical v for block b
            causal = v[None, :] < q0[lo:hi] + BLOCK
            if runs.size:
                j = np.searchsorted(runs[:, 0], t, side="right") - 1
                inside = (j >= 0) & (t < runs[np.maximum(j, 0), 1])
            else:
                inside = np.zeros_like(causal)
            free = (causal & ~inside).sum(axis=1)
            out[lo:hi] += -(-free // width)
    return out


# ---------------------------------------------------------------------------
# Permitted (query, key) pairs per query block: the "useful" work, 4 * d FLOP per
# pair, as opposed to the tile count above, which also pays for the masked part
# of every tile a kernel has to touch.
# ---------------------------------------------------------------------------
def nnz_dense(N):
    q0 = BLOCK * np.arange(N // BLOCK, dtype=np.int64)
    return BLOCK * q0 + BLOCK * (BLOCK + 1) // 2


def nnz_ashape(N, n_init, n_local):
    i = np.arange(N, dtype=np.int64)
    n_init, n_local = min(n_init, N), min(n_local, N)
    sink = np.minimum(i + 1, n_init)
    win_lo = np.maximum(np.maximum(i - n_local + 1, n_init), 0)
    win = np.maximum(i - win_lo + 1, 0)
    return (sink + win).reshape(-1, BLOCK).sum(axis=1)


def nnz_bs(blk_idx, blk_cnt):
    """blk_idx [NB, topk], blk_cnt [NB]: whole blocks below the diagonal, the lower triangle on it."""
    blk_idx = np.asarray(blk_idx, dtype=np.int64)
    cnt = np.asarray(blk_cnt, dtype=np.int64)
    NB, topk = blk_idx.shape
    valid = (np.arange(topk)[None, :] < cnt[:, None]) & (blk_idx >= 0)
    b = np.arange(NB, dtype=np.int64)[:, None]
    below = (valid & (blk_idx < b)).sum(axis=1)
    diag = (valid & (blk_idx == b)).any(axis=1)
    return BLOCK * BLOCK * below + diag * (BLOCK * (BLOCK + 1) // 2)


def nnz_vs(N, v_idx, runs):
    """Run [t0, t1) of block b (first row q0) permits key q0 - t for every t in the run with
    0 <= q0 - t: all 64 rows if t >= 0, the rows at or below the key (64 + t of them) if t < 0.
    A kept vertical outside every run counts for the rows at or below it."""
    NB = N // BLOCK
    q0 = BLOCK * np.arange(NB, dtype=np.int64)[:, None]
    runs = np.asarray(runs, dtype=np.int64).reshape(-1, 2)
    v = np.asarray(v_idx, dtype=np.int64)
    out = np.zeros(NB, dtype=np.int64)
    if runs.size:
        t0, t1 = runs[None, :, 0], runs[None, :, 1]
        full = np.maximum(np.minimum(t1, q0 + 1) - np.maximum(t0, 0), 0)           # t >= 0, key >= 0
        a, e = np.maximum(t0, -(BLOCK - 1)), np.minimum(t1, 0)                      # t in [a, e), t < 0
        m = np.maximum(e - a, 0)
        # sum over t = a .. e-1 of (64 + t); keys q0 - t <= q0 + 63 < N always hold for whole blocks
        part = m * BLOCK + (a + e - 1) * m // 2
        out += (BLOCK * full + part).sum(axis=1)
    if v.size:
        for lo in range(0, NB, 1024):
            hi = min(NB, lo + 1024)
            t = q0[lo:hi] - v[None, :]
            rows = np.clip(BLOCK + np.minimum(t, 0), 0, BLOCK)                     # 64 if v <= q0, fewer above
            if runs.size:
                j = np.searchsorted(runs[:, 0], t, side="right") - 1
                inside = (j >= 0) & (t < runs[np.maximum(j, 0), 1])
                rows = np.where(inside, 0, rows)
            out[lo:hi] += rows.sum(axis=1)
    return out


def vs_index_nnz(idx, N):
    counts = idx.counts.cpu().numpy()
    v_idx = idx.v_idx.cpu().numpy()
    cover = idx.cover.cpu().numpy()
    return np.stack([nnz_vs(N, v_idx[r, :counts[r, 0]], cover[r, :counts[r, 2]]) for r in range(idx.rows)])


def bs_index_nnz(idx):
    bi, bc = idx.blk_idx.cpu().numpy(), idx.blk_cnt.cpu().numpy()
    return np.stack([nnz_bs(bi[r], bc[r]) for r in range(idx.rows)])


def vs_index_tiles(idx, N):
    """Per-head tile counts [rows, NB] of a binding.VSIndex (copies it to the host)."""
    counts = idx.counts.cpu().numpy()
    v_idx = idx.v_idx.cpu().numpy()
    cover = idx.cover.cpu().numpy()
    return np.stack([tiles_vs(N, v_idx[r, :counts[r, 0]], cover[r, :counts[r, 2]])
                     for r in range(idx.rows)])


def vs_index_steps(idx, N):
    """Per-head counts [rows, NB] of the 64 x 32 steps the Vertical-Slash kernel executes."""
    counts = idx.counts.cpu().numpy()
    v_idx = idx.v_idx.cpu().numpy()
    cover = idx.cover.cpu().numpy()
    return np.stack([tiles_vs(N, v_idx[r, :counts[r, 0]], cover[r, :counts[r, 2]], width=STEP)
                     for r in range(idx.rows)])


def bs_index_tiles(idx):
    return idx.blk_cnt.cpu().numpy().astype(np.int64)


def sparsity(tiles, N):
    """Fraction of the causal tile triangle that is NOT computed (cf. App. F)."""
    return 1.0 - float(np.sum(tiles)) / float(tiles_dense(N).sum())
