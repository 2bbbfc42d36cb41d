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


def tiles_vs(N, v_idx, runs):
    """v_idx: ascending kept verticals; runs: [n, 2] offset runs [t0, t1)."""
    NB = N // BLOCK
    q0 = BLOCK * np.arange(NB, dtype=np.int64)[:, None]
    runs = np.asarray(runs, dtype=np.int64).reshape(-1, 2)
    v = np.asarray(v_idx, dtype=np.int64)
    out = np.zeros(NB, dtype=np.int64)
    if runs.size:
        ks = np.maximum(q0 - runs[None, :, 1] + 1, 0)
        ke = np.minimum(q0 - runs[None, :, 0] + 1, N)
        ln = np.maximum(ke - ks, 0)
        out += (-(-ln // BLOCK)).sum(axis=1)
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
            out[lo:hi] += -(-free // BLOCK)
    return out


def vs_index_tiles(idx, N):
    """Per-head tile counts [rows, NB] of a binding.VSIndex (copies it to the host)."""
    counts = idx.counts.cpu().numpy()
    v_idx = idx.v_idx.cpu().numpy()
    cover = idx.cover.cpu().numpy()
    return np.stack([tiles_vs(N, v_idx[r, :counts[r, 0]], cover[r, :counts[r, 2]])
                     for r in range(idx.rows)])


def bs_index_tiles(idx):
    return idx.blk_cnt.cpu().numpy().astype(np.int64)


def sparsity(tiles, N):
    """Fraction of the causal tile triangle that is NOT computed (cf. App. F)."""
    return 1.0 - float(np.sum(tiles)) / float(tiles_dense(N).sum())
