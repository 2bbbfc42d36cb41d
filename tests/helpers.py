"""Shared helpers of the parity tests (no method arithmetic here)."""
import numpy as np
import torch

# Parity bar for attention outputs with bf16 inputs (benchmark contract):
MAX_ABS = 2e-2
MEAN_ABS = 5e-3


def to_f64(t):
    return t.double().cpu().numpy()


def assert_close_rows(got_bf16, want_f64, what=""):
    got = got_bf16.double().cpu().numpy()
    err = np.abs(got - want_f64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.4g} > {MAX_ABS}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.4g} > {MEAN_ABS}"
    return err.max(), err.mean()


def random_qkv(seed, n_q, n_kv, N, d=128, device="cuda"):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(n_q, N, d, generator=g).to(torch.bfloat16)
    k = torch.randn(n_kv, N, d, generator=g).to(torch.bfloat16)
    v = torch.randn(n_kv, N, d, generator=g).to(torch.bfloat16)
    return q.to(device), k.to(device), v.to(device)


def check_topk(gpu_idx, oracle_scores, k, tol=1e-3, relative=True):
    """Index-set parity with the tie rule of the benchmark contract.

    The GPU set must equal the oracle's exact top-k except for swaps among
    scores within `tol` of the k-th largest oracle score (relative for the
    positive line scores of the Vertical-Slash estimate, absolute for the
    Block-Sparse block logits).  Returns the number of tolerated swaps.
    """
    from oracle import minference_oracle as O
    gpu_idx = np.asarray(gpu_idx, dtype=np.int64)
    want = O.topk_indices(oracle_scores, k)
    assert gpu_idx.size == want.size, f"set size {gpu_idx.size} != {want.size}"
    assert np.all(np.diff(gpu_idx) > 0), "indices must be ascending and unique"
    assert gpu_idx.size == 0 or (gpu_idx[0] >= 0 and gpu_idx[-1] < len(oracle_scores))
    extra = np.setdiff1d(gpu_idx, want)
    missing = np.setdiff1d(want, gpu_idx)
    if extra.size == 0:
        return 0
    s_k = np.sort(oracle_scores)[::-1][want.size - 1]
    if relative:
        lo, hi = s_k * (1 - tol), s_k * (1 + tol)
    else:
        lo, hi = s_k - tol, s_k + tol
    assert np.all(oracle_scores[extra] >= lo), "GPU kept an index whose oracle score is below the tie band"
    assert np.all(oracle_scores[missing] <= hi), "GPU dropped an index whose oracle score is above the tie band"
    return int(extra.size)
