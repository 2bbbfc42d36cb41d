"""Shared helpers of the parity tests (no method arithmetic here)."""
import numpy as np
import torch

# Parity bar for attention outputs with bf16 inputs (benchmark contract):
MAX_ABS = 2e-2
MEAN_ABS = 5e-3
# At 128K / 1M tokens an output element is ~0.02 in magnitude, so a whole lost 64-key tile stays
# inside the absolute bar.  Every checked group of rows (a 64-row query block as a rule) must
# therefore also be close in relative L2 norm.  The kernels round P to bf16 (relative 2^-9 per
# element, signs random) and accumulate in fp32: observed ||err|| / ||want|| is 1e-3 .. 4e-3 on
# every committed case; a dropped tile or a dropped gathered step moves it to several percent.
REL_L2 = 1.5e-2

_observed = {"max_abs": 0.0, "mean_abs": 0.0, "rel_l2": 0.0, "n": 0}


def to_f64(t):
    return t.double().cpu().numpy()


def observed_errors():
    """Largest errors seen by assert_close_rows so far in this process."""
    return dict(_observed)


def error_norms(got_f64, want_f64):
    """(max-abs, mean-abs, ||err||_2 / ||want||_2) of an output against the oracle's."""
    err = np.abs(got_f64 - want_f64)
    den = float(np.sqrt(np.sum(want_f64 * want_f64)))
    rel = float(np.sqrt(np.sum(err * err))) / den if den > 1e-9 else 0.0
    return float(err.max()), float(err.mean()), rel


def assert_close_rows(got_bf16, want_f64, what="", rel_l2=REL_L2):
    got = got_bf16.double().cpu().numpy()
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    mx, mean, rel = error_norms(got, want_f64)
    _observed["max_abs"] = max(_observed["max_abs"], mx)
    _observed["mean_abs"] = max(_observed["mean_abs"], mean)
    _observed["rel_l2"] = max(_observed["rel_l2"], rel)
    _observed["n"] += 1
    assert mx <= MAX_ABS, f"{what}: max-abs {mx:.4g} > {MAX_ABS} (mean {mean:.3g}, rel-L2 {rel:.3g})"
    assert mean <= MEAN_ABS, f"{what}: mean-abs {mean:.4g} > {MEAN_ABS} (max {mx:.3g}, rel-L2 {rel:.3g})"
    assert rel <= rel_l2, f"{what}: relative L2 error {rel:.4g} > {rel_l2} (max {mx:.3g}, mean {mean:.3g})"
    return mx, mean, rel


def random_qkv(seed, n_q, n_kv, N, d=128, device="cuda"):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(n_q, N, d, generator=g).to(torch.bfloat16)
    k = torch.randn(n_kv, N, d, generator=g).to(torch.bfloat16)
    v = torch.randn(n_kv, N, d, generator=g).to(torch.bfloat16)
    return q.to(device), k.to(device), v.to(device)


def check_topk(gpu_idx, oracle_scores, k, tol=1e-3, relative=True, max_swaps=None):
    """Index-set parity with the tie rule of the benchmark contract.

    The GPU set must equal the oracle's exact top-k except for swaps among
    scores within `tol` of the k-th largest oracle score (relative for the
    positive line scores of the Vertical-Slash estimate, absolute for the
    Block-Sparse block logits).  Returns the number of tolerated swaps, which
    must not exceed max_swaps when that is given.
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
    if max_swaps is not None:
        assert extra.size <= max_swaps, f"{extra.size} tolerated swaps > {max_swaps}"
    return int(extra.size)
