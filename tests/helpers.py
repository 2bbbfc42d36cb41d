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
