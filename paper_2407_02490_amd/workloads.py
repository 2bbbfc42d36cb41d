"""Seeded synthetic inputs for the sparse-prefill attention path.

This module only draws random tensors and applies rotary position embedding;
it holds none of the method's arithmetic (no attention, no top-k, no masks)
and is used both by the tests that drive the CPU oracle and by the callers of
the HIP library.

The paper evaluates on long-context benchmarks with trained models; neither
exists here.  These inputs take the paper's shapes (LLaMA-3-8B geometry:
32 query heads, 8 KV heads, d = 128; 128K and 1M tokens) and imitate the
structure its Section 2.2 describes: attention sinks / vertical lines, slash
lines at fixed offsets, spatially clustered blocks.

Recipe (all tensors [heads, N, d], bf16):
  base      Q, K, V ~ N(0, 1), drawn head by head from one seeded generator.
  RoPE      half-split pairing (x[f], x[f + d/2]), theta_f = base^(-2f/d),
            angles in float64, applied to Q and K.
  slash     two positional features, shared by a KV group, are added to every
            Q and K row after RoPE, so that <feature_i, feature_j> depends on
            the offset i-j only (a "periodic local-offset bias"):
            (a) local band: a moving average z_i over w white-noise vectors,
                E<z_i, z_j> ~ beta_local * sqrt(d) * max(0, 1 - |i-j|/w);
            (b) periodic slashes: F cosine/sine pairs at the harmonics of
                period T with Fejer weights, <phi_i, phi_j> =
                beta_period * sqrt(d) * (peaks of width ~T/F at multiples of T).
            beta is the logit boost at the peak.  Line scores of unstructured
            N(0,1) inputs are flat, their top-k scatters and the 64-wide
            slash tiles would then cover nearly the whole causal triangle.
  sinks     n_sink seeded key rows get +3 * mean of the last 64 query rows as
            they are after RoPE and the slash features (mean over the rows
            and over the query heads of the KV group), so those keys score
            high for the estimating queries.  With the slash features on this
            is a strong sink (tens of logits for the last rows), as attention
            sinks are in trained models.
  clusters  every 64-token block draws one of 64 seeded centroids ~ N(0, I);
            1.5 * centroid is added to the block's Q and K rows (after RoPE,
            so that the block affinity does not rotate away).
Order per KV group: features, K, then each query head, sinks, V.
"""
import math
from dataclasses import dataclass, field

import torch

__all__ = ["LayerInputs", "make_layer", "CONFIGS", "make_config", "head_assignment", "VS_BUDGET_SWEEP"]

BLOCK = 64

# Vertical-Slash budgets (vertical lines, slash lines) of the second workload:
# the four settings of the head-pattern search space (App. C.2, search-space
# table), the budget the 128K layer uses, and the two ablation limits that keep
# one line of the other kind (App. D.3, "only vertical" / "only slash").  They
# span the column-dominated and the slash-dominated extremes of the sparse kernel.
VS_BUDGET_SWEEP = [
    ("search (30, 2048)", 30, 2048),
    ("search (100, 1800)", 100, 1800),
    ("search (500, 1500)", 500, 1500),
    ("search (3000, 200)", 3000, 200),
    ("default (1000, 6096)", 1000, 6096),
    ("only vertical (1000, 1)", 1000, 1),
    ("only slash (1, 6096)", 1, 6096),
]


@dataclass
class LayerInputs:
    q: torch.Tensor            # [Hq, N, d] bf16
    k: torch.Tensor            # [Hkv, N, d] bf16
    v: torch.Tensor            # [Hkv, N, d] bf16
    sinks: torch.Tensor        # [Hkv, n_sink] int64 planted key positions (may be empty)
    meta: dict = field(default_factory=dict)

    @property
    def n_q_heads(self):
        return self.q.shape[0]

    @property
    def n_kv_heads(self):
        return self.k.shape[0]

    @property
    def seq_len(self):
        return self.q.shape[1]

    def head_f64(self, h):
        """(Q_h, K_kv(h), V_kv(h)) as float64 numpy arrays on the host."""
        g = self.n_q_heads // self.n_kv_heads
        kv = h // g
        return (self.q[h].double().cpu().numpy(), self.k[kv].double().cpu().numpy(),
                self.v[kv].double().cpu().numpy())


def _rope(x, base, chunk=1 << 16):
    """Rotate x [N, d] (float32) in place by position, half-split pairing."""
    N, d = x.shape
    half = d // 2
    inv = torch.pow(torch.tensor(float(base), dtype=torch.float64, device=x.device),
                    -torch.arange(half, dtype=torch.float64, device=x.device) * 2.0 / d)
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        ang = torch.arange(s, e, dtype=torch.float64, device=x.device)[:, None] * inv[None, :]
        c, sn = torch.cos(ang).float(), torch.sin(ang).float()
        a, b = x[s:e, :half].clone(), x[s:e, half:].clone()
        x[s:e, :half] = a * c - b * sn
        x[s:e, half:] = a * sn + b * c
    return x


def _slash_features(N, d, beta_local, w_local, beta_period, T, F, gen, device):
    """[N, d] float32 positional feature whose self inner products depend on
    the offset only: triangular local band plus Fejer peaks at multiples of T."""
    out = torch.zeros(N, d, dtype=torch.float32, device=device)
    if beta_local > 0:
        w = int(w_local)
        xi = torch.randn(N + w, d, generator=gen, device=device, dtype=torch.float32).double()
        c = torch.cumsum(xi, dim=0)
        del xi
        out += ((c[w:] - c[:-w]) * math.sqrt(beta_local / math.sqrt(d) / w)).float()
        del c
    if beta_period > 0:
        f = torch.arange(1, F + 1, dtype=torch.float64, device=device)
        lam = 1.0 - f / (F + 1)
        lam = lam / lam.sum()
        amp = torch.sqrt(lam * beta_period * math.sqrt(d))
        for s in range(0, N, 1 << 16):
            e = min(N, s + (1 << 16))
            ang = (torch.arange(s, e, dtype=torch.float64, device=device)[:, None]
                   * (2.0 * math.pi * f / T)[None, :])
            out[s:e, :F] += (amp * torch.cos(ang)).float()
            out[s:e, F:2 * F] += (amp * torch.sin(ang)).float()
    return out


def make_layer(seed, n_q_heads, n_kv_heads, N, d=128, rope_base=None, n_sink=0,
               slash=None, clusters=False, last_q=64, device="cpu"):
    """Draw one attention layer's Q, K, V.

    slash: None or dict(beta_local, w_local, beta_period, T, F).
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))
    g = n_q_heads // n_kv_heads
    NB = N // BLOCK
    q = torch.empty(n_q_heads, N, d, dtype=torch.bfloat16, device=dev)
    k = torch.empty(n_kv_heads, N, d, dtype=torch.bfloat16, device=dev)
    v = torch.empty(n_kv_heads, N, d, dtype=torch.bfloat16, device=dev)
    sinks = torch.empty(n_kv_heads, n_sink, dtype=torch.int64)

    cent = assign = None
    if clusters:
        cent = torch.randn(64, d, generator=gen, device=dev, dtype=torch.float32)
        assign = torch.randint(0, 64, (NB,), generator=gen, device=dev)

    R = min(last_q, N)
    for kv in range(n_kv_heads):
        feat = None
        if slash is not None:
            feat = _slash_features(N, d, slash["beta_local"], slash["w_local"],
                                   slash["beta_period"], slash["T"], slash["F"], gen, dev)
        kk = torch.randn(N, d, generator=gen, device=dev, dtype=torch.float32)
        if rope_base is not None:
            _rope(kk, rope_base)
        if feat is not None:
            kk += feat
        qlast_mean = torch.zeros(d, dtype=torch.float32, device=dev)
        for hq in range(kv * g, (kv + 1) * g):
            qq = torch.randn(N, d, generator=gen, device=dev, dtype=torch.float32)
            if rope_base is not None:
                _rope(qq, rope_base)
            if feat is not None:
                qq += feat
            qlast_mean += qq[N - R:].mean(dim=0) / g
            if clusters:
                qq.view(NB, BLOCK, d).add_(1.5 * cent[assign][:, None, :])
            q[hq] = qq.to(torch.bfloat16)
            del qq
        if n_sink > 0:
            pos = torch.randperm(N, generator=gen, device=dev)[:n_sink].sort().values
            kk[pos] += 3.0 * qlast_mean
            sinks[kv] = pos.cpu()
        if clusters:
            kk.view(NB, BLOCK, d).add_(1.5 * cent[assign][:, None, :])
        k[kv] = kk.to(torch.bfloat16)
        del kk
        v[kv] = torch.randn(N, d, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    meta = dict(seed=seed, N=N, d=d, rope_base=rope_base, n_sink=n_sink, slash=slash,
                clusters=clusters)
    return LayerInputs(q, k, v, sinks, meta)


# Offset structure used by the Vertical-Slash workloads: a local band that
# fades out over 16K tokens and slashes every 4096 tokens, ~128 tokens wide.
SLASH_128K = dict(beta_local=6.0, w_local=16384, beta_period=5.0, T=4096, F=32)

# The five workloads named by the benchmark contract.
CONFIGS = {
    "c0": dict(name="Vertical-Slash tiny", pattern="vs", n_q_heads=4, n_kv_heads=4, N=4096,
               rope_base=1.0e4, n_sink=16, slash=None, clusters=False,
               last_q=64, nv=256, ns=512),
    "c1": dict(name="A-shape 128K", pattern="ashape", n_q_heads=32, n_kv_heads=8, N=131072,
               rope_base=5.0e5, n_sink=0, slash=None, clusters=False,
               n_init=1024, n_local=4096),
    "c2": dict(name="Vertical-Slash 128K", pattern="vs", n_q_heads=32, n_kv_heads=8, N=131072,
               rope_base=5.0e5, n_sink=64, slash=SLASH_128K, clusters=False,
               last_q=64, nv=1000, ns=6096),
    "c3": dict(name="Block-Sparse 128K", pattern="bs", n_q_heads=32, n_kv_heads=8, N=131072,
               rope_base=None, n_sink=0, slash=None, clusters=True, topk=100),
    "c4": dict(name="Mixed-pattern 1M", pattern="mixed", n_q_heads=32, n_kv_heads=8, N=1048576,
               rope_base=5.0e5, n_sink=64, slash=SLASH_128K, clusters=True,
               last_q=64, nv=1000, ns=6096, topk=100, n_init=1024, n_local=4096,
               n_vs=24, n_bs=6, n_ashape=2),
}


def make_config(name, device="cpu", N=None, n_q_heads=None, n_kv_heads=None):
    """Inputs of workload `name` (seed = 1000 + its number).  N and the head
    counts may be overridden to get a reduced case of the same recipe."""
    c = dict(CONFIGS[name])
    if N is not None:
        c["N"] = N
    if n_q_heads is not None:
        c["n_q_heads"] = n_q_heads
    if n_kv_heads is not None:
        c["n_kv_heads"] = n_kv_heads
    seed = 1000 + int(name[1:])
    x = make_layer(seed, c["n_q_heads"], c["n_kv_heads"], c["N"], rope_base=c["rope_base"],
                   n_sink=c["n_sink"], slash=c["slash"], clusters=c["clusters"],
                   last_q=c.get("last_q", 64), device=device)
    x.meta.update(c)
    return x


def head_assignment(n_q_heads, n_vs, n_bs, n_ashape, seed=1004):
    """Seeded head -> pattern table of the mixed layer: a random permutation of
    the query heads, first n_vs Vertical-Slash, next n_bs Block-Sparse, rest
    A-shape.  Returns three ascending lists of head ids."""
    assert n_vs + n_bs + n_ashape == n_q_heads
    gen = torch.Generator()
    gen.manual_seed(seed)
    perm = torch.randperm(n_q_heads, generator=gen).tolist()
    return (sorted(perm[:n_vs]), sorted(perm[n_vs:n_vs + n_bs]), sorted(perm[n_vs + n_bs:]))
