#!/usr/bin/env python3
"""Benchmark of the sparse-prefill attention hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic layer: for the
default workload (c4: the mixed-pattern 1M-token layer, 24 Vertical-Slash +
6 Block-Sparse + 2 A-shape heads) that is both index builds and the three
attention calls, timed end to end with the inputs resident in HBM.  The same
run also reports the three single-pattern 128K layers (c1, c2, c3), our dense
causal kernel at both lengths for the speedup column, and the CPU oracle timed
on a bounded sample of the workload.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2407_02490_amd import binding as B          # noqa: E402
from paper_2407_02490_amd import costmodel as C        # noqa: E402
from paper_2407_02490_amd import workloads as W        # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
FT = C.tile_flops()


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def u8(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


class Timer:
    """HIP event pairs on torch's current stream (the stream every call here is enqueued on)."""

    def __init__(self):
        self.pairs = []

    def __enter__(self):
        self.a = torch.cuda.Event(enable_timing=True)
        self.b = torch.cuda.Event(enable_timing=True)
        self.a.record()
        return self

    def __exit__(self, *exc):
        self.b.record()
        self.pairs.append((self.a, self.b))

    def ms(self):
        return [a.elapsed_time(b) for a, b in self.pairs]

    def reset(self):
        self.pairs = []


class Layer:
    """One workload: buffers, the step function, tile counts."""

    def __init__(self, name):
        self.name = name
        c = W.CONFIGS[name]
        self.cfg = c
        t0 = time.time()
        self.x = W.make_config(name, device="cuda")
        torch.cuda.synchronize()
        log(f"{name}: inputs generated in {time.time() - t0:.1f}s")
        x = self.x
        self.N, self.Hq = x.seq_len, x.n_q_heads
        self.o = torch.empty_like(x.q)
        allh = list(range(self.Hq))
        if c["pattern"] == "mixed":
            self.vs_heads, self.bs_heads, self.a_heads = W.head_assignment(
                self.Hq, c["n_vs"], c["n_bs"], c["n_ashape"])
        else:
            self.vs_heads = allh if c["pattern"] == "vs" else []
            self.bs_heads = allh if c["pattern"] == "bs" else []
            self.a_heads = allh if c["pattern"] == "ashape" else []
        if self.vs_heads:
            self.vs_idx = B.alloc_vs_index(len(self.vs_heads), c["nv"], c["ns"], self.N)
            self.vs_ws = u8(B.minf_vs_index_workspace_bytes(x.q, x.k, len(self.vs_heads), c["last_q"]))
        if self.bs_heads:
            self.bs_idx = B.alloc_bs_index(len(self.bs_heads), self.N, c["topk"])
            self.bs_ws = u8(B.minf_bs_index_workspace_bytes(x.q, x.k, len(self.bs_heads), c["topk"]))
        self.t = {k: Timer() for k in ("vs_index", "bs_index", "ashape_attn", "vs_attn", "bs_attn", "vs_bs_attn")}
        self.one_launch = False

    def step(self):
        x, c, t = self.x, self.cfg, self.t
        if self.vs_heads:
            with t["vs_index"]:
                B.minf_build_vs_index(x.q, x.k, self.vs_heads, c["last_q"], c["nv"], c["ns"],
                                      self.vs_idx, self.vs_ws)
        if self.bs_heads:
            with t["bs_index"]:
                B.minf_build_bs_index(x.q, x.k, self.bs_heads, c["topk"], self.bs_idx, self.bs_ws)
        if self.a_heads:
            with t["ashape_attn"]:
                B.minf_ashape_attn(x.q, x.k, x.v, self.o, self.a_heads, c["n_init"], c["n_local"])
        if self.one_launch and self.vs_heads and self.bs_heads:
            with t["vs_bs_attn"]:           # both patterns in one launch (measured alternative, --one-launch)
                B.minf_vs_bs_attn(x.q, x.k, x.v, self.o, self.vs_heads, self.vs_idx, self.bs_heads, self.bs_idx)
            return
        if self.vs_heads:
            with t["vs_attn"]:
                B.minf_vs_attn(x.q, x.k, x.v, self.o, self.vs_heads, self.vs_idx)
        if self.bs_heads:
            with t["bs_attn"]:
                B.minf_bs_attn(x.q, x.k, x.v, self.o, self.bs_heads, self.bs_idx)

    def run(self, steps, warmup):
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        for t in self.t.values():
            t.reset()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        return wall_ms

    def tiles(self):
        """Tile counts per attention call (whole call, all its heads)."""
        out = {}
        if self.a_heads:
            out["ashape_attn"] = int(C.tiles_ashape(self.N, self.cfg["n_init"], self.cfg["n_local"]).sum()) * len(self.a_heads)
        if self.vs_heads:
            out["vs_attn"] = int(C.vs_index_tiles(self.vs_idx, self.N).sum())
        if self.bs_heads:
            out["bs_attn"] = int(C.bs_index_tiles(self.bs_idx).sum())
        return out

    def executed_tiles(self):
        """Work the attention kernels execute, in 64 x 64 tile units (what the FLOP rate is computed
        from).  Vertical-Slash: 64 x 32 steps / 2 (a run is walked 32 keys at a time, so a run whose
        length mod 64 is in 1 .. 32 costs half a tile less than the canonical count).  A-shape and
        Block-Sparse: the canonical tiles (the kernels run whole 64-key tiles / block pairs of steps)."""
        out = self.tiles()
        if self.vs_heads:
            out["vs_attn"] = int(C.vs_index_steps(self.vs_idx, self.N).sum()) / 2.0
        return out

    def nnz(self):
        """Permitted (query, key) pairs per attention call: the useful work, 4 * d FLOP each."""
        out = {}
        if self.a_heads:
            out["ashape_attn"] = int(C.nnz_ashape(self.N, self.cfg["n_init"], self.cfg["n_local"]).sum()) * len(self.a_heads)
        if self.vs_heads:
            out["vs_attn"] = int(C.vs_index_nnz(self.vs_idx, self.N).sum())
        if self.bs_heads:
            out["bs_attn"] = int(C.bs_index_nnz(self.bs_idx).sum())
        return out

    def report(self, wall_ms):
        tiles = self.tiles()
        done = self.executed_tiles()
        nnz = self.nnz()
        if self.one_launch and self.vs_heads and self.bs_heads:
            for d in (tiles, done, nnz):
                d["vs_bs_attn"] = d.pop("vs_attn") + d.pop("bs_attn")
        r = {"workload": self.name, "seq_len": self.N, "ms_per_layer": round(wall_ms, 4), "calls": {}}
        tot_tiles = tot_done = 0
        for k, t in self.t.items():
            ms = t.ms()
            if not ms:
                continue
            e = {"ms": round(float(np.mean(ms)), 4), "ms_min": round(float(np.min(ms)), 4)}
            if k == "vs_index":
                # one pass over K per K/V head in use, the estimating queries, the two line-score rows
                kv = len({h // (self.Hq // self.x.n_kv_heads) for h in self.vs_heads})
                by = kv * self.N * 256 + len(self.vs_heads) * (64 * 256 + 2 * self.N * 4)
                e.update({"algorithmic_bytes": by, "gb_per_s": round(by / (e["ms"] * 1e-3) / 1e9, 1),
                          "k_passes_run": "2 per K/V head in use (row max/sum, then normalised sums), "
                                          "each shared by the query heads of the group",
                          "workspace_mib": round(self.vs_ws.numel() / 2**20, 1)})
            if k == "bs_index":
                # all of Q of the heads and K of their K/V heads, once
                kv = len({h // (self.Hq // self.x.n_kv_heads) for h in self.bs_heads})
                by = (len(self.bs_heads) + kv) * self.N * 256
                nb = self.N // 64
                fl = len(self.bs_heads) * nb * (nb + 1) // 2 * 256          # causal block logits, fp32, d = 128
                e.update({"algorithmic_bytes": by, "gb_per_s": round(by / (e["ms"] * 1e-3) / 1e9, 1),
                          "logit_flop": fl, "fp32_tflops": round(fl / (e["ms"] * 1e-3) / 1e12, 2),
                          "workspace_mib": round(self.bs_ws.numel() / 2**20, 1)})
            if k in tiles:
                # tiles: canonical 64 x 64 decomposition of the mask (the cost model's unit);
                # executed_tiles: what the kernel computes (VS: 32-key steps); the rate uses the latter
                e["tiles"] = tiles[k]
                e["executed_tiles"] = done[k]
                e["tflops"] = round(done[k] * FT / (e["ms"] * 1e-3) / 1e12, 2)
                e["frac_of_bf16_peak"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
                e["tflops_of_canonical_tiles"] = round(tiles[k] * FT / (e["ms"] * 1e-3) / 1e12, 2)
                # FLOPs of the permitted pairs only (a tile also pays for its masked part)
                e["useful_tflops"] = round(4 * 128 * nnz[k] / (e["ms"] * 1e-3) / 1e12, 2)
                e["mask_fill_of_tiles"] = round(nnz[k] / (tiles[k] * 64 * 64), 4)
                tot_tiles += tiles[k]
                tot_done += done[k]
            r["calls"][k] = e
        r["tiles"] = tot_tiles
        r["executed_tiles"] = tot_done
        r["effective_tflops"] = round(tot_done * FT / (wall_ms * 1e-3) / 1e12, 2)
        dense_tiles = int(C.tiles_dense(self.N).sum()) * self.Hq
        r["sparsity_vs_causal"] = round(1.0 - tot_tiles / dense_tiles, 4)
        return r


def time_dense(x, heads, reps, keep=False):
    o = torch.empty_like(x.q)
    B.minf_dense_attn(x.q, x.k, x.v, o, heads[:1])       # touch the code path once, one head
    torch.cuda.synchronize()
    t = Timer()
    for _ in range(reps):
        with t:
            B.minf_dense_attn(x.q, x.k, x.v, o, heads)
    torch.cuda.synchronize()
    ms = float(np.mean(t.ms()))
    return (ms, o) if keep else ms


def output_distance(o_sparse, o_dense, heads):
    """Relative L2 distance of the sparse output from the dense causal one over
    the given heads -- the quantity the head-pattern search minimises (Alg. 1).
    Plain reductions over outputs both computed by the library."""
    num = den = 0.0
    for h in heads:
        a, b = o_sparse[h].float(), o_dense[h].float()
        num += float((a - b).square().sum())
        den += float(b.square().sum())
    return round(math.sqrt(num / den), 5) if den > 0 else None


def vs_budget_sweep(L, o_dense, reps=3):
    """Second workload: the Vertical-Slash budgets of W.VS_BUDGET_SWEEP on the
    inputs of a Vertical-Slash layer; index build and attention timed per call."""
    x, N = L.x, L.N
    heads = list(range(L.Hq))
    dense_tiles = int(C.tiles_dense(N).sum()) * L.Hq
    out = []
    for label, nv, ns in W.VS_BUDGET_SWEEP:
        idx = B.alloc_vs_index(len(heads), nv, ns, N)
        ws = u8(B.minf_vs_index_workspace_bytes(x.q, x.k, len(heads), L.cfg["last_q"]))
        ti, ta = Timer(), Timer()
        for r in range(reps + 1):
            with ti:
                B.minf_build_vs_index(x.q, x.k, heads, L.cfg["last_q"], nv, ns, idx, ws)
            with ta:
                B.minf_vs_attn(x.q, x.k, x.v, L.o, heads, idx)
            if r == 0:                      # warm-up
                torch.cuda.synchronize()
                ti.reset(); ta.reset()
        torch.cuda.synchronize()
        tiles = int(C.vs_index_tiles(idx, N).sum())
        done = int(C.vs_index_steps(idx, N).sum()) / 2.0
        ms_a = float(np.median(ta.ms()))
        e = {"setting": label, "nv": nv, "ns": ns, "index_ms": round(float(np.median(ti.ms())), 4),
             "attn_ms": round(ms_a, 4), "tiles": tiles, "executed_tiles": done,
             "tflops": round(done * FT / ms_a / 1e9, 2),
             "frac_of_bf16_peak": round(done * FT / ms_a / 1e9 / PEAK_BF16_TFLOPS, 4),
             "sparsity_vs_causal": round(1.0 - tiles / dense_tiles, 4)}
        if o_dense is not None:
            e["output_rel_l2_vs_dense"] = output_distance(L.o, o_dense, heads)
        out.append(e)
        del idx, ws
    return out


def short_context(lengths=(8192, 16384, 32768, 65536), reps=5):
    """Short prompts (App. D.2: below some length the index build is a large share of the
    time and sparse attention no faster than dense): the Vertical-Slash layer recipe at
    reduced lengths, default budgets; index, sparse attention and our dense kernel timed
    per call, all 32 heads."""
    out = []
    c = W.CONFIGS["c2"]
    for N in lengths:
        x = W.make_config("c2", device="cuda", N=N)
        heads = list(range(x.n_q_heads))
        o = torch.empty_like(x.q)
        idx = B.alloc_vs_index(len(heads), c["nv"], c["ns"], N)
        ws = u8(B.minf_vs_index_workspace_bytes(x.q, x.k, len(heads), c["last_q"]))
        ti, ta, td = Timer(), Timer(), Timer()
        for r in range(reps + 1):
            with ti:
                B.minf_build_vs_index(x.q, x.k, heads, c["last_q"], c["nv"], c["ns"], idx, ws)
            with ta:
                B.minf_vs_attn(x.q, x.k, x.v, o, heads, idx)
            with td:
                B.minf_dense_attn(x.q, x.k, x.v, o, heads)
            if r == 0:
                torch.cuda.synchronize()
                ti.reset(); ta.reset(); td.reset()
        torch.cuda.synchronize()
        mi, ma, md = (float(np.median(t.ms())) for t in (ti, ta, td))
        tiles = int(C.vs_index_tiles(idx, N).sum())
        out.append({"seq_len": N, "vs_index_ms": round(mi, 4), "vs_attn_ms": round(ma, 4), "dense_ms": round(md, 4),
                    "index_share": round(mi / (mi + ma), 3), "speedup_vs_our_dense": round(md / (mi + ma), 2),
                    "sparsity_vs_causal": round(1.0 - tiles / (int(C.tiles_dense(N).sum()) * len(heads)), 4)})
        del x, o, idx, ws
        torch.cuda.empty_cache()
    return out


def cpu_baseline(layer, budget_s=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the workload.  Every head pattern of
    the layer is sampled on its own -- the index build of one head (Vertical-Slash: in full;
    Block-Sparse: the pooling in full, block logits and top-k of sampled rows) and masked fp64
    attention on 64-row query blocks drawn uniformly over the sequence -- with a share of the
    time budget in proportion to the pattern's head count, and scaled linearly to the pattern's
    heads and the layer's query blocks."""
    from oracle import minference_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    c, N = layer.cfg, layer.N
    NB = N // 64
    rng = np.random.default_rng(7)
    groups = [(k, h) for k, h in (("vs", layer.vs_heads), ("bs", layer.bs_heads), ("ashape", layer.a_heads)) if h]
    n_all = sum(len(h) for _, h in groups)
    est_ms, measured, notes = 0.0, 0.0, []
    for kind, heads in groups:
        share = max(budget_s * len(heads) / n_all, 1.5)
        Qh, Kh, Vh = layer.x.head_f64(heads[0])
        t_index = t_index_measured = 0.0
        if kind == "vs":
            t0 = time.perf_counter()
            Vi, Si, _, _ = O.vs_index(Qh, Kh, c["last_q"], c["nv"], c["ns"])
            t_index = t_index_measured = time.perf_counter() - t0
            attend = lambda b: O.vs_attention(Qh, Kh, Vh, Vi, Si, 64 * b, 64 * b + 64)
            idx_note = f"index of 1 head in full {t_index:.2f}s"
        elif kind == "bs":
            t0 = time.perf_counter()
            Qp, Kp = O.bs_pool(Qh), O.bs_pool(Kh)
            t_pool = time.perf_counter() - t0
            tau = 1.0 / math.sqrt(Qh.shape[1])
            bi = -np.ones((NB, c["topk"]), dtype=np.int64)
            bc = np.zeros(NB, dtype=np.int64)

            def index_row(b):                    # Alg. 3 for one query block: block logits, top-k
                sel = O.topk_indices((Qp[b] @ Kp[:b + 1].T) * tau, c["topk"])
                bi[b, :sel.size], bc[b] = sel, sel.size

            t_rows, rows = 0.0, []
            while t_rows < share / 4 and len(rows) < 256:
                b = int(rng.integers(0, NB))
                t0 = time.perf_counter()
                index_row(b)
                t_rows += time.perf_counter() - t0
                rows.append(b)
            t_index = t_pool + t_rows / len(rows) * NB     # scaled to all rows
            t_index_measured = t_pool + t_rows

            def attend(b):
                if bc[b] == 0:
                    index_row(b)
                return O.bs_attention(Qh, Kh, Vh, bi, bc, 64 * b, 64 * b + 64)
            idx_note = f"pooling in full {t_pool:.2f}s + {len(rows)} index rows {t_rows:.2f}s (scaled to {NB} rows)"
        else:
            attend = lambda b: O.ashape_attention(Qh, Kh, Vh, c["n_init"], c["n_local"], 64 * b, 64 * b + 64)
            idx_note = "no index"
        t_attn, blocks = 0.0, []
        while t_attn + (t_index if kind == "vs" else 0.0) < share and len(blocks) < 64:
            b = int(rng.integers(0, NB))
            t0 = time.perf_counter()
            attend(b)
            t_attn += time.perf_counter() - t0
            blocks.append(b)
        measured += t_index_measured + t_attn
        est_ms += (t_index + t_attn / len(blocks) * NB) * len(heads) * 1e3
        notes.append(f"{kind} x{len(heads)}: {idx_note}, attention of {len(blocks)} blocks {t_attn:.2f}s")
        del Qh, Kh, Vh
    return {"value": round(est_ms, 1), "unit": "ms/layer (extrapolated)", "cores": int(cores), "kind": "oracle",
            "sample": f"{layer.name}: " + "; ".join(notes) + f"; each scaled to its heads and {NB} query blocks per head",
            "measured_s": round(measured, 2)}


def device_peak():
    """The bf16 dense MFMA peak derived from what the device reports: compute units x 4 SIMDs x
    1024 FLOP per SIMD and clock (v_mfma_f32_32x32x16_bf16: 32768 FLOP in 8 passes of 4 clocks)
    x the maximum engine clock (read from rocminfo's GPU agent).  roofline.frac divides by the
    published 2.5 PFLOP/s."""
    import re
    import subprocess
    p = torch.cuda.get_device_properties(0)
    cus, mhz = int(p.multi_processor_count), None
    try:
        txt = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=30).stdout
        for agent in txt.split("Agent ")[1:]:
            if "gfx" in agent and re.search(r"Device Type:\s*GPU", agent):
                m = re.search(r"Max Clock Freq\. \(MHz\):\s*(\d+)", agent)
                c = re.search(r"Compute Unit:\s*(\d+)", agent)
                if m:
                    mhz = float(m.group(1))
                if c:
                    cus = int(c.group(1))
                break
    except Exception:
        pass
    out = {"device": p.name, "compute_units": cus, "max_engine_clock_mhz": mhz, "flop_per_clock_per_cu": 4096,
           "published_bf16_tflops": PEAK_BF16_TFLOPS}
    if mhz:
        out["derived_bf16_tflops"] = round(cus * 4096 * mhz * 1e6 / 1e12, 1)
    return out


def roofline_of(rep, workload):
    """Roofline entry of a layer report: its attention call with the largest time."""
    dom = max((k for k in rep["calls"] if "tiles" in rep["calls"][k]), key=lambda k: rep["calls"][k]["ms"])
    d = rep["calls"][dom]
    return {"bound": "mfma", "kernel": dom, "achieved": d["tflops"], "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": round(d["tflops"] / PEAK_BF16_TFLOPS, 4),
            "traffic": read_traffic(f"{dom}:{workload}"),
            "flops_per_launch": d["executed_tiles"] * FT, "avg_launch_ms": d["ms"],
            # the same launch priced by the canonical 64 x 64 tiles of its mask (the unit earlier
            # versions of this line used; higher for Vertical-Slash, whose steps are 32 keys wide)
            "achieved_canonical_tiles": d["tflops_of_canonical_tiles"],
            "frac_canonical_tiles": round(d["tflops_of_canonical_tiles"] / PEAK_BF16_TFLOPS, 4)}


def read_traffic(kernel_tag):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3
    counter summary (profiles/*.txt, line 'traffic_bytes_per_launch[<tag>]: <n>')."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    key = f"traffic_bytes_per_launch[{kernel_tag}]:"
    for fn in sorted(os.listdir(pdir)):
        if fn.endswith((".txt", ".md")):
            for line in open(os.path.join(pdir, fn)):
                if line.strip().startswith(key):
                    try:
                        return float(line.strip()[len(key):].split()[0])
                    except ValueError:
                        return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--no-128k", action="store_true", help="skip the three 128K single-pattern layers")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense causal baseline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--one-launch", action="store_true",
                    help="run the Vertical-Slash and the Block-Sparse heads of the layer in one launch "
                         "(minf_vs_bs_attn: the measured, slower alternative) instead of two")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (known HBM bytes) so that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings can be scaled")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (heads would shard across "
              "GPUs without any exchange inside attention)", file=sys.stderr)
        sys.exit(2)
    B.lib()
    torch.cuda.set_device(0)
    if a.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 2.0, out=dst)          # a plain streaming kernel: reads 2^30 B, writes 2^30 B
        torch.cuda.synchronize()
        log("copy calibration: 3 x (1 GiB read + 1 GiB write) elementwise launches done")
        del src, dst
        torch.cuda.empty_cache()

    extra = {}
    # ---- 128K single-pattern layers first (smaller; freed before the 1M layer)
    if not a.no_128k and a.workload == "c4":
        at128 = {}
        for name in ("c1", "c2", "c3"):
            L = Layer(name)
            wall = L.run(max(a.steps, 3), a.warmup)
            at128[name] = L.report(wall)
            at128[name]["roofline"] = roofline_of(at128[name], name)
            log(name, json.dumps(at128[name]))
            o_dense = None
            if not a.no_dense:
                # the dense causal output of the same inputs: timed once (on c1's inputs), and the
                # reference of the output distance of every sparse layer
                ms, o_dense = time_dense(L.x, list(range(L.Hq)), 2 if name == "c1" else 1, keep=True)
                if name == "c1":
                    dt = int(C.tiles_dense(L.N).sum()) * L.Hq
                    at128["dense"] = {"ms": round(ms, 3), "tiles": dt, "tflops": round(dt * FT / ms / 1e9, 2)}
                    log("dense 128K", json.dumps(at128["dense"]))
                at128[name]["output_rel_l2_vs_dense"] = output_distance(L.o, o_dense, list(range(L.Hq)))
            if name == "c2":
                at128["c2_budget_sweep"] = vs_budget_sweep(L, o_dense)
                log("c2 budget sweep", json.dumps(at128["c2_budget_sweep"]))
            del L, o_dense
            torch.cuda.empty_cache()
        if "dense" in at128:
            for name in ("c1", "c2", "c3"):
                at128[name]["speedup_vs_our_dense"] = round(at128["dense"]["ms"] / at128[name]["ms_per_layer"], 2)
        extra["at_128k"] = at128
        extra["short_context"] = short_context()
        log("short context", json.dumps(extra["short_context"]))

    # ---- the timed workload
    L = Layer(a.workload)
    L.one_launch = a.one_launch
    torch.cuda.synchronize()
    wall = L.run(a.steps, a.warmup)
    rep = L.report(wall)
    log(a.workload, json.dumps(rep))

    # dominant kernel = the attention call with the largest time
    roofline = roofline_of(rep, a.workload)
    roofline["peak_derivation"] = device_peak()
    log("peak", json.dumps(roofline["peak_derivation"]))

    if not a.no_dense:
        if L.N > 262144:
            heads = list(range(L.Hq // L.x.n_kv_heads))        # one KV group, scaled to the layer
            ms = time_dense(L.x, heads, 1) * (L.Hq / len(heads))
            note = f"1 rep of one KV group ({len(heads)} heads) x {L.Hq // len(heads)}, extrapolated"
        else:
            ms = time_dense(L.x, list(range(L.Hq)), 2)
            note = "all heads, mean of 2 reps"
        dt = int(C.tiles_dense(L.N).sum()) * L.Hq
        extra["dense"] = {"ms": round(ms, 2), "tflops": round(dt * FT / ms / 1e9, 2), "how": note}
        extra["speedup_vs_our_dense"] = round(ms / wall, 2)
        log("dense", json.dumps(extra["dense"]))

    cpu = None if a.no_cpu else cpu_baseline(L)
    if cpu:
        log("cpu_baseline", json.dumps(cpu))

    c = L.cfg
    out = {
        "metric": "sparse-attn prefill ms/layer",
        "value": round(wall, 4), "unit": "ms/layer", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(wall, 4), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {c['name']}", "seq_len": L.N, "n_q_heads": L.Hq,
                   "n_kv_heads": L.x.n_kv_heads, "head_dim": 128,
                   "heads": {"vs": len(L.vs_heads), "bs": len(L.bs_heads), "ashape": len(L.a_heads)},
                   "budgets": {k: c[k] for k in ("nv", "ns", "topk", "n_init", "n_local", "last_q") if k in c}},
        "effective_tflops": rep["effective_tflops"],
        "frac_of_bf16_peak": round(rep["effective_tflops"] / PEAK_BF16_TFLOPS, 4),
        "breakdown": rep, "roofline": roofline, "cpu_baseline": cpu,
    }
    out.update(extra)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
