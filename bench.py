#!/usr/bin/env python3
"""Benchmark of the BSA hot path on one MI355X.

A step is one attention layer, forward + backward, through all five C-ABI calls
(pool Q, pool K, select, prune, attention fwd, attention bwd) on a seeded synthetic
video-shaped workload that is resident in HBM before the timed region starts.

Prints ONE JSON line: ms per layer (the headline metric, lower is better), effective
(dense-equivalent) and actual TFLOP/s, the roofline of the dominant kernel measured live
with events on the launch stream, the in-repo dense baseline at the same shape, and the CPU
oracle timed on this host's cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor
from math import sqrt

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def measured_traffic_bytes(workload: str, kernel: str):
    """Bytes per launch between L2 and the memory side of `kernel`, read from the table that the
    rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE, scaled by a 1 GiB copy's readings) left in
    profiles/bench_<workload>.md; None when there is no such profile.  Hardware counters cannot
    be read from inside this process, so the committed summary is the source."""
    import re

    path = os.path.join(ROOT, "profiles", f"bench_{workload}.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    if "## Traffic" not in text:
        return None
    best = None
    for m in re.finditer(r"^\| `bsa::" + re.escape(kernel) + r"<[^`]*` \| ([0-9.]+) \| ([0-9.]+) \|$", text.split("## Traffic", 1)[1], re.M):
        tot = (float(m.group(1)) + float(m.group(2))) * 1e6
        best = tot if best is None else max(best, tot)  # the main launch, not its small combine launch
    return best


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="wan1p3b", help="tiny | wan1p3b | hd720p | long")
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--threshold", type=float, default=None)
    ap.add_argument("--keep-ratio", type=float, default=None)
    ap.add_argument("--block-major", action="store_true",
                    help="hold the tensors in block-major token order (the tokens of a block adjacent) instead of raster order")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-attention baseline")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the second workload (hd720p: 70,400 tokens, 40 heads) that the default run times after the "
                         "benchmark workload and reports under extra_workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-heads", type=int, default=3, help="heads of the workload the CPU oracle is timed on")
    ap.add_argument("--sweep", action="store_true",
                    help="the sparsity sweep instead of the single benchmark: sigma x threshold x keep_ratio on the "
                         "workload's shape, one JSON line per point (seed = point index)")
    ap.add_argument("--length-sweep", action="store_true",
                    help="speedup over the in-repo dense kernel versus sequence length (forward only and forward + "
                         "backward), one JSON line per length, at the paper's token counts from 23K to 153K")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain elementwise copy of this many MiB (read + write that much each), "
                         "the known-traffic dispatch that hardware-counter readings are scaled by")
    return ap.parse_args()


def make_inputs(wl, torch):
    from bsa_workloads import TENSOR_NAMES, head_tensor

    dt = torch.float32 if wl.dtype == "fp32" else torch.bfloat16
    jobs = [(n, b, h) for n in TENSOR_NAMES for b in range(wl.B) for h in range(wl.H)]
    host = {n: torch.empty((wl.B, wl.H, wl.L, wl.d), dtype=dt, pin_memory=True) for n in TENSOR_NAMES}

    def one(job):
        n, b, h = job
        host[n][b, h] = torch.from_numpy(head_tensor(wl, n, b, h)).to(dt)

    with ThreadPoolExecutor(max_workers=min(16, len(os.sched_getaffinity(0)))) as ex:
        list(ex.map(one, jobs))
    return {n: t.cuda() for n, t in host.items()}


def timed(torch, fn, iters):
    """Average ms per call of fn over `iters` calls, events on the current (launch) stream."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def timed_each(torch, fn, iters):
    """(mean, median) ms per call of fn: the mean over one bracket of exactly `iters` calls, the
    median over the calls' own event pairs (events on the launch stream)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(iters):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
    mid = each[iters // 2] if iters % 2 else 0.5 * (each[iters // 2 - 1] + each[iters // 2])
    return ev[0].elapsed_time(ev[iters]) / iters, mid


def cpu_baseline(wl, heads: int):
    """The oracle as it stands, on this host's cores: `heads` heads of the same workload."""
    import numpy as np

    from bsa_workloads import head_inputs
    from oracle import bsa_oracle as o

    part = o.Partition(*wl.grid, *wl.block, *wl.window, wl.block_major)
    dtype = np.float64 if wl.L <= 4096 else np.float32  # attention GEMMs; decisions are always fp64
    t = 0.0
    for h in range(heads):
        x = head_inputs(wl, 0, h)
        t0 = time.perf_counter()
        o.bsa_head(x["Q"], x["K"], x["V"], x["dO"], part, wl.threshold, wl.keep_ratio, dtype=dtype)
        t += time.perf_counter() - t0
    per_layer_ms = t / heads * wl.B * wl.H * 1e3
    return {
        "value": per_layer_ms, "unit": "ms/layer (fwd+bwd)", "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
        "sample": f"{heads} of {wl.B * wl.H} heads timed ({t:.1f} s), scaled by heads (heads are independent); "
                  f"attention GEMMs in {np.dtype(dtype).name}",
    }


def sweep(args, torch, B):
    """Config 4: 3 noise levels x 4 mass thresholds x 3 keep ratios on the benchmark shape."""
    from bsa_workloads import WORKLOADS

    dev = torch.device("cuda:0")
    base = WORKLOADS[args.workload]
    point = 0
    for sigma in (0.1, 0.3, 1.0):
        for p in (0.5, 0.8, 0.9, 0.95):
            for r in (0.25, 0.5, 1.0):
                wl = base.replace(sigma=sigma, threshold=p, keep_ratio=r, seed=point)
                shp = B.Shape(wl.B, wl.H, *wl.grid, *wl.block, wl.d, B.F32 if wl.dtype == "fp32" else B.BF16, *wl.window, int(wl.block_major))
                x = make_inputs(wl, torch)
                Q, K, V, dO = x["Q"], x["K"], x["V"], x["dO"]
                nk = B.n_keep(shp, r)
                lists = B.alloc_kv_lists(shp, dev)
                O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
                LSE = torch.empty((wl.B, wl.H, wl.L), dtype=torch.float32, device=dev)
                ws = torch.empty(max(1, B.bwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
                fws = torch.empty(max(1, B.fwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
                state = {}

                def indices():
                    state["lists"] = B.select_kv(shp, B.pool_blocks(shp, Q), B.pool_blocks(shp, K), p, out=lists)
                    state["keep"] = B.prune_q(shp, Q, r)

                def fwd():
                    B.attn_fwd(shp, Q, K, V, lists, state["keep"], O=O, LSE=LSE, workspace=fws)

                def bwd():
                    B.attn_bwd(shp, Q, K, V, O, LSE, dO, lists, state["keep"], dQ=dQ, dK=dK, dV=dV, workspace=ws)

                indices(); fwd(); bwd()
                t_idx, t_f, t_b = timed(torch, indices, args.steps), timed(torch, fwd, args.steps), timed(torch, bwd, args.steps)
                nnz = int(lists.nnz.item())
                f = nnz / (shp.rows * shp.N)
                flops = 14.0 * wl.d * nk * shp.Bk * nnz
                print(json.dumps({
                    "point": point, "sigma": sigma, "threshold": p, "keep_ratio": r, "n_keep": nk,
                    "selected_block_fraction": f, "sparsity": 1.0 - (nk / shp.Bk) * f,
                    "ms_indices": t_idx, "ms_fwd": t_f, "ms_bwd": t_b, "ms_layer": t_idx + t_f + t_b,
                    "actual_tflops": flops / ((t_f + t_b) * 1e-3) / 1e12,
                    "effective_tflops": 14.0 * wl.B * wl.H * wl.L * wl.L * wl.d / ((t_idx + t_f + t_b) * 1e-3) / 1e12,
                }), flush=True)
                point += 1
                del x, Q, K, V, dO, O, dQ, dK, dV, lists, ws, fws


# Latent grids for the paper's sequence lengths (Table 1 and the speedup-versus-length figure:
# 23,296 ... 153,600 tokens).  The paper does not print the grids: the two end points follow
# from its video sizes (61x448x832 and 157x768x1280 with a 4x8x8 VAE and 1x2x2 patches); the
# three in between are grids of about the quoted lengths that 4x4x4 blocks divide.
LENGTH_GRIDS = ((16, 28, 52), (16, 44, 64), (24, 44, 56), (36, 48, 68), (40, 48, 80))


def length_sweep(args, torch, B):
    from bsa_workloads import WORKLOADS

    dev = torch.device("cuda:0")
    base = WORKLOADS["wan1p3b_win"]  # the paper's defaults: 4x4x4 blocks, (2,2,2) windows, r = 0.5
    for grid in LENGTH_GRIDS:
        for p, r in ((0.9, 0.5), (0.6, 0.5), (0.8, 0.25)):
            wl = base.replace(grid=grid, threshold=p, keep_ratio=r)
            shp = B.Shape(wl.B, wl.H, *wl.grid, *wl.block, wl.d, B.BF16, *wl.window)
            x = make_inputs(wl, torch)
            Q, K, V, dO = x["Q"], x["K"], x["V"], x["dO"]
            nk = B.n_keep(shp, wl.keep_ratio)
            lists = B.alloc_kv_lists(shp, dev)
            O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
            LSE = torch.empty((wl.B, wl.H, wl.L), dtype=torch.float32, device=dev)
            ws = torch.empty(max(1, B.bwd_workspace_bytes(shp, nk), B.dense_bwd_workspace_bytes(shp)), dtype=torch.uint8, device=dev)
            fws = torch.empty(max(1, B.fwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
            state = {}

            def fwd():  # everything a forward pass needs: indices and attention
                B.select_kv(shp, B.pool_blocks(shp, Q), B.pool_blocks(shp, K), p, out=lists)
                state["keep"] = B.prune_q(shp, Q, wl.keep_ratio)
                B.attn_fwd(shp, Q, K, V, lists, state["keep"], O=O, LSE=LSE, workspace=fws)

            def bwd():
                B.attn_bwd(shp, Q, K, V, O, LSE, dO, lists, state["keep"], dQ=dQ, dK=dK, dV=dV, workspace=ws)

            dfw = lambda: B.dense_attn_fwd(shp, Q, K, V, O=O, LSE=LSE)
            dbw = lambda: B.dense_attn_bwd(shp, Q, K, V, O, LSE, dO, dQ=dQ, dK=dK, dV=dV, workspace=ws)
            fwd(); bwd()
            t_f, t_b = timed(torch, fwd, args.steps), timed(torch, bwd, args.steps)
            nnz = int(lists.nnz.item())
            dfw(); dbw()
            n = max(1, min(2, args.steps))
            td_f, td_b = timed(torch, dfw, n), timed(torch, dbw, n)
            f = nnz / (shp.rows * shp.N)
            print(json.dumps({
                "tokens": wl.L, "grid": list(grid), "threshold": p, "keep_ratio": wl.keep_ratio, "window": list(wl.window),
                "selected_block_fraction": f, "sparsity": 1.0 - (nk / shp.Bk) * f,
                "bsa_fwd_ms": t_f, "bsa_bwd_ms": t_b, "dense_fwd_ms": td_f, "dense_bwd_ms": td_b,
                "speedup_fwd": td_f / t_f, "speedup_fwd_bwd": (td_f + td_b) / (t_f + t_b),
                "ideal_speedup": 1.0 / ((nk / shp.Bk) * f),
            }), flush=True)
            del x, Q, K, V, dO, O, dQ, dK, dV, lists, ws, fws


def measure(wl, steps, warmup, torch, B, traffic=True):
    """One workload: `warmup` untimed layers, then exactly `steps` layers (all five calls, forward +
    backward) in one event bracket, then the per-call breakdown.  Returns the result dict and the
    device buffers (for the dense baseline)."""
    shp = B.Shape(wl.B, wl.H, *wl.grid, *wl.block, wl.d, B.F32 if wl.dtype == "fp32" else B.BF16, *wl.window, int(wl.block_major))
    dev = torch.device("cuda:0")
    x = make_inputs(wl, torch)
    Q, K, V, dO = x["Q"], x["K"], x["V"], x["dO"]

    # every output and workspace is allocated once, outside the timed region
    nk = B.n_keep(shp, wl.keep_ratio)
    Qbar = torch.empty((wl.B, wl.H, shp.N, wl.d), dtype=torch.float64, device=dev)
    Kbar = torch.empty_like(Qbar)
    lists = B.alloc_kv_lists(shp, dev)
    keep = torch.empty((wl.B, wl.H, shp.N, nk), dtype=torch.int32, device=dev)
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    LSE = torch.empty((wl.B, wl.H, wl.L), dtype=torch.float32, device=dev)
    ws = torch.empty(max(1, B.bwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
    fws = torch.empty(max(1, B.fwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)

    def indices():
        B.pool_blocks(shp, Q, Qbar)
        B.pool_blocks(shp, K, Kbar)
        B.select_kv(shp, Qbar, Kbar, wl.threshold, out=lists)
        B.prune_q(shp, Q, wl.keep_ratio, keep)

    def fwd():
        B.attn_fwd(shp, Q, K, V, lists, keep, O=O, LSE=LSE, workspace=fws)

    def bwd(stages=None):
        B.attn_bwd(shp, Q, K, V, O, LSE, dO, lists, keep, dQ=dQ, dK=dK, dV=dV, workspace=ws, stages=stages)

    def step():
        indices()
        fwd()
        bwd()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_step, ms_median = timed_each(torch, step, steps)
    wall = time.perf_counter() - t0

    # per-call breakdown (same buffers, separate event brackets)
    parts = {
        "pool_q": timed(torch, lambda: B.pool_blocks(shp, Q, Qbar), steps),
        "pool_k": timed(torch, lambda: B.pool_blocks(shp, K, Kbar), steps),
        "select": timed(torch, lambda: B.select_kv(shp, Qbar, Kbar, wl.threshold, out=lists), steps),
        "prune": timed(torch, lambda: B.prune_q(shp, Q, wl.keep_ratio, keep), steps),
        "attn_fwd": timed(torch, fwd, steps),
        "attn_bwd": timed(torch, bwd, steps),
        "bwd_pre": timed(torch, lambda: bwd(B.BWD_PRE), steps),
        "bwd_dq": timed(torch, lambda: bwd(B.BWD_DQ), steps),
        "bwd_dkv": timed(torch, lambda: bwd(B.BWD_DKV), steps),
    }
    nnz = int(lists.nnz.item())
    f = nnz / (shp.rows * shp.N)
    pair_flops = wl.d * nk * shp.Bk * nnz  # x4 fwd, x10 bwd (FlashAttention convention: one S recompute)
    t_attn = parts["attn_fwd"] + parts["attn_bwd"]
    actual_tflops = 14 * pair_flops / (t_attn * 1e-3) / 1e12
    dense_flops = 14.0 * wl.B * wl.H * wl.L * wl.L * wl.d
    # credited FLOPs per listed (query block, KV block) pair, in units of d*n_keep*Bk:
    # forward 4 (QK^T, PV); dK/dV kernel 8 (S, dP, dV, dK); dQ kernel 2 (its S/dP recompute is not credited)
    kernels = {"fwd_pipe_kernel": ("attn_fwd", 4), "bwd_dkv_pipe_kernel": ("bwd_dkv", 8), "bwd_dq_pipe_kernel": ("bwd_dq", 2)}
    dominant = max(kernels, key=lambda k: parts[kernels[k][0]])

    # second denominator: what a register-resident MFMA loop sustains on this GPU (two workgroups per CU)
    sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    B.mfma_probe(512, 2000, sink)
    probe_flops = [0]

    def probe():
        probe_flops[0] = B.mfma_probe(512, 20000, sink)

    t_probe = timed(torch, probe, 3)
    probe_tflops = probe_flops[0] / (t_probe * 1e-3) / 1e12

    def roof(kname):
        call, mult = kernels[kname]
        tf = mult * pair_flops / (parts[call] * 1e-3) / 1e12
        return {"kernel": kname, "bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / PEAK_BF16_TFLOPS, "frac_of_measured_mfma_loop": tf / probe_tflops,
                "traffic": measured_traffic_bytes(wl.name, kname) if traffic else None, "avg_launch_ms": parts[call],
                "algorithmic_flops_per_launch": mult * pair_flops}

    out = {
        "metric": "bsa_fwd_bwd_ms_per_layer", "value": ms_step, "unit": "ms", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_step, "ms_per_step_median": ms_median, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "H": wl.H, "d": wl.d, "grid": list(wl.grid), "block": list(wl.block),
                   "tokens": wl.L, "threshold": wl.threshold, "keep_ratio": wl.keep_ratio, "sigma": wl.sigma,
                   "window": list(wl.window), "layout": "block_major" if wl.block_major else "raster"},
        "selected_block_fraction": f, "nnz": nnz, "n_keep": nk,
        "ms_per_call": parts,
        "effective_tflops": dense_flops / (ms_step * 1e-3) / 1e12,
        "actual_tflops": actual_tflops,
        "actual_pct_of_bf16_peak": 100.0 * actual_tflops / PEAK_BF16_TFLOPS,
        "roofline": roof(dominant),
        "roofline_other": [roof(k) for k in kernels if k != dominant],
        "wall_s_timed_region": wall,
        "mfma_loop_measured_tflops": probe_tflops,
        "memory": {"torch_max_allocated_bytes": int(torch.cuda.max_memory_allocated()),
                   "bwd_workspace_bytes": int(B.bwd_workspace_bytes(shp, nk)), "fwd_workspace_bytes": int(B.fwd_workspace_bytes(shp, nk)),
                   "kv_list_capacity_bytes": int(sum(t.numel() * t.element_size() for t in (lists.q2k_ptr, lists.q2k_idx, lists.k2q_ptr, lists.k2q_idx))),
                   "select_workspace_bytes": int(lists.workspace.numel())},
    }
    pool_bytes = 2 * Q.numel() * Q.element_size() + 2 * Qbar.numel() * 8 + keep.numel() * 4 + Q.numel() * Q.element_size()
    t_stream = parts["pool_q"] + parts["pool_k"] + parts["prune"]
    out["index_prep_hbm"] = {"bytes": pool_bytes, "achieved_GBs": pool_bytes / (t_stream * 1e-3) / 1e9, "peak_GBs": PEAK_HBM_GBS}
    # selection: reads the pooled vectors, writes the CSR and its transpose; nominally HBM, in practice fp64 ALU work
    sel_bytes = 2 * Qbar.numel() * 8 + 2 * nnz * 4 + 2 * (shp.rows + 1) * 4
    out["select_hbm"] = {"bytes": sel_bytes, "achieved_GBs": sel_bytes / (parts["select"] * 1e-3) / 1e9, "peak_GBs": PEAK_HBM_GBS,
                         "pct_of_layer_time": 100.0 * parts["select"] / ms_step,
                         "fp64_gflop": 2.0 * shp.rows * shp.N * wl.d / 1e9}

    ctx = dict(shp=shp, dev=dev, Q=Q, K=K, V=V, dO=dO, dQ=dQ, dK=dK, dV=dV, LSE=LSE, dense_flops=dense_flops)
    return out, ctx


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    from bsa_workloads import WORKLOADS
    from paper_2509_01085_amd import binding as B

    if args.sweep or args.length_sweep:
        torch.cuda.set_device(0)
        (sweep if args.sweep else length_sweep)(args, torch, B)
        return
    wl = WORKLOADS[args.workload]
    over = {k: v for k, v in (("sigma", args.sigma), ("threshold", args.threshold), ("keep_ratio", args.keep_ratio)) if v is not None}
    if args.block_major:
        over["block_major"] = True
    if over:
        wl = wl.replace(**over)
    torch.cuda.set_device(0)
    out, ctx = measure(wl, args.steps, args.warmup, torch, B, traffic=not over)
    shp, dev, Q, K, V, dO, dQ, dK, dV, LSE = (ctx[k] for k in ("shp", "dev", "Q", "K", "V", "dO", "dQ", "dK", "dV", "LSE"))
    dense_flops, ms_step = ctx["dense_flops"], out["ms_per_step"]

    if not args.no_dense and wl.L <= 40000:
        dws = torch.empty(max(1, B.dense_bwd_workspace_bytes(shp)), dtype=torch.uint8, device=dev)
        Od, LSEd = torch.empty_like(Q), torch.empty_like(LSE)
        dfw = lambda: B.dense_attn_fwd(shp, Q, K, V, O=Od, LSE=LSEd)
        dbw = lambda: B.dense_attn_bwd(shp, Q, K, V, Od, LSEd, dO, dQ=dQ, dK=dK, dV=dV, workspace=dws)
        dfw(); dbw()
        n = max(1, min(3, args.steps))
        td_f, td_b = timed(torch, dfw, n), timed(torch, dbw, n)
        out["dense_baseline"] = {"fwd_ms": td_f, "bwd_ms": td_b, "ms": td_f + td_b,
                                 "tflops": dense_flops / ((td_f + td_b) * 1e-3) / 1e12,
                                 "speedup_of_bsa": (td_f + td_b) / ms_step}
    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)  # one vectorized elementwise dispatch: reads and writes calibration_copy_mib MiB
        torch.cuda.synchronize()
        out["calibration_copy_mib"] = args.calibration_copy_mib
    if args.workload == "wan1p3b" and not over and not args.no_extra:
        # the ~70K-token grid of the target (config 2), timed in the same run: 3 layers after 1 warm-up
        del ctx, Q, K, V, dO, dQ, dK, dV, LSE
        torch.cuda.empty_cache()
        ex, _ = measure(WORKLOADS["hd720p"], 3, 1, torch, B)
        keep_keys = ("config", "steps", "warmup", "ms_per_step", "ms_per_step_median", "ms_per_call", "nnz", "selected_block_fraction",
                     "effective_tflops", "actual_tflops", "actual_pct_of_bf16_peak", "roofline", "roofline_other", "memory")
        out["extra_workloads"] = {"hd720p": {"ms_per_layer": ex["ms_per_step"], **{k: ex[k] for k in keep_keys}}}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, max(1, min(args.cpu_heads, wl.H)))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
