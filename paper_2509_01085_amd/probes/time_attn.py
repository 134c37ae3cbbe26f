"""Probe, not part of the library: average launch time of the attention calls of one workload
with the library BSA_LIB points at (default: the in-tree build).  One JSON line.

    [BSA_LIB=variant.so] python -m paper_2509_01085_amd.probes.time_attn [workload] [--p=threshold] [--r=keep_ratio] [--bwd]"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import torch  # noqa: E402

from bench import make_inputs, timed  # noqa: E402
from bsa_workloads import WORKLOADS  # noqa: E402
from paper_2509_01085_amd import binding as B  # noqa: E402


def main():
    wl = WORKLOADS[next((a for a in sys.argv[1:] if not a.startswith("--")), "wan1p3b")]
    for a in sys.argv[1:]:
        if a.startswith("--r="):
            wl = wl.replace(keep_ratio=float(a[4:]))
        if a.startswith("--p="):
            wl = wl.replace(threshold=float(a[4:]))
    shp = B.Shape(wl.B, wl.H, *wl.grid, *wl.block, wl.d, B.BF16, *wl.window)
    x = make_inputs(wl, torch)
    Q, K, V, dO = x["Q"], x["K"], x["V"], x["dO"]
    lists = B.select_kv(shp, B.pool_blocks(shp, Q), B.pool_blocks(shp, K), wl.threshold)
    keep = B.prune_q(shp, Q, wl.keep_ratio)
    nk = keep.shape[-1]
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    LSE = torch.empty((wl.B, wl.H, wl.L), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(1, B.bwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device="cuda")
    fws = torch.empty(max(1, B.fwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device="cuda")
    fwd = lambda: B.attn_fwd(shp, Q, K, V, lists, keep, O=O, LSE=LSE, workspace=fws)
    for _ in range(10):
        fwd()
    r = {"lib": os.path.basename(os.environ.get("BSA_LIB", "libbsa.so")), "workload": wl.name, "threshold": wl.threshold,
         "keep_ratio": wl.keep_ratio, "nnz": int(lists.nnz.item()), "fwd_ms": round(timed(torch, fwd, 20), 4)}
    if "--bwd" in sys.argv:
        bwd = lambda st: B.attn_bwd(shp, Q, K, V, O, LSE, dO, lists, keep, dQ=dQ, dK=dK, dV=dV, workspace=ws, stages=st)
        for _ in range(3):
            bwd(7)
        r.update(dq_ms=round(timed(torch, lambda: bwd(B.BWD_DQ), 20), 4), dkv_ms=round(timed(torch, lambda: bwd(B.BWD_DKV), 20), 4))
    print(json.dumps(r), flush=True)


if __name__ == "__main__":
    main()
