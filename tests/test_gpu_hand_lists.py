"""The attention calls take any CSR a caller hands them, not only what Eq. 4 selects: lists
made by hand (one block, all blocks, random subsets, KV blocks that nobody lists) go through
bsa_attn_fwd / bsa_attn_bwd and are compared with the oracle's Eq. 5 + filling + backward on
the same lists.  Retained queries still come from Eq. 2 (the fill needs the critical tokens)."""
from math import sqrt

import numpy as np
import pytest
import torch

from bsa_workloads import Workload, head_inputs
from oracle import bsa_oracle as o
from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu

CASES = {
    "mfma_d128": Workload("hand_d128", 1, 2, 128, "bf16", (8, 8, 12), (4, 4, 4), keep_ratio=0.5),
    "mfma_d64_win": Workload("hand_d64", 2, 1, 64, "bf16", (4, 8, 20), (4, 4, 4), keep_ratio=0.5, window=(2, 2, 2)),
    "mfma_r100": Workload("hand_r100", 1, 1, 128, "bf16", (4, 8, 12), (4, 4, 4), keep_ratio=1.0),
    # 16 retained queries: two query blocks per wavefront and per backward record; 15 blocks, so the last has no partner
    "mfma_packed": Workload("hand_packed", 1, 2, 128, "bf16", (4, 12, 20), (4, 4, 4), keep_ratio=0.25),
    "generic_f32": Workload("hand_f32", 1, 2, 72, "fp32", (6, 6, 10), (3, 2, 5), keep_ratio=0.4),
}


def hand_lists(N: int, rng) -> list:
    """Row 0: its own block only; row 1: every block but the last; the others random subsets of
    random size that never contain the last block, which therefore gets zero dK, dV."""
    rows = []
    for i in range(N):
        if i == 0:
            rows.append(np.array([0]))
        elif i == 1:
            rows.append(np.arange(N - 1))
        else:
            k = int(rng.integers(1, N))
            rows.append(np.sort(rng.choice(N - 1, size=min(k, N - 1), replace=False)))
    return rows


@pytest.mark.parametrize("name", list(CASES))
def test_hand_made_lists(name):
    wl = CASES[name]
    U.progress(f"hand-made lists {name}")
    shp, part = U.shape_of(wl), U.part_of(wl)
    N, scale = shp.N, 1 / sqrt(wl.d)
    rng = np.random.default_rng(11)
    per_head = {(b, h): hand_lists(N, rng) for b in range(wl.B) for h in range(wl.H)}
    # global CSR over rows (b, h, i) and its transpose over (b, h, j)
    ptr, idx, tptr, tidx = [0], [], [0], []
    for b in range(wl.B):
        for h in range(wl.H):
            rows = per_head[b, h]
            hp = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
            hi = np.concatenate(rows).astype(np.int32)
            kp, ki = o.transpose_csr(hp, hi, N)
            idx.append(hi); ptr.extend((hp[1:] + ptr[-1]).tolist())
            tidx.append(ki); tptr.extend((np.asarray(kp[1:]) + tptr[-1]).tolist())
    dev = torch.device("cuda")
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    lists = B.KvLists(i32(ptr), i32(np.concatenate(idx)), i32(tptr), i32(np.concatenate(tidx)),
                      torch.tensor([ptr[-1]], dtype=torch.int64, device=dev), torch.empty(1, dtype=torch.uint8, device=dev))
    x = U.device_inputs(wl)
    keep = B.prune_q(shp, x["Q"], wl.keep_ratio)
    O, LSE = B.attn_fwd(shp, x["Q"], x["K"], x["V"], lists, keep)
    dQ, dK, dV = B.attn_bwd(shp, x["Q"], x["K"], x["V"], O, LSE, x["dO"], lists, keep)
    torch.cuda.synchronize()
    tok = part.block_tokens()
    for (b, h), rows in per_head.items():
        xi = head_inputs(wl, b, h)
        hp = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
        hi = np.concatenate(rows).astype(np.int32)
        keep_h = keep[b, h].cpu().numpy()
        assert np.array_equal(keep_h, o.prune_q(xi["Q"], part, wl.keep_ratio)[0])
        rO, rLSE = o.attn_fwd(xi["Q"], xi["K"], xi["V"], part, hp, hi, keep_h, scale)
        rdQ, rdK, rdV = o.attn_bwd(xi["Q"], xi["K"], xi["V"], xi["dO"], part, hp, hi, keep_h, scale,
                                   O_in=U.o_storage_of(wl)(rO))
        kp, ki = o.transpose_csr(hp, hi, N)
        ix = o.HeadResult(None, None, hp, hi, np.asarray(kp), np.asarray(ki), keep_h, 0.0, 0.0)
        sg = U.T.rounding_sigma(xi, part, ix, scale) if wl.dtype == "bf16" else None
        U.check_tensors("hand " + name, f"b{b} h{h}", wl.dtype,
                        [(nm, U.host_f64(got[b, h]), ref) for nm, got, ref in (("O", O, rO), ("dQ", dQ, rdQ), ("dK", dK, rdK), ("dV", dV, rdV))],
                        sigma=sg, lse=(U.host_f64(LSE[b, h]), rLSE))
        # the block nobody lists receives exactly zero gradient
        last = tok[N - 1]
        assert not dK[b, h].float().cpu().numpy()[last].any() and not dV[b, h].float().cpu().numpy()[last].any()
