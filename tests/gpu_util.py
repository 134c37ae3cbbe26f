"""Helpers for the GPU parity tests: move seeded workloads to the device, run the C-ABI
path through the binding, run the CPU oracle per head, compare."""
from __future__ import annotations

from math import sqrt
from typing import Dict, Iterable, Optional

import numpy as np
import torch

from bsa_workloads import Workload, bf16_round, head_inputs, head_tensor
from oracle import bsa_oracle as o
from paper_2509_01085_amd import binding as B

# Deciding comparisons closer to equality than this (relative to the row's total mass) are
# within reach of the one non-reproducible step (exp of libm vs the device, summation tree
# of the scan): such a row may legitimately differ by its boundary block.
SELECT_MARGIN = 1e-10


def progress(msg: str) -> None:
    """Progress line of a long test: stdout (visible with -s) and a log file in the run's output
    folder, so that a run whose output pytest captures is still seen to be alive."""
    import os
    import time

    print(msg, flush=True)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        with open(os.path.join(root, "gpurun_out", "test_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def shape_of(wl: Workload) -> B.Shape:
    return B.Shape(wl.B, wl.H, *wl.grid, *wl.block, wl.d, B.F32 if wl.dtype == "fp32" else B.BF16, *wl.window, int(wl.block_major))


def part_of(wl: Workload) -> o.Partition:
    return o.Partition(*wl.grid, *wl.block, *wl.window, wl.block_major)


def device_inputs(wl: Workload, names=("Q", "K", "V", "dO"), heads: Optional[Iterable[int]] = None) -> Dict[str, torch.Tensor]:
    """[B,H,L,d] device tensors of the workload's dtype (heads not listed stay zero)."""
    dt = torch.float32 if wl.dtype == "fp32" else torch.bfloat16
    out = {}
    for name in names:
        host = torch.zeros((wl.B, wl.H, wl.L, wl.d), dtype=dt)
        for b in range(wl.B):
            for h in (range(wl.H) if heads is None else heads):
                host[b, h] = torch.from_numpy(head_tensor(wl, name, b, h)).to(dt)  # exact: values are bf16 already
        out[name] = host.cuda()
    return out


def run_indices(wl: Workload, x: Dict[str, torch.Tensor], threshold=None, keep_ratio=None):
    shp = shape_of(wl)
    Qbar = B.pool_blocks(shp, x["Q"])
    Kbar = B.pool_blocks(shp, x["K"])
    lists = B.select_kv(shp, Qbar, Kbar, wl.threshold if threshold is None else threshold)
    keep = B.prune_q(shp, x["Q"], wl.keep_ratio if keep_ratio is None else keep_ratio)
    return shp, Qbar, Kbar, lists, keep


def lists_to_host(shp: B.Shape, lists: B.KvLists):
    torch.cuda.synchronize()
    nnz = int(lists.nnz.item())
    q2k_ptr = lists.q2k_ptr.cpu().numpy()
    assert q2k_ptr[-1] == nnz
    return dict(q2k_ptr=q2k_ptr, q2k_idx=lists.q2k_idx[:nnz].cpu().numpy(),
                k2q_ptr=lists.k2q_ptr.cpu().numpy(), k2q_idx=lists.k2q_idx[:nnz].cpu().numpy(), nnz=nnz)


def head_csr(host: dict, shp: B.Shape, b: int, h: int, which="q2k"):
    """Slice one head's CSR out of the all-rows CSR, rebased to start at 0."""
    r0 = (b * shp.H + h) * shp.N
    ptr = host[which + "_ptr"][r0:r0 + shp.N + 1]
    return (ptr - ptr[0]).astype(np.int32), host[which + "_idx"][ptr[0]:ptr[-1]]


def check_lists_against_oracle(wl: Workload, shp: B.Shape, host: dict, b: int, h: int, ix: o.HeadResult, scores=None):
    """Bit-exact CSR and transposed CSR; a row may differ only if its margin is below SELECT_MARGIN."""
    ptr, idx = head_csr(host, shp, b, h, "q2k")
    if np.array_equal(ptr, ix.q2k_ptr) and np.array_equal(idx, ix.q2k_idx):
        tptr, tidx = head_csr(host, shp, b, h, "k2q")
        assert np.array_equal(tptr, ix.k2q_ptr) and np.array_equal(tidx, ix.k2q_idx)
        return 0
    assert scores is not None, "lists differ from the oracle"
    bad = 0
    for i in range(shp.N):
        mine = idx[ptr[i]:ptr[i + 1]]
        ref = ix.q2k_idx[ix.q2k_ptr[i]:ix.q2k_ptr[i + 1]]
        if not np.array_equal(mine, ref):
            sel = o.select_row(scores[i], wl.threshold)
            assert sel.margin < SELECT_MARGIN, (i, sel.margin)
            assert abs(len(mine) - len(ref)) == 1 and len(np.setxor1d(mine, ref)) == 1
            bad += 1
    return bad


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / RMS(ref): the plain tolerance metric."""
    rms = float(np.sqrt(np.mean(np.asarray(ref, dtype=np.float64) ** 2)))
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(rms, 1e-30))


BF16_U = 2.0 ** -8  # unit roundoff of bfloat16 (8 significant bits, round to nearest even)


def rounding_bounds(xi: dict, part: o.Partition, ix, sm_scale: float, q_blocks=None):
    """First-order bounds E_X (X in O, dQ, dK, dV), element by element, on what storing
    the intermediate operands in bfloat16 can do to X.  With u = 2^-8:

      g  (folded upstream gradient) is rounded before it enters a contraction: |dg| <= u |g|
         hence |d(dP)| <= u |g| |v|^T
      P  is rounded before P v and P^T g:                  |dP~| <= u P
      dS = P (dP - delta) is rounded before dS k, dS^T q:  |d(dS)| <= P u |g||v|^T + u |dS|

      E_O  = u P |v|              E_dV = 2u P^T |g|
      E_dQ = scale |d(dS)| |k|    E_dK = scale |d(dS)|^T |q|

    Q, K, V, dO are exact in both implementations and accumulation is fp32 or better.
    The rounding of the stored result itself, u |X|, is added by parity_excess()."""
    u = BF16_U
    tok = part.block_tokens()
    X = {k: np.asarray(v, dtype=np.float64) for k, v in xi.items()}
    E = {k: np.zeros((part.L, X["Q"].shape[1])) for k in ("O", "dQ", "dK", "dV")}
    for i in (range(part.N) if q_blocks is None else q_blocks):
        rows = tok[i, ix.keep_idx[i]]
        keys = tok[ix.q2k_idx[ix.q2k_ptr[i]:ix.q2k_ptr[i + 1]]].reshape(-1)
        q, k, v = X["Q"][rows], X["K"][keys], X["V"][keys]
        out, _, P = o.attend_block(q, k, v, sm_scale)
        g = o.folded_grad(X["dO"], part, ix.keep_idx, i, tok)
        dS = P * (g @ v.T - (g * out).sum(axis=1, keepdims=True))
        ddS = u * (P * (np.abs(g) @ np.abs(v).T) + np.abs(dS))
        eO = u * (P @ np.abs(v))
        cpos = np.searchsorted(ix.keep_idx[i], part.center_of())  # each token's window center among the retained rows
        E["O"][tok[i]] = eO[cpos]
        E["O"][rows] = eO
        E["dQ"][rows] = sm_scale * (ddS @ np.abs(k))
        E["dK"][keys] += sm_scale * (ddS.T @ np.abs(q))
        E["dV"][keys] += 2 * u * (P.T @ np.abs(g))
    return E


def parity_excess(got: np.ndarray, ref: np.ndarray, dtype: str, E: Optional[np.ndarray] = None) -> float:
    """The parity figure compared with the tolerance (1e-4 for fp32, 2e-2 for bf16).

    fp32: max |got - ref| / RMS(ref).
    bf16: max (|got - ref| - E - u |ref|) / RMS(ref), E from rounding_bounds(): what is left
    after the unavoidable effect of bfloat16 storage of operands and of the result must
    stay below the tolerance."""
    got = np.asarray(got, dtype=np.float64)
    rms = max(float(np.sqrt(np.mean(np.asarray(ref, dtype=np.float64) ** 2))), 1e-30)
    err = np.abs(got - ref)
    if dtype == "bf16":
        assert E is not None
        err = np.maximum(err - E - BF16_U * np.abs(ref), 0.0)
    return float(err.max() / rms)


def o_storage_of(wl: Workload):
    """How the forward output is stored before the backward reads it back (None: exactly)."""
    if wl.dtype == "fp32":
        return lambda O: np.asarray(O, dtype=np.float32)
    return lambda O: bf16_round(np.asarray(O, dtype=np.float32))


def tol_of(wl: Workload) -> float:
    return 1e-4 if wl.dtype == "fp32" else 2e-2


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def rounding_bounds_kv_block(xi: dict, part: o.Partition, ix, sm_scale: float, j: int):
    """E_dK, E_dV of rounding_bounds() for the Bk tokens of KV block j alone."""
    u = BF16_U
    tok = part.block_tokens()
    X = {k: np.asarray(v, dtype=np.float64) for k, v in xi.items()}
    kj, vj = X["K"][tok[j]], X["V"][tok[j]]
    EK, EV = np.zeros_like(kj), np.zeros_like(vj)
    for i in ix.k2q_idx[ix.k2q_ptr[j]:ix.k2q_ptr[j + 1]]:
        rows = tok[i, ix.keep_idx[i]]
        keys = tok[ix.q2k_idx[ix.q2k_ptr[i]:ix.q2k_ptr[i + 1]]].reshape(-1)
        q = X["Q"][rows]
        out, lse, _ = o.attend_block(q, X["K"][keys], X["V"][keys], sm_scale)
        g = o.folded_grad(X["dO"], part, ix.keep_idx, int(i), tok)
        Pj = np.exp((q @ kj.T) * sm_scale - lse[:, None])
        dSj = Pj * (g @ vj.T - (g * out).sum(axis=1, keepdims=True))
        ddS = u * (Pj * (np.abs(g) @ np.abs(vj).T) + np.abs(dSj))
        EK += sm_scale * (ddS.T @ np.abs(q))
        EV += 2 * u * (Pj.T @ np.abs(g))
    return EK, EV
