"""GPU parity at the full sizes of the named workloads, in the launch configuration the
benchmark times.  Index work is compared bit for bit on whole heads; attention outputs and
gradients on sampled query blocks (O, LSE, dQ) and sampled KV blocks (dK, dV), which the
oracle computes one by one in fp64.  Heads that are not sampled hold zeros on the device
(they still run through every kernel)."""
from math import sqrt

import numpy as np
import pytest
import torch

from bsa_workloads import WORKLOADS, head_inputs
from oracle import bsa_oracle as o
from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu

# workload -> (heads checked, query blocks sampled per head, KV blocks sampled per head)
PLAN = {
    "wan1p3b": ((0, 7, 11), 6, 2),
    "wan1p3b_win": ((4,), 4, 1),
    "hd720p": ((3, 39), 4, 1),
    "long": ((5,), 4, 1),
    # 16 retained queries per block: two query blocks per wavefront, paired backward records
    "wan1p3b_r25": ((2,), 4, 1),
}
FULL = dict(WORKLOADS, wan1p3b_r25=WORKLOADS["wan1p3b"].replace(name="wan1p3b_r25", keep_ratio=0.25, window=(2, 2, 2)))


# dK/dV of one KV block cost one oracle forward per query block that lists it: the sample takes
# the longest k2q list that is not beyond this many listers
MAX_LISTERS = {"wan1p3b": 600, "wan1p3b_win": 600, "wan1p3b_r25": 600, "hd720p": 600, "long": 400}


def _sample(rng, n, k, always=()):
    picks = set(always)
    while len(picks) < min(n, k + len(always)):
        picks.add(int(rng.integers(0, n)))
    return sorted(picks)


# ---- which units the launches split (the host-side launch plan of the MFMA kernels, restated) ----
# A launch covers `units` units; XCD x owns the contiguous range [x*q + min(x, r), ...) of q or
# q + 1 units (q, r = divmod(units, 8)) and walks the last n of it in four segments that a
# combine launch merges.  Forward and dQ: unit = a group of 4 query blocks (8 when n_keep <= 16),
# n = ceil(q / 5) when q >= 5 and the launch is shorter than 12 rounds of the chip's slots.
# dK/dV: unit = a pair of KV blocks, n = min(q mod 32 + 8, q / 2) when 4 <= q < 2048.
def _split_units(units, n):
    q, r = divmod(units, 8)
    out = []
    for x in range(8):
        start, cnt = x * q + min(x, r), q + (1 if x < r else 0)
        out.extend(range(start + cnt - n, start + cnt))
    return out


def split_query_blocks(N, BH, n_keep, h):
    """Query blocks of head h (B = 1) whose forward / dQ walk is split, or []."""
    pg = 8 if n_keep <= 16 else 4
    groups = -(-N // pg)
    units = groups * BH
    q = units // 8
    slots = 256 * (1 if n_keep > 32 else 2)
    if not (q >= 5 and units < 12 * slots):
        return []
    return [(u % groups) * pg for u in _split_units(units, (q + 4) // 5) if u // groups == h]


def split_kv_blocks(N, BH, h):
    """KV blocks of head h (B = 1) that belong to a pair whose dK/dV walk is split, or []."""
    pairs = -(-N // 2)
    units = pairs * BH
    q = units // 8
    if not (4 <= q < 64 * 32):
        return []
    return [(u % pairs) * 2 for u in _split_units(units, min(q % 32 + 8, q // 2)) if u // pairs == h]


@pytest.mark.parametrize("name", list(PLAN))
def test_full_size_parity(name):
    wl = FULL[name]
    heads, n_qb, n_kb = PLAN[name]
    part = U.part_of(wl)
    tok = part.block_tokens()
    scale = 1 / sqrt(wl.d)
    U.progress(f"[{name}] generating heads {heads}")
    x = U.device_inputs(wl, heads=heads)
    shp, Qbar, Kbar, lists, keep = U.run_indices(wl, x)
    O, LSE = B.attn_fwd(shp, x["Q"], x["K"], x["V"], lists, keep)
    dQ, dK, dV = B.attn_bwd(shp, x["Q"], x["K"], x["V"], O, LSE, x["dO"], lists, keep)
    torch.cuda.synchronize()
    host = U.lists_to_host(shp, lists)
    U.progress(f"[{name}] GPU done, nnz={host['nnz']} f={host['nnz'] / (shp.rows * shp.N):.3f}")
    rng = np.random.default_rng(123)
    compared = 0
    for h in heads:
        xi = head_inputs(wl, 0, h)
        ix = o.bsa_indices(xi["Q"], xi["K"], part, wl.threshold, wl.keep_ratio)
        # ---- index work: whole head, bit for bit
        assert np.array_equal(Qbar[0, h].cpu().numpy(), ix.Qbar) and np.array_equal(Kbar[0, h].cpu().numpy(), ix.Kbar)
        assert np.array_equal(keep[0, h].cpu().numpy(), ix.keep_idx)
        scores = o.block_scores(ix.Qbar, ix.Kbar, scale) if ix.select_margin <= U.SELECT_MARGIN else None
        differing = U.check_lists_against_oracle(wl, shp, host, 0, h, ix, scores)
        U.progress(f"[{name}] head {h}: lists ok (margin {ix.select_margin:.2e}, rows within rounding reach: {differing})")
        if differing:
            continue  # attention below assumes identical lists
        assert ix.prune_gap > 0  # the keep lists compared above were decided by a strict inequality
        # ---- forward and dQ on sampled query blocks: always the longest and the shortest list
        # and, where the launch splits walks, a query block of a split unit
        lens = np.diff(ix.q2k_ptr)
        nk = keep.shape[-1]
        always = [int(np.argmax(lens)), int(np.argmin(lens))] + split_query_blocks(part.N, wl.H, nk, h)[:1]
        qb = _sample(rng, part.N, n_qb, always=always)
        rO, rL = o.attn_fwd(xi["Q"], xi["K"], xi["V"], part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale, q_blocks=qb)
        O_in = U.o_storage_of(wl)(rO)
        rdQ, _, _ = o.attn_bwd(xi["Q"], xi["K"], xi["V"], xi["dO"], part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale,
                               q_blocks=qb, O_in=O_in)
        sg = U.T.rounding_sigma(xi, part, ix, scale, q_blocks=qb) if wl.dtype == "bf16" else {"dQ": None}
        sel = tok[qb].reshape(-1)
        gO, gL, gdQ = (U.host_f64(t[0, h])[sel] for t in (O, LSE, dQ))
        # RMS over the sampled rows stands in for the tensor's RMS
        figs = U.check_tensors(name, f"h{h} query blocks {qb}", wl.dtype, [("O", gO, rO[sel]), ("dQ", gdQ, rdQ[sel])],
                               sigma={"dQ": sg["dQ"][sel]} if wl.dtype == "bf16" else None, lse=(gL, rL[sel]))
        U.progress(f"[{name}] head {h}: query blocks {qb}: {figs}")
        # ---- dK, dV on sampled KV blocks: the longest k2q list within the cost cap, the shortest
        # non-empty one, and a KV block whose walk the dK/dV launch splits
        klens = np.diff(ix.k2q_ptr)
        cap = MAX_LISTERS[name]
        listed = [int(j) for j in np.argsort(klens, kind="stable") if klens[j] > 0]
        order = [j for j in listed if klens[j] <= cap] or listed[:1]  # (every list beyond the cap: the shortest one)
        kb = [order[-1], order[0]][:max(n_kb, 1)]
        split = sorted(split_kv_blocks(part.N, wl.H, h), key=lambda j: klens[j])
        kb += [j for j in split if klens[j] > 0][:1]
        for j in sorted(set(kb)):
            # the stored O the backward reads, for every query block that lists j
            need = [int(i) for i in ix.k2q_idx[ix.k2q_ptr[j]:ix.k2q_ptr[j + 1]]]
            fO, _ = o.attn_fwd(xi["Q"], xi["K"], xi["V"], part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale, q_blocks=need)
            rdK, rdV = o.attn_bwd_kv_block(xi["Q"], xi["K"], xi["V"], xi["dO"], part, ix.q2k_ptr, ix.q2k_idx,
                                           ix.k2q_ptr, ix.k2q_idx, ix.keep_idx, scale, j, O_in=U.o_storage_of(wl)(fO))
            sK, sV = U.T.rounding_sigma_kv_block(xi, part, ix, scale, j) if wl.dtype == "bf16" else (None, None)
            gdK, gdV = U.host_f64(dK[0, h])[tok[j]], U.host_f64(dV[0, h])[tok[j]]
            f2 = U.check_tensors(name, f"h{h} KV block {j} ({klens[j]} listers)", wl.dtype, [("dK", gdK, rdK), ("dV", gdV, rdV)],
                                 sigma={"dK": sK, "dV": sV})
            U.progress(f"[{name}] head {h}: KV block {j} ({klens[j]} listers): {f2}")
        compared += 1
    assert compared, "no head could be compared"
