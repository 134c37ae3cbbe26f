"""The floating-point parity criteria of the GPU tests, and the model behind the bf16 ones.
Pure numpy + oracle (no GPU, no binding), so the criteria themselves are tested on the CPU
(tests/test_tolerance_model.py feeds them perturbed oracle results and requires failure).

fp32 path: every tensor  max |got - ref| / RMS(ref) <= 1e-4  (the stated tolerance).

bf16 path (inputs and results stored in bfloat16, unit roundoff u = 2^-8):
  LSE      fp32 on both sides: |got - ref| <= 1e-4.
  all      RMS(got - ref) / RMS(ref) <= 5e-3.  bf16 rounding of operands and of the result
           gives 2-3e-3; a 1 % scale error gives 1e-2.
  O        element by element  |got - ref| <= 2e-2 RMS(ref) + u |ref|: the stated tolerance plus
           the rounding of the stored value itself.  The plain figure max |got - ref| / RMS(ref)
           is logged beside it; it stays below 2e-2 whenever max |O| / RMS(O) < 5.1, and cannot be
           guaranteed beyond (the largest entry alone may then be stored u |O| > 2e-2 RMS off).
  dQ,dK,dV element by element
               |got - ref| <= 2e-2 RMS(ref) + u |ref| + 6 sigma,
           because the gradients are heavy-tailed (max |x| / RMS of 15-45: the fill gradient folds
           a window's dO rows into its critical token's row), so storing even the exact value
           in bf16 moves the largest entries by more than 2e-2 RMS (u |ref|), and so does the
           bf16 rounding of the MFMA operands g, P and dS (sigma).  sigma is the standard
           deviation of that operand-rounding error under independent relative errors of
           variance u^2/3 per rounded value (a root-sum-square, not a worst case):

             g~ = g (1 + e)         rounded once per (query, channel)
             P~ = P (1 + e)         per (query, key), before P^T g
             dS~ = dS (1 + e)       per (query, key), before dS k and dS^T q
             dS  = P (g~ v^T - delta)

             var dV[m,c] = s2 sum_n P_nm^2 g_nc^2 * 2
             var dK[m,c] = s2 scale^2 sum_n q_nc^2 (dS_nm^2 + P_nm^2 sum_c' g_nc'^2 v_mc'^2 [+ P_nm^2 vd_n])
             var dQ[n,c] = s2 scale^2 (sum_m dS_nm^2 k_mc^2 + sum_c' g_nc'^2 A_n[c',c]^2 [+ vd_n kbar_nc^2])
             A_n = V^T diag(P_n) K,  kbar_n = P_n K,  s2 = u^2 / 3

           The bracketed terms (vd_n = sum_c g_nc^2 O_nc^2: delta = <g, O> formed from a stored O
           that differs from the reference's stored O by rounding flips) apply only when the
           backward under test read its own forward's output; a backward that was handed the
           reference's stored O is held to the bound without them.
"""
from __future__ import annotations

from math import sqrt
from typing import Dict, Optional, Sequence

import numpy as np

from oracle import bsa_oracle as o

BF16_U = 2.0 ** -8      # unit roundoff of bfloat16 (8 significant bits, round to nearest even)
RSS_MULTIPLE = 6.0      # how many standard deviations of the operand-rounding model are allowed
TOL_F32 = 1e-4
TOL_BF16 = 2e-2
TOL_RMS_BF16 = 5e-3
TOL_LSE = 1e-4


def _rms(x) -> float:
    x = np.asarray(x, dtype=np.float64)
    return max(float(np.sqrt(np.mean(x * x))), 1e-30)


def rounding_sigma(xi: dict, part: o.Partition, ix, sm_scale: float, q_blocks: Optional[Sequence[int]] = None,
                   own_forward: bool = True, O_in=None) -> Dict[str, np.ndarray]:
    """sigma_X (X in dQ, dK, dV), element by element [L, d], of the model in the module docstring.
    With `q_blocks` only those query blocks contribute (dK/dV are then partial, like the
    oracle's attn_bwd with the same argument).  `O_in`: the stored output delta is formed from
    (default: the exact one; the difference only matters for a deliberately different O)."""
    s2 = BF16_U ** 2 / 3.0
    tok = part.block_tokens()
    X = {k: np.asarray(v, dtype=np.float64) for k, v in xi.items()}
    L, d = X["Q"].shape
    var = {k: np.zeros((L, d)) for k in ("dQ", "dK", "dV")}
    for i in (range(part.N) if q_blocks is None else q_blocks):
        rows = tok[i, ix.keep_idx[i]]
        keys = tok[ix.q2k_idx[ix.q2k_ptr[i]:ix.q2k_ptr[i + 1]]].reshape(-1)
        q, k, v = X["Q"][rows], X["K"][keys], X["V"][keys]
        out, _, P = o.attend_block(q, k, v, sm_scale)
        g = o.folded_grad(X["dO"], part, ix.keep_idx, i, tok)
        if O_in is not None:
            out = np.asarray(O_in, dtype=np.float64)[rows]
        dS = P * (g @ v.T - (g * out).sum(axis=1, keepdims=True))
        g2, P2 = g * g, P * P
        vd = (g2 * out * out).sum(axis=1) if own_forward else np.zeros(len(rows))
        var["dV"][keys] += 2.0 * s2 * (P2.T @ g2)
        var["dK"][keys] += s2 * sm_scale ** 2 * ((dS * dS + P2 * (g2 @ (v * v).T) + P2 * vd[:, None]).T @ (q * q))
        vq = (dS * dS) @ (k * k)
        for n in range(len(rows)):
            A = (v * P[n][:, None]).T @ k  # [d, d]
            vq[n] += g2[n] @ (A * A)
        kbar = P @ k
        var["dQ"][rows] = s2 * sm_scale ** 2 * (vq + vd[:, None] * kbar * kbar)
    return {k: np.sqrt(x) for k, x in var.items()}


def rounding_sigma_kv_block(xi: dict, part: o.Partition, ix, sm_scale: float, j: int, own_forward: bool = True):
    """sigma_dK, sigma_dV of rounding_sigma() for the Bk tokens of KV block j alone."""
    s2 = BF16_U ** 2 / 3.0
    tok = part.block_tokens()
    X = {k: np.asarray(v, dtype=np.float64) for k, v in xi.items()}
    kj, vj = X["K"][tok[j]], X["V"][tok[j]]
    vK, vV = np.zeros_like(kj), np.zeros_like(vj)
    for i in ix.k2q_idx[ix.k2q_ptr[j]:ix.k2q_ptr[j + 1]]:
        rows = tok[i, ix.keep_idx[i]]
        keys = tok[ix.q2k_idx[ix.q2k_ptr[i]:ix.q2k_ptr[i + 1]]].reshape(-1)
        q = X["Q"][rows]
        out, lse, _ = o.attend_block(q, X["K"][keys], X["V"][keys], sm_scale)
        g = o.folded_grad(X["dO"], part, ix.keep_idx, int(i), tok)
        Pj = np.exp((q @ kj.T) * sm_scale - lse[:, None])
        dSj = Pj * (g @ vj.T - (g * out).sum(axis=1, keepdims=True))
        g2, P2 = g * g, Pj * Pj
        vd = (g2 * out * out).sum(axis=1) if own_forward else np.zeros(len(rows))
        vK += s2 * sm_scale ** 2 * ((dSj * dSj + P2 * (g2 @ (vj * vj).T) + P2 * vd[:, None]).T @ (q * q))
        vV += 2.0 * s2 * (P2.T @ g2)
    return np.sqrt(vK), np.sqrt(vV)


def figures(got, ref, sigma=None) -> Dict[str, float]:
    """plain: max |got - ref| / RMS(ref);  rms: RMS(got - ref) / RMS(ref);
    excess: max (|got - ref| - u |ref| - 6 sigma) / RMS(ref), floored at 0 (sigma = 0 if not given)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = _rms(ref)
    err = np.abs(got - ref)
    f = {"plain": float(err.max() / rms), "rms": float(np.sqrt(np.mean(err * err)) / rms)}
    slack = BF16_U * np.abs(ref) + (RSS_MULTIPLE * sigma if sigma is not None else 0.0)
    f["excess"] = float(np.maximum(err - slack, 0.0).max() / rms)
    return f


def failures(name: str, f: Dict[str, float], dtype: str):
    """The criteria `f` (figures() of tensor `name`) violates; empty when the tensor passes."""
    bad = []
    if dtype == "fp32":
        if not f["plain"] <= TOL_F32:
            bad.append(f"{name}: max-abs/RMS {f['plain']:.3e} > {TOL_F32}")
        return bad
    if not f["rms"] <= TOL_RMS_BF16:
        bad.append(f"{name}: RMS error / RMS {f['rms']:.3e} > {TOL_RMS_BF16}")
    if not f["excess"] <= TOL_BF16:
        what = "(|err| - u|ref|)/RMS" if name == "O" else f"(|err| - u|ref| - {RSS_MULTIPLE:g} sigma)/RMS"
        bad.append(f"{name}: {what} {f['excess']:.3e} > {TOL_BF16}")
    return bad
