"""CPU oracle for Bidirectional Sparse Attention (BSA).  TEST INFRASTRUCTURE ONLY.

A plain, slow numpy implementation of what the BSA hot path computes, written
from the paper's statement of the method, one head at a time (the paper states
everything "for a single attention head", Sec. 3.1).  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import it; the product path
never does, and this file shares nothing with the HIP sources.

Passages followed (paper section / equation):
  * token <-> grid index map and block partition ....... Sec. 3.1, Sec. 3.2.1
  * block-level representations and inter-block scores .. Sec. 3.2.3
  * minimal cumulative-mass KV-block set ................ Sec. 3.2.3, Eq. 4
  * statistical dynamic threshold (candidate filter) .... Sec. 3.2.3, Eq. 3  (PARITY UNPINNED:
    the equation is ambiguous about U, the std divisor, what p thresholds and how it
    combines with Eq. 4; the reading taken is in select_row's docstring and the design
    notes; the arithmetic of that reading is pinned, the reading itself cannot be)
  * query pruning by cosine similarity to the center .... Sec. 3.2.2, Eq. 2
  * window-based critical tokens ....................... Sec. 3.2.2 ("Critical Token")
  * token filling ...................................... Sec. 3.2.2 ("Token Filling")
  * sparse attention over selected queries / KV blocks .. Sec. 3.2.4, Eq. 5; mask of Sec. 3.1
  * backward ........................................... derived from Eq. 5 + token filling
    (the paper only says separate backward kernels reuse the same masks, Sec. 3.3)

Readings taken where the paper is silent (each is listed with its reason in
the design notes): mean pooling of all tokens of a block; block logits scaled
by 1/sqrt(d); a fixed probability-mass threshold p in Eq. 4 with p >= 1 meaning
"all blocks"; ties broken toward the lower index; the center token is local
coordinate (Ct//2, Ch//2, Cw//2), always kept and counted inside the quota
ceil(r*|block|) (with windows: the same per window, center (Wt//2, Wh//2, Ww//2),
quota ceil(r*|window|), fill from the window's own center); cosine with a zero
vector is 0; the softmax of Eq. 5 is
normalised over the selected keys only; selection and pruning are constants
for the backward pass and the fill copy back-propagates into the center row.

Pins: every function here is checked in tests/test_oracle_pins.py against
something other than itself (dense softmax attention and torch autograd on
the masked dense form, finite differences, brute force over subsets, closed
forms).  What needs the paper's trained activations (the sparsity levels of
its Table 3, any quality number) is "parity unpinned".

Decision arithmetic (pooling sums, block scores, cosine terms) is fp64,
accumulated strictly in index order with separate multiply and add roundings,
so that another implementation that fixes the same order reproduces every
comparison bit for bit.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import ceil, sqrt
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------
# Sec. 3.1 / Sec. 3.2.1: raster index n = t*Hs*Ws + h*Ws + w and 3D blocks
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Partition:
    T: int
    Hs: int
    Ws: int
    Ct: int
    Ch: int
    Cw: int
    # Window of the critical-token mechanism (Sec. 3.2.2 "Critical Token"): every block is
    # cut into windows (Wt, Wh, Ww) that divide it evenly, each with its own center token;
    # 0 means the whole block is one window (a single critical token per block).
    Wt: int = 0
    Wh: int = 0
    Ww: int = 0
    # Token order of the tensors: raster (Sec. 3.1), or after the one-time reorder of
    # Sec. 3.2.1 that makes the tokens of a block adjacent (row i*Bk + c = token c of block i).
    block_major: bool = False

    def __post_init__(self):
        if min(self.T, self.Hs, self.Ws, self.Ct, self.Ch, self.Cw) <= 0:
            raise ValueError("grid and block extents must be positive")
        if self.T % self.Ct or self.Hs % self.Ch or self.Ws % self.Cw:
            raise ValueError("block shape must divide the grid (Sec. 3.2.1)")
        wt, wh, ww = self.window
        if min(wt, wh, ww) <= 0 or self.Ct % wt or self.Ch % wh or self.Cw % ww:
            raise ValueError("window shape must divide the block evenly (Sec. 3.2.2)")

    @property
    def window(self) -> Tuple[int, int, int]:
        return (self.Wt or self.Ct, self.Wh or self.Ch, self.Ww or self.Cw)

    @property
    def Wk(self) -> int:
        """Tokens per window."""
        wt, wh, ww = self.window
        return wt * wh * ww

    @property
    def nwin(self) -> int:
        return self.Bk // self.Wk

    def window_of(self) -> np.ndarray:
        """win[c] = window (numbered raster-wise over the block's window grid) of intra-block token c."""
        wt, wh, ww = self.window
        nh, nw = self.Ch // wh, self.Cw // ww
        win = np.empty(self.Bk, dtype=np.int64)
        for ct in range(self.Ct):
            for ch in range(self.Ch):
                for cw in range(self.Cw):
                    win[(ct * self.Ch + ch) * self.Cw + cw] = ((ct // wt) * nh + ch // wh) * nw + cw // ww
        return win

    def centers(self) -> np.ndarray:
        """cen[w] = intra-block id of the critical token of window w: local coordinate
        (Wt//2, Wh//2, Ww//2) inside the window."""
        wt, wh, ww = self.window
        nt, nh, nw = self.Ct // wt, self.Ch // wh, self.Cw // ww
        cen = np.empty(self.nwin, dtype=np.int64)
        for a in range(nt):
            for b in range(nh):
                for c in range(nw):
                    ct, ch, cw = a * wt + wt // 2, b * wh + wh // 2, c * ww + ww // 2
                    cen[(a * nh + b) * nw + c] = (ct * self.Ch + ch) * self.Cw + cw
        return cen

    def center_of(self) -> np.ndarray:
        """For every intra-block token, the intra-block id of its window's critical token."""
        return self.centers()[self.window_of()]

    @property
    def L(self) -> int:
        return self.T * self.Hs * self.Ws

    @property
    def Bk(self) -> int:
        return self.Ct * self.Ch * self.Cw

    @property
    def nblk(self) -> Tuple[int, int, int]:
        return (self.T // self.Ct, self.Hs // self.Ch, self.Ws // self.Cw)

    @property
    def N(self) -> int:
        nt, nh, nw = self.nblk
        return nt * nh * nw

    @property
    def center(self) -> int:
        """Intra-block id of the critical (center) token of a block that is one window."""
        if self.nwin != 1:
            raise ValueError("a block with several windows has several critical tokens: use centers()")
        return (self.Ct // 2) * self.Ch * self.Cw + (self.Ch // 2) * self.Cw + (self.Cw // 2)

    def n_keep_window(self, r: float) -> int:
        """Retained tokens per window: ceil(r * |window|) (Eq. 2 applied per window)."""
        if not (0.0 < r <= 1.0):
            raise ValueError("retained ratio r must lie in (0, 1] (Eq. 2)")
        return int(ceil(r * self.Wk - 1e-12))

    def n_keep(self, r: float) -> int:
        """Retained tokens per block: the windows' quotas concatenated."""
        return self.nwin * self.n_keep_window(r)

    def block_tokens(self) -> np.ndarray:
        """tok[i, c] = row (raster index, or i*Bk + c in block-major order) of intra-block token c of block i.

        Blocks are numbered raster-wise over the block grid, tokens raster-wise
        inside the block."""
        nt, nh, nw = self.nblk
        if self.block_major:
            return np.arange(self.N * self.Bk, dtype=np.int64).reshape(self.N, self.Bk)
        tok = np.empty((self.N, self.Bk), dtype=np.int64)
        for bt in range(nt):
            for bh in range(nh):
                for bw in range(nw):
                    i = (bt * nh + bh) * nw + bw
                    c = 0
                    for ct in range(self.Ct):
                        for ch in range(self.Ch):
                            for cw in range(self.Cw):
                                t = bt * self.Ct + ct
                                h = bh * self.Ch + ch
                                w = bw * self.Cw + cw
                                tok[i, c] = (t * self.Hs + h) * self.Ws + w
                                c += 1
        return tok


def _seq_sum(x: np.ndarray, axis: int) -> np.ndarray:
    """Sum along `axis` strictly in index order (numpy's own sum is pairwise)."""
    x = np.moveaxis(np.asarray(x, dtype=np.float64), axis, 0)
    acc = np.zeros(x.shape[1:], dtype=np.float64)
    for k in range(x.shape[0]):
        acc = acc + x[k]
    return acc


def _seq_dot(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """sum_c a[..., c] * b[..., c] in fp64, c ascending, product rounded before the add."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    acc = np.zeros(np.broadcast_shapes(a.shape[:-1], b.shape[:-1]), dtype=np.float64)
    for c in range(a.shape[-1]):
        acc = acc + a[..., c] * b[..., c]
    return acc


# --------------------------------------------------------------------------
# Sec. 3.2.3: block-level representations (mean pooling) and block scores
# --------------------------------------------------------------------------
def pool_blocks(X: np.ndarray, part: Partition) -> np.ndarray:
    """Xbar[i, :] = mean of the Bk token vectors of block i.  X: [L, d]."""
    tok = part.block_tokens()
    Xb = np.asarray(X, dtype=np.float64)[tok]  # [N, Bk, d]
    return _seq_sum(Xb, axis=1) / np.float64(part.Bk)


def block_scores(Qbar: np.ndarray, Kbar: np.ndarray, score_scale: float) -> np.ndarray:
    """s[i, j] = score_scale * <Qbar_i, Kbar_j>  (the logits inside Eq. 4)."""
    return _seq_dot(Qbar[:, None, :], Kbar[None, :, :]) * np.float64(score_scale)


# --------------------------------------------------------------------------
# Eq. 4: minimal index set whose softmax mass reaches p
# --------------------------------------------------------------------------
@dataclass
class RowSelection:
    idx: np.ndarray  # selected KV block ids, ascending
    k: int  # |S_i|
    margin: float  # distance of the deciding comparisons from equality, relative to Z


def stat_quantile(k: int, n: int) -> float:
    """U(1 - k/n) of Eq. 3 with U read as the quantile function of the standard normal
    distribution: the z for which about k of n normally distributed scores exceed
    mean + z * std.  k = n gives -inf (no score is excluded)."""
    if not (1 <= k <= n):
        raise ValueError("Eq. 3 needs 1 <= k <= n")
    if k == n:
        return float("-inf")
    from statistics import NormalDist

    return NormalDist().inv_cdf(1.0 - k / n)


def stat_threshold(s: np.ndarray, z: float) -> float:
    """Eq. 3: mean(s) + std(s) * z, std with the n-1 divisor (0 for a single score)."""
    s = np.asarray(s, dtype=np.float64)
    if z == float("-inf"):
        return float("-inf")
    std = float(np.std(s, ddof=1)) if s.shape[0] > 1 else 0.0
    return float(np.mean(s)) + std * float(z)


def select_row(s: np.ndarray, p: float, z: Optional[float] = None) -> RowSelection:
    """Minimal prefix, in descending score order, with cumulative mass >= p.

    Order: score descending, ties by lower block id.  Mass is accumulated in
    that order; the test is c_k >= p * Z with Z the total of the same
    accumulation.  p >= 1 selects every block.

    With `z` (Eq. 3, statistical dynamic threshold) only the blocks whose score
    reaches tau = mean(s) + std(s) * z are candidates: the prefix is cut to the
    candidates (they are themselves a prefix of the order); if none qualifies the
    single best block is kept.  The softmax of Eq. 4 stays normalised over all
    blocks, as printed.  The margin then also covers the comparisons with tau,
    relative to |tau| + std."""
    if not (0.0 < p <= 1.0):
        raise ValueError("mass threshold p must lie in (0, 1]")
    s = np.asarray(s, dtype=np.float64)
    n = s.shape[0]
    order = np.lexsort((np.arange(n), -s))  # primary key -s, secondary key j
    e = np.exp(s[order] - s[order[0]])
    c = np.cumsum(e)  # sequential accumulation in sorted order
    Z = c[-1]
    if p >= 1.0:
        k, margin = n, float("inf")
    else:
        target = np.float64(p) * Z
        k = int(np.argmax(c >= target)) + 1  # first k with c_k >= p Z  (c_n = Z >= pZ)
        margin = (c[k - 1] - target) / Z
        if k >= 2:
            margin = min(margin, (target - c[k - 2]) / Z)
    if z is not None and z != float("-inf"):
        tau = stat_threshold(s, z)
        cand = int(np.count_nonzero(s >= tau))
        k = min(k, max(cand, 1))
        std = float(np.std(s, ddof=1)) if n > 1 else 0.0
        margin = min(float(margin), float(np.abs(s - tau).min() / (abs(tau) + std + 1e-300)))
    return RowSelection(np.sort(order[:k]).astype(np.int32), k, float(margin))


def select_kv(scores: np.ndarray, p: float, z: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray, float]:
    """CSR (q2k_ptr[N+1], q2k_idx[nnz]) of Eq. 4 (optionally behind Eq. 3's candidate
    filter) for one head, plus the smallest margin."""
    n_rows = scores.shape[0]
    ptr = np.zeros(n_rows + 1, dtype=np.int32)
    cols: List[np.ndarray] = []
    margin = float("inf")
    for i in range(n_rows):
        sel = select_row(scores[i], p, z)
        cols.append(sel.idx)
        ptr[i + 1] = ptr[i] + sel.k
        margin = min(margin, sel.margin)
    return ptr, np.concatenate(cols).astype(np.int32), margin


def transpose_csr(ptr: np.ndarray, idx: np.ndarray, n_cols: int) -> Tuple[np.ndarray, np.ndarray]:
    """k2q lists: for each KV block j, the query blocks i with j in S_i, ascending."""
    lists: List[List[int]] = [[] for _ in range(n_cols)]
    for i in range(len(ptr) - 1):
        for j in idx[ptr[i]:ptr[i + 1]]:
            lists[int(j)].append(i)
    tptr = np.zeros(n_cols + 1, dtype=np.int32)
    for j in range(n_cols):
        tptr[j + 1] = tptr[j] + len(lists[j])
    tidx = np.array([i for l in lists for i in l], dtype=np.int32)
    return tptr, tidx


# --------------------------------------------------------------------------
# Eq. 2: keep the ceil(r*Bk) tokens least similar to the block's center
# --------------------------------------------------------------------------
def cosine_to_center(Q: np.ndarray, part: Partition) -> np.ndarray:
    """cos[i, c] between token c of block i and the center token of c's window."""
    tok = part.block_tokens()
    cof = part.center_of()
    Qb = np.asarray(Q, dtype=np.float64)[tok]  # [N, Bk, d]
    qc = Qb[:, cof, :]
    dot = _seq_dot(Qb, qc)
    nrm = _seq_dot(Qb, Qb)
    nc = nrm[:, cof]
    den = np.sqrt(nrm * nc)
    cos = np.zeros_like(dot)
    np.divide(dot, den, out=cos, where=den > 0.0)  # zero-norm vector: cos := 0
    return cos


def prune_q(Q: np.ndarray, part: Partition, r: float) -> Tuple[np.ndarray, float]:
    """keep_idx[i, :] = ascending intra-block ids of the retained queries of block i.

    Per window: its center is always retained and counts toward the window's quota
    kw = ceil(r*|window|); the other kw-1 are the window's tokens with the smallest
    cosine to that center (ties: lower id first).  The windows' selections are
    concatenated.  Also returns the smallest gap between the last kept and the
    first pruned cosine of any window."""
    kw = part.n_keep_window(r)
    cos = cosine_to_center(Q, part)
    win, cen = part.window_of(), part.centers()
    keep = np.empty((part.N, part.nwin * kw), dtype=np.int32)
    gap = float("inf")
    for i in range(part.N):
        sel = []
        for w in range(part.nwin):
            others = np.array([c for c in range(part.Bk) if win[c] == w and c != cen[w]], dtype=np.int64)
            sel.append(cen[w])
            if len(others) == 0:
                continue
            order = others[np.lexsort((others, cos[i, others]))]  # cosine ascending, then id ascending
            sel.extend(order[: kw - 1])
            if 1 <= kw - 1 < len(order):
                gap = min(gap, float(cos[i, order[kw - 1]] - cos[i, order[kw - 2]]))
        keep[i] = np.sort(np.array(sel))
    return keep, gap


# --------------------------------------------------------------------------
# Eq. 5 + token filling: forward
# --------------------------------------------------------------------------
def attend_block(q: np.ndarray, Ksel: np.ndarray, Vsel: np.ndarray, sm_scale: float):
    """Exact softmax attention of rows q over the given keys.  Returns (o, lse, P)."""
    s = (q @ Ksel.T) * q.dtype.type(sm_scale)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    P = e / z
    return P @ Vsel, (m + np.log(z))[:, 0], P


def attn_fwd(Q, K, V, part: Partition, q2k_ptr, q2k_idx, keep_idx, sm_scale: float,
             dtype=np.float64, q_blocks: Optional[Sequence[int]] = None):
    """Sparse attention forward for one head, block-list form.

    For each query block i: the retained tokens attend to every token of every
    KV block in S_i (Eq. 5); each pruned token then takes its block center's
    output and log-sum-exp (token filling).  Returns O[L, d], LSE[L]; if
    `q_blocks` is given only those blocks' rows are computed (others stay 0)."""
    tok = part.block_tokens()
    cof = part.center_of()
    Q = np.asarray(Q, dtype=dtype)
    K = np.asarray(K, dtype=dtype)
    V = np.asarray(V, dtype=dtype)
    O = np.zeros_like(Q)
    LSE = np.zeros(Q.shape[0], dtype=dtype)
    for i in (range(part.N) if q_blocks is None else q_blocks):
        rows = tok[i, keep_idx[i]]
        keys = tok[q2k_idx[q2k_ptr[i]:q2k_ptr[i + 1]]].reshape(-1)
        o, lse, _ = attend_block(Q[rows], K[keys], V[keys], sm_scale)
        cpos = np.searchsorted(keep_idx[i], cof)  # position of each token's window center among the retained rows
        O[tok[i]] = o[cpos]  # fill every token with its window center's output ...
        LSE[tok[i]] = lse[cpos]
        O[rows] = o  # ... then overwrite the retained ones with their own
        LSE[rows] = lse
    return O, LSE


def dense_mask(part: Partition, q2k_ptr, q2k_idx) -> np.ndarray:
    """Token-level mask M in {-inf, 0}^{L x L} of Sec. 3.1 induced by the block lists."""
    tok = part.block_tokens()
    M = np.full((part.L, part.L), -np.inf)
    for i in range(part.N):
        keys = tok[q2k_idx[q2k_ptr[i]:q2k_ptr[i + 1]]].reshape(-1)
        M[np.ix_(tok[i], keys)] = 0.0
    return M


def attn_fwd_dense_masked(Q, K, V, part: Partition, q2k_ptr, q2k_idx, keep_idx, sm_scale: float):
    """Second form of the forward: full L x L masked softmax, then filling (small L only)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S = (Q @ K.T) * sm_scale + dense_mask(part, q2k_ptr, q2k_idx)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    z = E.sum(axis=1, keepdims=True)
    O = (E / z) @ V
    LSE = (m + np.log(z))[:, 0]
    src = fill_source(part, keep_idx)
    return O[src], LSE[src]


def fill_source(part: Partition, keep_idx) -> np.ndarray:
    """src[n] = n for a retained token, the raster index of its window's center otherwise."""
    tok = part.block_tokens()
    cof = part.center_of()
    src = np.empty(part.L, dtype=np.int64)
    for i in range(part.N):
        src[tok[i]] = tok[i, cof]
        src[tok[i, keep_idx[i]]] = tok[i, keep_idx[i]]
    return src


# --------------------------------------------------------------------------
# backward of (Eq. 5 + token filling), indices held constant
# --------------------------------------------------------------------------
def folded_grad(dO: np.ndarray, part: Partition, keep_idx, i: int, tok=None) -> np.ndarray:
    """g for the retained rows of block i: dO of the row itself, and for a window's
    center additionally the dO of every pruned token of that window (it was copied to them)."""
    tok = part.block_tokens() if tok is None else tok
    cof = part.center_of()
    g = np.array(dO[tok[i, keep_idx[i]]])
    pruned = np.setdiff1d(np.arange(part.Bk), keep_idx[i])
    for c in pruned:  # ascending intra-block id
        cpos = int(np.searchsorted(keep_idx[i], cof[c]))
        g[cpos] = g[cpos] + dO[tok[i, c]]
    return g


def attn_bwd(Q, K, V, dO, part: Partition, q2k_ptr, q2k_idx, keep_idx, sm_scale: float,
             dtype=np.float64, q_blocks: Optional[Sequence[int]] = None, O_in=None):
    """dQ, dK, dV for one head.

    With P = softmax(sm_scale * q k^T) over the selected keys, o = P v and g the
    folded upstream gradient:  delta_n = <g_n, o_n>;  dV += P^T g;
    dS = P * (g v^T - delta);  dQ = sm_scale * dS k;  dK += sm_scale * dS^T q.
    Rows of pruned queries get dQ = 0.  If `q_blocks` is given, only those
    query blocks contribute (dK/dV are then partial sums).

    `O_in` [L, d]: the forward output as a caller stored it (possibly rounded to
    the storage type).  A backward entry point receives O as an argument, and
    delta is then formed from that stored O; None means the exact o."""
    tok = part.block_tokens()
    Q = np.asarray(Q, dtype=dtype)
    K = np.asarray(K, dtype=dtype)
    V = np.asarray(V, dtype=dtype)
    dO = np.asarray(dO, dtype=dtype)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for i in (range(part.N) if q_blocks is None else q_blocks):
        rows = tok[i, keep_idx[i]]
        keys = tok[q2k_idx[q2k_ptr[i]:q2k_ptr[i + 1]]].reshape(-1)
        q, k, v = Q[rows], K[keys], V[keys]
        o, _, P = attend_block(q, k, v, sm_scale)
        if O_in is not None:
            o = np.asarray(O_in, dtype=dtype)[rows]
        g = folded_grad(dO, part, keep_idx, i, tok)
        delta = (g * o).sum(axis=1, keepdims=True)
        dS = P * (g @ v.T - delta)
        dQ[rows] = (dS @ k) * dtype(sm_scale)
        dK[keys] += (dS.T @ q) * dtype(sm_scale)  # keys of one list are distinct
        dV[keys] += P.T @ g
    return dQ, dK, dV


def attn_bwd_kv_block(Q, K, V, dO, part: Partition, q2k_ptr, q2k_idx, k2q_ptr, k2q_idx,
                      keep_idx, sm_scale: float, j: int, dtype=np.float64, O_in=None):
    """dK, dV of the Bk tokens of KV block j alone (sum over the query blocks that list j)."""
    tok = part.block_tokens()
    Q = np.asarray(Q, dtype=dtype)
    K = np.asarray(K, dtype=dtype)
    V = np.asarray(V, dtype=dtype)
    dO = np.asarray(dO, dtype=dtype)
    kj, vj = K[tok[j]], V[tok[j]]
    dKj = np.zeros_like(kj)
    dVj = np.zeros_like(vj)
    for i in k2q_idx[k2q_ptr[j]:k2q_ptr[j + 1]]:
        rows = tok[i, keep_idx[i]]
        keys = tok[q2k_idx[q2k_ptr[i]:q2k_ptr[i + 1]]].reshape(-1)
        q = Q[rows]
        o, lse, _ = attend_block(q, K[keys], V[keys], sm_scale)
        if O_in is not None:
            o = np.asarray(O_in, dtype=dtype)[rows]
        g = folded_grad(dO, part, keep_idx, int(i), tok)
        delta = (g * o).sum(axis=1, keepdims=True)
        Pj = np.exp((q @ kj.T) * dtype(sm_scale) - lse[:, None])
        dSj = Pj * (g @ vj.T - delta)
        dKj += (dSj.T @ q) * dtype(sm_scale)
        dVj += Pj.T @ g
    return dKj, dVj


# --------------------------------------------------------------------------
# whole pipeline for one head
# --------------------------------------------------------------------------
@dataclass
class HeadResult:
    Qbar: np.ndarray
    Kbar: np.ndarray
    q2k_ptr: np.ndarray
    q2k_idx: np.ndarray
    k2q_ptr: np.ndarray
    k2q_idx: np.ndarray
    keep_idx: np.ndarray
    select_margin: float
    prune_gap: float


def bsa_indices(Q, K, part: Partition, threshold: float, keep_ratio: float,
                score_scale: Optional[float] = None, stat_z: Optional[float] = None) -> HeadResult:
    """Pool -> block scores -> (Eq. 3 filter ->) Eq. 4 selection, and Eq. 2 pruning, for one head."""
    d = Q.shape[1]
    score_scale = 1.0 / sqrt(d) if score_scale is None else score_scale
    Qbar = pool_blocks(Q, part)
    Kbar = pool_blocks(K, part)
    ptr, idx, margin = select_kv(block_scores(Qbar, Kbar, score_scale), threshold, stat_z)
    tptr, tidx = transpose_csr(ptr, idx, part.N)
    keep, gap = prune_q(Q, part, keep_ratio)
    return HeadResult(Qbar, Kbar, ptr, idx, tptr, tidx, keep, margin, gap)


def bsa_head(Q, K, V, dO, part: Partition, threshold: float, keep_ratio: float,
             sm_scale: Optional[float] = None, dtype=np.float64, o_storage=None):
    """Full fwd+bwd of one head.  Returns (indices, O, LSE, dQ, dK, dV).

    `o_storage`: optional function modelling how O is stored between the two
    passes (e.g. rounding to bfloat16); the backward then reads that stored O."""
    sm_scale = 1.0 / sqrt(Q.shape[1]) if sm_scale is None else sm_scale
    ix = bsa_indices(Q, K, part, threshold, keep_ratio)
    O, LSE = attn_fwd(Q, K, V, part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, sm_scale, dtype)
    O_in = None if o_storage is None else o_storage(O)
    dQ, dK, dV = attn_bwd(Q, K, V, dO, part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, sm_scale, dtype, O_in=O_in)
    return ix, O, LSE, dQ, dK, dV
