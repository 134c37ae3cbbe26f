"""Pins for the CPU oracle: each check compares it with something that is not
the oracle itself (a textbook definition, a library's autograd, brute force,
a closed form, a finite difference), so that a dropped term, wrong sign, wrong
index or transposed operand in the oracle fails here.  All CPU, no GPU."""
import itertools
from math import ceil, sqrt

import numpy as np
import pytest
import torch

from bsa_workloads import WORKLOADS, head_inputs
from oracle import bsa_oracle as o

TINY = WORKLOADS["tiny"]


def tiny_part():
    return o.Partition(*TINY.grid, *TINY.block)


def tiny_inputs(h=0, dtype=np.float64):
    x = head_inputs(TINY, 0, h)
    return {k: v.astype(dtype) for k, v in x.items()}


# ---------------------------------------------------------------- partition
def test_partition_is_a_bijection_with_raster_formula():
    part = o.Partition(4, 6, 8, 2, 3, 4)
    tok = part.block_tokens()
    assert tok.shape == (part.N, part.Bk) == (8, 24)
    assert sorted(tok.reshape(-1).tolist()) == list(range(part.L))
    # n = t*Hs*Ws + h*Ws + w (Sec. 3.1): block (1,0,1), local (1,2,3)
    i = (1 * 2 + 0) * 2 + 1
    c = (1 * 3 + 2) * 4 + 3
    t, h, w = 1 * 2 + 1, 0 * 3 + 2, 1 * 4 + 3
    assert tok[i, c] == t * 6 * 8 + h * 8 + w
    # tokens adjacent along w inside a block are adjacent in the sequence
    assert np.all(np.diff(tok[:, :4], axis=1) == 1)


def test_partition_rejects_non_dividing_blocks():
    with pytest.raises(ValueError):
        o.Partition(4, 6, 8, 3, 3, 4)


def test_center_token_of_the_papers_block_shapes():
    assert o.Partition(4, 4, 4, 4, 4, 4).center == 42  # local (2,2,2)
    assert tiny_part().center == 26  # local (1,2,2) of a 2x4x4 block


def test_paper_default_keep_count():
    # Sec. 4.1 "Implement Details": r = 0.5 on 4x4x4 blocks gives a query block of 32
    lines = open(__file__.replace("test_oracle_pins.py", "golden/paper_constants.txt")).read().split("\n")
    vals = dict(l.split("=")[0:2] for l in lines if "=" in l and not l.startswith("#"))
    part = o.Partition(4, 4, 4, 4, 4, 4)
    assert part.n_keep(float(vals["keep_ratio"])) == int(vals["query_block_size"].split()[0])
    # Table 3: query sparsity 0.5 and KV sparsity 0.86 compose to 0.93 = 1 - r*f
    r, f = 1 - float(vals["sparse_query_sparsity"]), 1 - float(vals["sparse_kv_sparsity"])
    assert round(1 - r * f, 2) == float(vals["combined_sparsity"].split()[0])


# ------------------------------------------------------------------ pooling
def test_pool_dot_equals_mean_of_token_logits():
    part = tiny_part()
    x = tiny_inputs()
    Qb, Kb = o.pool_blocks(x["Q"], part), o.pool_blocks(x["K"], part)
    tok = part.block_tokens()
    logits = x["Q"] @ x["K"].T
    for i, j in [(0, 0), (3, 5), (7, 1)]:
        mean_logit = logits[np.ix_(tok[i], tok[j])].mean()
        assert abs(Qb[i] @ Kb[j] - mean_logit) < 1e-10
    s = o.block_scores(Qb, Kb, 0.125)
    assert np.allclose(s, 0.125 * (Qb @ Kb.T), rtol=0, atol=1e-12)
    assert not np.allclose(s, s.T)  # a transposed operand would show


def test_pool_of_blockwise_constant_field():
    part = o.Partition(4, 4, 8, 2, 2, 4)
    tok = part.block_tokens()
    X = np.zeros((part.L, 3))
    for i in range(part.N):
        X[tok[i]] = [i, -i, 0.5]
    Xb = o.pool_blocks(X, part)
    assert np.array_equal(Xb[:, 0], np.arange(part.N))
    assert np.array_equal(Xb[:, 1], -np.arange(part.N))


# ---------------------------------------------------------------- selection
def _brute_force_min_set(s, p):
    e = np.exp(s - s.max())
    prob = e / e.sum()
    n = len(s)
    for size in range(1, n + 1):
        best = max(itertools.combinations(range(n), size), key=lambda c: prob[list(c)].sum())
        if prob[list(best)].sum() >= p:
            return size, prob[list(best)].sum()
    raise AssertionError


@pytest.mark.parametrize("p", [0.3, 0.5, 0.8, 0.9, 0.95, 0.999])
def test_select_is_minimal_and_maximal_mass_by_brute_force(p):
    part = tiny_part()
    x = tiny_inputs(1)
    s = o.block_scores(o.pool_blocks(x["Q"], part), o.pool_blocks(x["K"], part), 1 / sqrt(TINY.d)) * 6.0
    for i in range(part.N):
        sel = o.select_row(s[i], p)
        size, mass = _brute_force_min_set(s[i], p)
        assert sel.k == size
        prob = np.exp(s[i] - s[i].max())
        prob /= prob.sum()
        assert abs(prob[sel.idx].sum() - mass) < 1e-12
        assert prob[sel.idx].sum() >= p - 1e-12
        assert np.all(np.diff(sel.idx) > 0)


def test_select_closed_forms():
    n = 10
    for p in (0.05, 0.31, 0.5, 0.9):
        sel = o.select_row(np.zeros(n), p)  # uniform: ceil(p n) lowest ids
        assert sel.k == ceil(p * n - 1e-12)
        assert sel.idx.tolist() == list(range(sel.k))
    s = np.zeros(n)
    s[7] = 50.0  # one dominant block
    sel = o.select_row(s, 0.99)
    assert sel.idx.tolist() == [7]
    assert o.select_row(np.random.default_rng(0).normal(size=n), 1.0).k == n
    # two-point row: masses 0.75 / 0.25
    s2 = np.array([0.0, np.log(3.0)])
    assert o.select_row(s2, 0.7).idx.tolist() == [1]
    assert o.select_row(s2, 0.8).idx.tolist() == [0, 1]


def test_select_nesting_and_tie_break():
    rng = np.random.default_rng(1)
    s = rng.normal(size=40) * 2
    prev = set()
    for p in (0.2, 0.5, 0.8, 0.9, 0.97, 1.0):
        cur = set(o.select_row(s, p).idx.tolist())
        assert prev <= cur
        prev = cur
    s = np.array([1.0, 2.0, 2.0, 2.0, 0.0])  # ties go to the lower id
    assert o.select_row(s, 0.5).idx.tolist() == [1, 2]


def test_select_margin_closed_form_and_boundary_nudges():
    """The margin a row reports is how far its deciding comparisons are from equality, relative
    to the row's total mass Z: min(c_k - pZ, pZ - c_{k-1}) / Z at the cut k (only the first term
    when k = 1).  Pinned by the two-block closed form and by moving the threshold itself: the
    selection must survive p -> p -+ 0.99 margin and must change at p + 1.01 (c_k - pZ)/Z or
    p - 1.01 (pZ - c_{k-1})/Z."""
    # two blocks with masses e1 > e2: Z = e1 + e2, c_1 = e1
    s = np.log(np.array([3.0, 1.0]))
    for p, k, m in ((0.5, 1, 0.25), (0.7, 1, 0.05), (0.8, 2, 0.05), (0.9, 2, 0.1)):
        sel = o.select_row(s, p)
        assert sel.k == k and sel.margin == pytest.approx(m, rel=1e-12), (p, sel)
    assert o.select_row(s, 1.0).margin == float("inf")
    rng = np.random.default_rng(5)
    for trial in range(20):
        s = rng.normal(size=8) * 1.5
        p = float(rng.uniform(0.2, 0.95))
        sel = o.select_row(s, p)
        order = np.lexsort((np.arange(8), -s))
        c = np.cumsum(np.exp(s[order] - s[order[0]]))
        Z = c[-1]
        up = (c[sel.k - 1] - p * Z) / Z            # room before one more block is needed
        down = (p * Z - c[sel.k - 2]) / Z if sel.k >= 2 else float("inf")  # room before one block fewer suffices
        assert sel.margin == pytest.approx(min(up, down), rel=1e-9)
        for dp in (-0.99 * sel.margin, 0.99 * sel.margin):
            if 0.0 < p + dp < 1.0:
                assert o.select_row(s, p + dp).k == sel.k
        if p + 1.01 * up < 1.0:
            assert o.select_row(s, p + 1.01 * up).k == sel.k + 1
        if sel.k >= 2 and p - 1.01 * down > 0.0:
            assert o.select_row(s, p - 1.01 * down).k == sel.k - 1
    # select_kv reports the smallest margin of its rows
    S = rng.normal(size=(6, 8))
    assert o.select_kv(S, 0.8)[2] == min(o.select_row(S[i], 0.8).margin for i in range(6))


def test_select_rejects_bad_threshold():
    for p in (0.0, -0.1, 1.5):
        with pytest.raises(ValueError):
            o.select_row(np.zeros(4), p)


def test_transpose_csr_roundtrip_and_counts():
    rng = np.random.default_rng(2)
    s = rng.normal(size=(12, 12)) * 3
    ptr, idx, _ = o.select_kv(s, 0.8)
    tptr, tidx = o.transpose_csr(ptr, idx, 12)
    assert tptr[-1] == ptr[-1] == len(idx) == len(tidx)
    dense = np.zeros((12, 12), bool)
    for i in range(12):
        dense[i, idx[ptr[i]:ptr[i + 1]]] = True
    denseT = np.zeros((12, 12), bool)
    for j in range(12):
        denseT[j, tidx[tptr[j]:tptr[j + 1]]] = True
        assert np.all(np.diff(tidx[tptr[j]:tptr[j + 1]]) > 0)
    assert np.array_equal(dense.T, denseT)
    p2, i2 = o.transpose_csr(tptr, tidx, 12)
    assert np.array_equal(p2, ptr) and np.array_equal(i2, idx)


# ------------------------------------------------------------------ pruning
def test_cosine_matches_definition():
    part = tiny_part()
    x = tiny_inputs()
    cos = o.cosine_to_center(x["Q"], part)
    tok = part.block_tokens()
    for i, c in [(0, 0), (2, 31), (5, 26), (7, 13)]:
        a, b = x["Q"][tok[i, c]], x["Q"][tok[i, part.center]]
        assert abs(cos[i, c] - a @ b / (np.linalg.norm(a) * np.linalg.norm(b))) < 1e-12
    assert np.allclose(cos[:, part.center], 1.0)


@pytest.mark.parametrize("r", [0.25, 0.5, 0.75, 1.0, 1 / 32])
def test_prune_invariants(r):
    part = tiny_part()
    x = tiny_inputs()
    keep, _ = o.prune_q(x["Q"], part, r)
    cos = o.cosine_to_center(x["Q"], part)
    n_keep = ceil(r * part.Bk - 1e-12)
    assert keep.shape == (part.N, n_keep)
    for i in range(part.N):
        ks = keep[i].tolist()
        assert ks == sorted(set(ks)) and part.center in ks
        pruned = [c for c in range(part.Bk) if c not in ks]
        kept_others = [c for c in ks if c != part.center]
        if pruned and kept_others:  # the least similar tokens are the retained ones
            assert cos[i, kept_others].max() <= cos[i, pruned].min()
    if r == 1.0:
        assert np.array_equal(keep, np.tile(np.arange(part.Bk), (part.N, 1)))


def test_prune_gap_is_the_distance_between_the_last_kept_and_the_first_pruned_cosine():
    """prune_q's second result: over all windows, the smallest difference between the first
    pruned cosine and the last retained one (ascending order, center aside).  Zero exactly when
    some decision was a tie; positive means every keep list was decided by a strict inequality."""
    part = tiny_part()
    x = tiny_inputs()
    for r in (0.25, 0.5, 0.75):
        keep, gap = o.prune_q(x["Q"], part, r)
        cos = o.cosine_to_center(x["Q"], part)
        want = float("inf")
        for i in range(part.N):
            kept = [c for c in keep[i] if c != part.center]
            pruned = [c for c in range(part.Bk) if c not in keep[i]]
            want = min(want, cos[i, pruned].min() - cos[i, kept].max())
        assert gap == pytest.approx(want, abs=0.0) and gap > 0.0
    assert o.prune_q(np.ones((part.L, 8)), part, 0.25)[1] == 0.0  # identical tokens: every decision a tie
    assert o.prune_q(x["Q"], part, 1.0)[1] == float("inf")       # nothing pruned: nothing decided
    assert o.bsa_indices(x["Q"], x["K"], part, 0.9, 0.5).prune_gap == o.prune_q(x["Q"], part, 0.5)[1]


def test_prune_identical_tokens_and_zero_vectors():
    part = tiny_part()
    Q = np.ones((part.L, 8))
    keep, _ = o.prune_q(Q, part, 0.25)  # all cos == 1: center + lowest ids
    assert keep[0].tolist() == list(range(7)) + [part.center]
    Q = np.ones((part.L, 8))
    tok = part.block_tokens()
    Q[tok[0, 30]] = 0.0  # zero vector: cos := 0, the least similar
    Q[tok[0, 29]] = -1.0  # cos = -1, even less similar
    keep, _ = o.prune_q(Q, part, 3 / 32)
    assert keep[0].tolist() == [26, 29, 30]


# ---------------------------------------------------- attention, both forms
def _torch_dense(Q, K, V, dO, scale, M=None, src=None):
    q, k, v = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (Q, K, V))
    S = q @ k.T * scale
    if M is not None:
        S = S + torch.tensor(M)
    out = torch.softmax(S, dim=1) @ v
    lse = torch.logsumexp(S, dim=1)
    if src is not None:
        out, lse = out[torch.tensor(src)], lse[torch.tensor(src)]
    (out * torch.tensor(dO, dtype=torch.float64)).sum().backward()
    return out.detach().numpy(), lse.detach().numpy(), q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


def test_threshold_one_no_pruning_is_full_softmax_attention():
    part = tiny_part()
    x = tiny_inputs()
    scale = 1 / sqrt(TINY.d)
    ix, O, LSE, dQ, dK, dV = o.bsa_head(x["Q"], x["K"], x["V"], x["dO"], part, 1.0, 1.0)
    assert np.array_equal(np.diff(ix.q2k_ptr), np.full(part.N, part.N))
    tO, tL, tdQ, tdK, tdV = _torch_dense(x["Q"], x["K"], x["V"], x["dO"], scale)
    for a, b in ((O, tO), (LSE, tL), (dQ, tdQ), (dK, tdK), (dV, tdV)):
        assert np.abs(a - b).max() < 1e-12 * max(1.0, np.abs(b).max())


@pytest.mark.parametrize("p,r", [(0.9, 0.5), (0.5, 0.25), (0.3, 1.0), (1.0, 0.5)])
def test_sparse_fwd_bwd_against_autograd_of_masked_dense_form(p, r):
    """Mask of Sec. 3.1 + token filling written with torch ops; autograd supplies
    the gradients, including the fill copy's gradient into the center row."""
    part = tiny_part()
    x = tiny_inputs(1)
    x["Q"], x["K"] = x["Q"] * 3.0, x["K"] * 3.0  # sharper block scores: p actually prunes
    scale = 1 / sqrt(TINY.d)
    ix, O, LSE, dQ, dK, dV = o.bsa_head(x["Q"], x["K"], x["V"], x["dO"], part, p, r)
    if p < 1.0:
        assert ix.q2k_ptr[-1] < part.N * part.N
    M = o.dense_mask(part, ix.q2k_ptr, ix.q2k_idx)
    src = o.fill_source(part, ix.keep_idx)
    tO, tL, tdQ, tdK, tdV = _torch_dense(x["Q"], x["K"], x["V"], x["dO"], scale, M, src)
    for a, b in ((O, tO), (LSE, tL), (dQ, tdQ), (dK, tdK), (dV, tdV)):
        assert np.abs(a - b).max() < 1e-11 * max(1.0, np.abs(b).max())
    O2, L2 = o.attn_fwd_dense_masked(x["Q"], x["K"], x["V"], part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale)
    assert np.abs(O - O2).max() < 1e-12 and np.abs(LSE - L2).max() < 1e-12


def test_forward_invariants():
    part = tiny_part()
    x = tiny_inputs()
    x["Q"], x["K"] = x["Q"] * 3.0, x["K"] * 3.0
    scale = 1 / sqrt(TINY.d)
    ix = o.bsa_indices(x["Q"], x["K"], part, 0.6, 0.5)
    args = (part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale)
    O, LSE = o.attn_fwd(x["Q"], x["K"], x["V"], *args)
    # constant values -> constant output (softmax normalised over the selected set)
    v0 = np.linspace(-1, 1, TINY.d)
    Oc, _ = o.attn_fwd(x["Q"], x["K"], np.tile(v0, (part.L, 1)), *args)
    assert np.abs(Oc - v0).max() < 1e-13
    # K -> K + u shifts logits and LSE by scale*q.u, output unchanged (lists held fixed)
    u = np.random.default_rng(3).normal(size=TINY.d)
    Ou, Lu = o.attn_fwd(x["Q"], x["K"] + u, x["V"], *args)
    src = o.fill_source(part, ix.keep_idx)
    assert np.abs(Ou - O).max() < 1e-12
    assert np.abs(Lu - LSE - scale * (x["Q"] @ u)[src]).max() < 1e-12
    # token filling: pruned rows equal their center's row bit for bit
    tok = part.block_tokens()
    for i in range(part.N):
        for c in range(part.Bk):
            if c not in ix.keep_idx[i]:
                assert np.array_equal(O[tok[i, c]], O[tok[i, part.center]])
                assert LSE[tok[i, c]] == LSE[tok[i, part.center]]


def test_backward_finite_differences_and_invariants():
    part = tiny_part()
    x = tiny_inputs(1)
    x["Q"], x["K"] = x["Q"] * 3.0, x["K"] * 3.0
    scale = 1 / sqrt(TINY.d)
    ix = o.bsa_indices(x["Q"], x["K"], part, 0.6, 0.5)
    args = (part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale)
    dQ, dK, dV = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], *args)

    def loss(Q, K, V):
        return float((o.attn_fwd(Q, K, V, *args)[0] * x["dO"]).sum())

    rng = np.random.default_rng(4)
    eps = 1e-6
    for name, grad in (("Q", dQ), ("K", dK), ("V", dV)):
        for _ in range(6):
            dirn = rng.normal(size=grad.shape)
            plus = dict(x)
            minus = dict(x)
            plus[name] = x[name] + eps * dirn
            minus[name] = x[name] - eps * dirn
            fd = (loss(plus["Q"], plus["K"], plus["V"]) - loss(minus["Q"], minus["K"], minus["V"])) / (2 * eps)
            an = float((grad * dirn).sum())
            assert abs(fd - an) < 1e-6 * max(1.0, abs(an)), (name, fd, an)
    # rows of P sum to one and the fill gradient is folded in: sum dV == sum dO
    assert np.abs(dV.sum(axis=0) - x["dO"].sum(axis=0)).max() < 1e-10
    tok = part.block_tokens()
    for i in range(part.N):
        pruned = [c for c in range(part.Bk) if c not in ix.keep_idx[i]]
        assert not dQ[tok[i, pruned]].any()
    # a KV block that no query block lists receives exactly zero gradient
    ptr = np.arange(0, 3 * part.N + 1, 3, dtype=np.int32)
    idx = np.array([[0, 2, 6] if i % 2 else [1, 2, 7] for i in range(part.N)], dtype=np.int32).reshape(-1)
    _, dK2, dV2 = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], part, ptr, idx, ix.keep_idx, scale)
    for j in range(part.N):
        zero = not dK2[tok[j]].any() and not dV2[tok[j]].any()
        assert zero == (j in (3, 4, 5))


def test_per_kv_block_gradient_matches_full_backward():
    part = tiny_part()
    x = tiny_inputs()
    x["Q"], x["K"] = x["Q"] * 3.0, x["K"] * 3.0
    scale = 1 / sqrt(TINY.d)
    ix = o.bsa_indices(x["Q"], x["K"], part, 0.6, 0.5)
    _, dK, dV = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale)
    tok = part.block_tokens()
    for j in (0, 3, 7):
        dKj, dVj = o.attn_bwd_kv_block(x["Q"], x["K"], x["V"], x["dO"], part, ix.q2k_ptr, ix.q2k_idx,
                                       ix.k2q_ptr, ix.k2q_idx, ix.keep_idx, scale, j)
        assert np.abs(dKj - dK[tok[j]]).max() < 1e-12
        assert np.abs(dVj - dV[tok[j]]).max() < 1e-12


def test_float32_attention_path_tracks_float64():
    part = tiny_part()
    x = tiny_inputs()
    scale = 1 / sqrt(TINY.d)
    ix = o.bsa_indices(x["Q"], x["K"], part, 0.9, 0.5)
    args = (part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale)
    O64, _ = o.attn_fwd(x["Q"], x["K"], x["V"], *args)
    O32, _ = o.attn_fwd(x["Q"], x["K"], x["V"], *args, dtype=np.float32)
    assert O32.dtype == np.float32 and np.abs(O32 - O64).max() < 1e-5
    g64 = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], *args)
    g32 = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], *args, dtype=np.float32)
    for a, b in zip(g32, g64):
        assert np.abs(a - b).max() < 1e-4


# ---------------------------------------------------------- input generator
def test_generator_is_seeded_and_bf16_exact():
    wl = WORKLOADS["wan1p3b"].replace(grid=(4, 8, 8), H=2)
    a = head_inputs(wl, 0, 1)
    b = head_inputs(wl, 0, 1)
    c = head_inputs(wl, 0, 0)
    for k in a:
        assert np.array_equal(a[k], b[k]) and not np.array_equal(a[k], c[k])
        assert np.array_equal(a[k].view(np.uint32) & 0xFFFF, np.zeros_like(a[k], dtype=np.uint32))
    assert 1.2 < a["Q"].std() < 1.8  # four unit sinusoids (var 2) + noise 0.09
    assert 0.9 < a["dO"].std() < 1.1


def test_backward_with_stored_output_equals_exact_backward_when_storage_is_exact():
    part = tiny_part()
    x = tiny_inputs()
    scale = 1 / sqrt(TINY.d)
    ix = o.bsa_indices(x["Q"], x["K"], part, 0.6, 0.5)
    args = (part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale)
    O, _ = o.attn_fwd(x["Q"], x["K"], x["V"], *args)
    exact = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], *args)
    stored = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], *args, O_in=O)
    for a, b in zip(exact, stored):
        assert np.abs(a - b).max() < 1e-13
    # a perturbed stored O changes dQ and dK through delta only, never dV
    bumped = o.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], *args, O_in=O + 1e-3)
    assert np.array_equal(bumped[2], exact[2]) and np.abs(bumped[0] - exact[0]).max() > 1e-6


# ------------------------------------------- window-based critical tokens (Sec. 3.2.2)
def win_part():
    """The tiny grid with its 2x4x4 blocks cut into (1,2,2) windows: 8 windows of 4 tokens."""
    return o.Partition(*TINY.grid, *TINY.block, 1, 2, 2)


def _window_center_by_coordinates(part, n):
    """Raster index of the critical token of raster token n's window, from coordinates alone."""
    wt, wh, ww = part.window
    t, h, w = n // (part.Hs * part.Ws), (n // part.Ws) % part.Hs, n % part.Ws
    lt, lh, lw = t % part.Ct, h % part.Ch, w % part.Cw  # local coordinates inside the block
    ct = t - lt + (lt // wt) * wt + wt // 2
    ch = h - lh + (lh // wh) * wh + wh // 2
    cw = w - lw + (lw // ww) * ww + ww // 2
    return (ct * part.Hs + ch) * part.Ws + cw


def test_window_tables_of_the_papers_default():
    lines = open(__file__.replace("test_oracle_pins.py", "golden/paper_constants.txt")).read().split("\n")
    vals = dict(l.split("=")[0:2] for l in lines if "=" in l and not l.startswith("#"))
    block = tuple(int(v) for v in vals["block"].split(","))
    window = tuple(int(v) for v in vals["window"].split(","))
    part = o.Partition(*block, *block, *window)  # one block
    assert (part.nwin, part.Wk) == (8, 8)
    # Sec. 4.1: r = 0.5 still gives a query block of 32 with (2,2,2) windows (4 of 8 per window)
    assert part.n_keep(float(vals["keep_ratio"])) == int(vals["query_block_size"].split()[0])
    win, cen = part.window_of(), part.centers()
    assert win[0] == 0 and win[63] == 7 and win[2] == 1 and win[8] == 2 and win[32] == 4
    assert cen.tolist() == [21, 23, 29, 31, 53, 55, 61, 63]  # local (1,1,1) of each 2x2x2 window
    assert sorted(np.bincount(win).tolist()) == [8] * 8
    tok = part.block_tokens()
    for c in range(64):
        assert tok[0, part.center_of()[c]] == _window_center_by_coordinates(part, tok[0, c])
    with pytest.raises(ValueError):
        o.Partition(4, 4, 4, 4, 4, 4, 3, 2, 2)  # must divide the block evenly


def test_window_equal_to_the_block_is_the_single_center_method():
    x = tiny_inputs()
    a, _ = o.prune_q(x["Q"], tiny_part(), 0.5)
    b, _ = o.prune_q(x["Q"], o.Partition(*TINY.grid, *TINY.block, *TINY.block), 0.5)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("r", [0.25, 0.5, 0.75, 1.0])
def test_window_prune_invariants(r):
    part = win_part()
    x = tiny_inputs()
    keep, _ = o.prune_q(x["Q"], part, r)
    kw = ceil(r * part.Wk - 1e-12)
    assert keep.shape == (part.N, part.nwin * kw)
    tok = part.block_tokens()
    win, cen = part.window_of(), part.centers()
    for i in range(part.N):
        ks = keep[i].tolist()
        assert ks == sorted(set(ks))
        for w in range(part.nwin):
            members = [c for c in range(part.Bk) if win[c] == w]
            kept = [c for c in members if c in ks]
            assert len(kept) == kw and cen[w] in kept  # every window fills its own quota, center included
            qc = x["Q"][tok[i, cen[w]]]
            cos = {c: float(x["Q"][tok[i, c]] @ qc / (np.linalg.norm(x["Q"][tok[i, c]]) * np.linalg.norm(qc))) for c in members}
            pruned = [c for c in members if c not in ks]
            kept_others = [c for c in kept if c != cen[w]]
            if pruned and kept_others:
                assert max(cos[c] for c in kept_others) <= min(cos[c] for c in pruned) + 1e-12


@pytest.mark.parametrize("p,r", [(0.9, 0.5), (0.5, 0.25)])
def test_window_fwd_bwd_against_autograd_of_masked_dense_form(p, r):
    """As the single-center test, with the fill map built from window coordinates here."""
    part = win_part()
    x = tiny_inputs(1)
    x["Q"], x["K"] = x["Q"] * 3.0, x["K"] * 3.0
    scale = 1 / sqrt(TINY.d)
    ix, O, LSE, dQ, dK, dV = o.bsa_head(x["Q"], x["K"], x["V"], x["dO"], part, p, r)
    tok = part.block_tokens()
    src = np.empty(part.L, dtype=np.int64)
    for i in range(part.N):
        kept = set(tok[i, ix.keep_idx[i]].tolist())
        for n in tok[i]:
            src[n] = n if n in kept else _window_center_by_coordinates(part, n)
    assert np.array_equal(src, o.fill_source(part, ix.keep_idx))
    M = o.dense_mask(part, ix.q2k_ptr, ix.q2k_idx)
    tO, tL, tdQ, tdK, tdV = _torch_dense(x["Q"], x["K"], x["V"], x["dO"], scale, M, src)
    for a, b in ((O, tO), (LSE, tL), (dQ, tdQ), (dK, tdK), (dV, tdV)):
        assert np.abs(a - b).max() < 1e-11 * max(1.0, np.abs(b).max())
    # every center keeps its own gradient plus its window's fill copies: column sums are conserved
    assert np.abs(dV.sum(axis=0) - x["dO"].sum(axis=0)).max() < 1e-10
    pruned_any = False
    for i in range(part.N):
        for c in range(part.Bk):
            if c not in ix.keep_idx[i]:
                pruned_any = True
                assert np.array_equal(O[tok[i, c]], O[_window_center_by_coordinates(part, tok[i, c])])
                assert not dQ[tok[i, c]].any()
    assert pruned_any


# ----------------------------- Eq. 3: statistical dynamic threshold (reading; arithmetic pinned)
def test_stat_quantile_selects_about_k_of_n_normal_scores():
    """The paper's stated purpose of Eq. 3: the threshold is such that k key samples pass."""
    from statistics import NormalDist

    n = 2000
    s = np.array([NormalDist(mu=1.5, sigma=0.7).inv_cdf((j + 0.5) / n) for j in range(n)])  # an exactly normal sample
    for k in (20, 200, 1000, 1800):
        tau = o.stat_threshold(s, o.stat_quantile(k, n))
        assert abs(int((s >= tau).sum()) - k) <= 2
    # tabulated standard-normal quantiles: U(0.9), U(0.975), U(0.5), U(0.1)
    assert o.stat_quantile(1, 10) == pytest.approx(1.2815515655446004, abs=1e-12)
    assert o.stat_quantile(1, 40) == pytest.approx(1.959963984540054, abs=1e-12)
    assert o.stat_quantile(9, 10) == pytest.approx(-1.2815515655446004, abs=1e-12)
    assert o.stat_quantile(n, n) == float("-inf")
    assert abs(o.stat_quantile(n // 2, n)) < 1e-12  # the median: z = 0
    with pytest.raises(ValueError):
        o.stat_quantile(0, 10)


def test_stat_threshold_hand_example_and_invariances():
    s = np.array([0.0, 1.0, 2.0, 3.0, 4.0])
    assert o.stat_threshold(s, 0.0) == 2.0
    assert abs(o.stat_threshold(s, 1.0) - (2.0 + sqrt(2.5))) < 1e-15  # n-1 divisor: var = 10/4
    sel = o.select_row(s, 1.0, 0.0)  # mass threshold off: exactly the candidates {2,3,4}
    assert sel.idx.tolist() == [2, 3, 4]
    assert o.select_row(s, 1.0, 5.0).idx.tolist() == [4]  # no candidate: the best block alone
    # z = -inf (k = n) and z = None are plain Eq. 4
    rng = np.random.default_rng(11)
    r = rng.normal(size=40) * 2
    for p in (0.5, 0.9):
        a, b, c = o.select_row(r, p), o.select_row(r, p, float("-inf")), o.select_row(r, p, -50.0)
        assert a.idx.tolist() == b.idx.tolist() == c.idx.tolist()
    # the candidate set is invariant under s -> a s + b (a > 0)
    z = 0.3
    base = set(o.select_row(r, 1.0, z).idx.tolist())
    assert base == set(o.select_row(3.0 * r - 7.0, 1.0, z).idx.tolist())
    # the result is the intersection of Eq. 4's prefix with the candidates, never empty
    for p in (0.3, 0.7, 0.95):
        for z in (-1.0, 0.0, 1.0, 2.5):
            full = o.select_row(r, p).idx.tolist()
            cand = [j for j in range(40) if r[j] >= o.stat_threshold(r, z)]
            got = o.select_row(r, p, z).idx.tolist()
            want = sorted(set(full) & set(cand)) or [int(np.argmax(r))]
            assert got == want


# ------------------------------------------------ block-major token order (Sec. 3.2.1 reorder)
def test_block_major_order_is_the_partitions_block_table():
    from bsa_workloads import block_major_order

    part = o.Partition(4, 6, 8, 2, 3, 4)
    assert np.array_equal(block_major_order((4, 6, 8), (2, 3, 4)), part.block_tokens().reshape(-1))
    bm = o.Partition(4, 6, 8, 2, 3, 4, 0, 0, 0, True)
    assert np.array_equal(bm.block_tokens().reshape(-1), np.arange(bm.L))
    assert bm.center == part.center and np.array_equal(bm.window_of(), part.window_of())


def test_block_major_layout_gives_the_same_video_the_same_results():
    """Reordering the tokens once (blocks adjacent) and telling the partition so must permute
    every output and change nothing else: the method is defined on the video, not on the order."""
    part = win_part()
    bm = o.Partition(*TINY.grid, *TINY.block, 1, 2, 2, True)
    order = part.block_tokens().reshape(-1)
    x = tiny_inputs(1)
    x["Q"], x["K"] = x["Q"] * 3.0, x["K"] * 3.0
    xb = {k: v[order] for k, v in x.items()}
    a = o.bsa_head(x["Q"], x["K"], x["V"], x["dO"], part, 0.6, 0.5)
    b = o.bsa_head(xb["Q"], xb["K"], xb["V"], xb["dO"], bm, 0.6, 0.5)
    assert np.array_equal(a[0].q2k_idx, b[0].q2k_idx) and np.array_equal(a[0].keep_idx, b[0].keep_idx)
    for ta, tb in zip(a[1:], b[1:]):
        assert np.array_equal(ta[order], tb)
