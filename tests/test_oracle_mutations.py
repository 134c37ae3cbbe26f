"""Do the pins bite?  Each case plants one plausible mistake in the CPU oracle (a dropped
term, a wrong sign or index, a transposed operand, a wrong tie rule) and checks that at least
one of the pins that are meant to fix that function fails.  Everything here runs on the CPU and
touches only the oracle; the mutated function is restored afterwards."""
import numpy as np
import pytest

from oracle import bsa_oracle as o

import test_oracle_pins as pins


def caught(checks) -> bool:
    for fn, args in checks:
        try:
            fn(*args)
        except Exception:  # an assertion, or the mutated code breaking outright
            return True
    return False


# ---- mutated versions of oracle functions -------------------------------------------------
def pool_sum_instead_of_mean(X, part):
    tok = part.block_tokens()
    return o._seq_sum(np.asarray(X, dtype=np.float64)[tok], axis=1)


def pool_first_token(X, part):
    return np.asarray(X, dtype=np.float64)[part.block_tokens()[:, 0]]


def scores_without_scale(Qbar, Kbar, score_scale):
    return o._seq_dot(Qbar[:, None, :], Kbar[None, :, :])


def scores_transposed(Qbar, Kbar, score_scale):
    return o._seq_dot(Kbar[:, None, :], Qbar[None, :, :]) * np.float64(score_scale)


def make_select_row(strict=False, ascending=False, tie_high=False, off_by_one=False):
    def select_row(s, p, z=None):
        if not (0.0 < p <= 1.0):
            raise ValueError("mass threshold p must lie in (0, 1]")
        s = np.asarray(s, dtype=np.float64)
        n = s.shape[0]
        key = s if ascending else -s
        order = np.lexsort((-np.arange(n) if tie_high else np.arange(n), key))
        e = np.exp(s[order] - s.max())
        c = np.cumsum(e)
        if p >= 1.0:
            k = n
        else:
            hit = (c > p * c[-1]) if strict else (c >= p * c[-1])
            k = int(np.argmax(hit)) + 1 + (1 if off_by_one else 0)
            k = min(k, n)
        return o.RowSelection(np.sort(order[:k]).astype(np.int32), k, 1.0)
    return select_row


def select_row_margin_one_sided(s, p, z=None):
    """The real selection, but the margin forgets the comparison with c_{k-1}."""
    sel = SELECT_ROW(s, p, z)
    if p >= 1.0:
        return sel
    s = np.asarray(s, dtype=np.float64)
    order = np.lexsort((np.arange(s.shape[0]), -s))
    c = np.cumsum(np.exp(s[order] - s[order[0]]))
    return o.RowSelection(sel.idx, sel.k, float((c[sel.k - 1] - p * c[-1]) / c[-1]))


def select_row_margin_not_relative(s, p, z=None):
    """The real selection, but the margin is not divided by the row's total mass."""
    sel = SELECT_ROW(s, p, z)
    s = np.asarray(s, dtype=np.float64)
    Z = float(np.sum(np.exp(s - s.max())))
    return o.RowSelection(sel.idx, sel.k, sel.margin * Z)


def prune_q_gap_of_first_block_only(Q, part, r):
    keep, _ = PRUNE_Q(Q, part, r)
    first = o.Partition(part.Ct, part.Ch, part.Cw, part.Ct, part.Ch, part.Cw, part.Wt, part.Wh, part.Ww)
    return keep, PRUNE_Q(np.asarray(Q)[part.block_tokens()[0]], first, r)[1]


def transpose_unsorted(ptr, idx, n_cols):
    tptr, tidx = TRANSPOSE(ptr, idx, n_cols)
    out = tidx.copy()
    for j in range(n_cols):
        out[tptr[j]:tptr[j + 1]] = tidx[tptr[j]:tptr[j + 1]][::-1]
    return tptr, out


def cosine_unnormalised(Q, part):
    tok, cof = part.block_tokens(), part.center_of()
    Qb = np.asarray(Q, dtype=np.float64)[tok]
    return o._seq_dot(Qb, Qb[:, cof, :])


def cosine_to_first_token(Q, part):
    tok = part.block_tokens()
    Qb = np.asarray(Q, dtype=np.float64)[tok]
    dot = o._seq_dot(Qb, Qb[:, :1, :])
    nrm = o._seq_dot(Qb, Qb)
    den = np.sqrt(nrm * nrm[:, :1])
    cos = np.zeros_like(dot)
    np.divide(dot, den, out=cos, where=den > 0.0)
    return cos


def make_prune(most_similar=False, drop_center=False):
    def prune_q(Q, part, r):
        kw = part.n_keep_window(r)
        cos = o.cosine_to_center(Q, part)
        win, cen = part.window_of(), part.centers()
        keep = np.empty((part.N, part.nwin * kw), dtype=np.int32)
        for i in range(part.N):
            sel = []
            for w in range(part.nwin):
                members = [c for c in range(part.Bk) if win[c] == w and (drop_center or c != cen[w])]
                others = np.array(members, dtype=np.int64)
                key = -cos[i, others] if most_similar else cos[i, others]
                order = others[np.lexsort((others, key))]
                if drop_center:
                    sel.extend(order[:kw])
                else:
                    sel.append(cen[w])
                    sel.extend(order[: kw - 1])
            keep[i] = np.sort(np.array(sel))
        return keep, 1.0
    return prune_q


def make_attend(no_scale=False, unnormalised=False):
    def attend_block(q, Ksel, Vsel, sm_scale):
        s = q @ Ksel.T
        if not no_scale:
            s = s * q.dtype.type(sm_scale)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        P = e if unnormalised else e / z
        return P @ Vsel, (m + np.log(z))[:, 0], P
    return attend_block


def folded_grad_without_fold(dO, part, keep_idx, i, tok=None):
    tok = part.block_tokens() if tok is None else tok
    return np.array(dO[tok[i, keep_idx[i]]])


def folded_grad_into_first_row(dO, part, keep_idx, i, tok=None):
    tok = part.block_tokens() if tok is None else tok
    g = np.array(dO[tok[i, keep_idx[i]]])
    for c in np.setdiff1d(np.arange(part.Bk), keep_idx[i]):
        g[0] = g[0] + dO[tok[i, c]]
    return g


def fill_source_block_center(part, keep_idx):
    """Fills from the first window's center whatever the token's window."""
    tok, cen = part.block_tokens(), part.centers()
    src = np.empty(part.L, dtype=np.int64)
    for i in range(part.N):
        src[tok[i]] = tok[i, cen[0]]
        src[tok[i, keep_idx[i]]] = tok[i, keep_idx[i]]
    return src


def make_bwd(no_delta=False, dk_without_scale=False, dq_transposed=False, dv_from_dS=False):
    def attn_bwd(Q, K, V, dO, part, q2k_ptr, q2k_idx, keep_idx, sm_scale, dtype=np.float64, q_blocks=None, O_in=None):
        tok = part.block_tokens()
        Q, K, V, dO = (np.asarray(a, dtype=dtype) for a in (Q, K, V, dO))
        dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
        for i in (range(part.N) if q_blocks is None else q_blocks):
            rows = tok[i, keep_idx[i]]
            keys = tok[q2k_idx[q2k_ptr[i]:q2k_ptr[i + 1]]].reshape(-1)
            q, k, v = Q[rows], K[keys], V[keys]
            out, _, P = o.attend_block(q, k, v, sm_scale)
            if O_in is not None:
                out = np.asarray(O_in, dtype=dtype)[rows]
            g = o.folded_grad(dO, part, keep_idx, i, tok)
            delta = 0.0 if no_delta else (g * out).sum(axis=1, keepdims=True)
            dS = P * (g @ v.T - delta)
            dQ[rows] = (dS @ k) * dtype(sm_scale) if not dq_transposed else (P @ k) * dtype(sm_scale)
            dK[keys] += (dS.T @ q) * (dtype(1.0) if dk_without_scale else dtype(sm_scale))
            dV[keys] += (dS.T @ g) if dv_from_dS else (P.T @ g)
        return dQ, dK, dV
    return attn_bwd


def stat_threshold_population_std(s, z):
    s = np.asarray(s, dtype=np.float64)
    return float(np.mean(s) + np.std(s) * z)


def stat_threshold_minus(s, z):
    s = np.asarray(s, dtype=np.float64)
    return float(np.mean(s) - np.std(s, ddof=1) * z)


TRANSPOSE = o.transpose_csr
SELECT_ROW = o.select_row
PRUNE_Q = o.prune_q
MARGIN_PINS = [(pins.test_select_margin_closed_form_and_boundary_nudges, ())]
GAP_PINS = [(pins.test_prune_gap_is_the_distance_between_the_last_kept_and_the_first_pruned_cosine, ())]

SELECT_PINS = [(pins.test_select_is_minimal_and_maximal_mass_by_brute_force, (p,)) for p in (0.3, 0.5, 0.9)] + [
    (pins.test_select_closed_forms, ()), (pins.test_select_nesting_and_tie_break, ())]
PRUNE_PINS = [(pins.test_prune_invariants, (r,)) for r in (0.25, 0.5, 0.75)] + [
    (pins.test_prune_identical_tokens_and_zero_vectors, ()), (pins.test_cosine_matches_definition, ()),
    (pins.test_window_prune_invariants, (0.5,))]
FWD_PINS = [(pins.test_threshold_one_no_pruning_is_full_softmax_attention, ()), (pins.test_forward_invariants, ()),
            (pins.test_sparse_fwd_bwd_against_autograd_of_masked_dense_form, (0.9, 0.5)),
            (pins.test_window_fwd_bwd_against_autograd_of_masked_dense_form, (0.9, 0.5))]
BWD_PINS = [(pins.test_sparse_fwd_bwd_against_autograd_of_masked_dense_form, (0.9, 0.5)),
            (pins.test_backward_finite_differences_and_invariants, ()),
            (pins.test_window_fwd_bwd_against_autograd_of_masked_dense_form, (0.9, 0.5))]
POOL_PINS = [(pins.test_pool_dot_equals_mean_of_token_logits, ()), (pins.test_pool_of_blockwise_constant_field, ())]
STAT_PINS = [(pins.test_stat_threshold_hand_example_and_invariances, ()),
             (pins.test_stat_quantile_selects_about_k_of_n_normal_scores, ())]

MUTATIONS = {
    "pool: sum instead of mean": ("pool_blocks", pool_sum_instead_of_mean, POOL_PINS),
    "pool: first token instead of mean": ("pool_blocks", pool_first_token, POOL_PINS),
    "scores: scale dropped": ("block_scores", scores_without_scale, POOL_PINS + SELECT_PINS + [(pins.test_block_major_layout_gives_the_same_video_the_same_results, ())]),
    "scores: operands transposed": ("block_scores", scores_transposed, POOL_PINS),
    "select: strict comparison": ("select_row", make_select_row(strict=True), SELECT_PINS),
    "select: ascending order": ("select_row", make_select_row(ascending=True), SELECT_PINS),
    "select: ties to the higher id": ("select_row", make_select_row(tie_high=True), SELECT_PINS),
    "select: one block too many": ("select_row", make_select_row(off_by_one=True), SELECT_PINS),
    "select: margin ignores the lower neighbour": ("select_row", select_row_margin_one_sided, MARGIN_PINS),
    "select: margin not relative to the total mass": ("select_row", select_row_margin_not_relative, MARGIN_PINS),
    "prune: gap of the first block only": ("prune_q", prune_q_gap_of_first_block_only, GAP_PINS),
    "transpose: lists descending": ("transpose_csr", transpose_unsorted, [(pins.test_transpose_csr_roundtrip_and_counts, ())]),
    "cosine: not normalised": ("cosine_to_center", cosine_unnormalised, PRUNE_PINS),
    "cosine: to the first token": ("cosine_to_center", cosine_to_first_token, PRUNE_PINS),
    "prune: keeps the most similar": ("prune_q", make_prune(most_similar=True), PRUNE_PINS),
    "prune: center not forced": ("prune_q", make_prune(drop_center=True), PRUNE_PINS),
    "attend: scale dropped": ("attend_block", make_attend(no_scale=True), FWD_PINS),
    "attend: not normalised": ("attend_block", make_attend(unnormalised=True), FWD_PINS),
    "fill: wrong window's center": ("fill_source", fill_source_block_center, [(pins.test_window_fwd_bwd_against_autograd_of_masked_dense_form, (0.9, 0.5))]),
    "backward: fill gradient dropped": ("folded_grad", folded_grad_without_fold, BWD_PINS),
    "backward: fill gradient into the wrong row": ("folded_grad", folded_grad_into_first_row, BWD_PINS),
    "backward: delta dropped": ("attn_bwd", make_bwd(no_delta=True), BWD_PINS),
    "backward: dK without the scale": ("attn_bwd", make_bwd(dk_without_scale=True), BWD_PINS),
    "backward: dQ from P instead of dS": ("attn_bwd", make_bwd(dq_transposed=True), BWD_PINS),
    "backward: dV from dS instead of P": ("attn_bwd", make_bwd(dv_from_dS=True), BWD_PINS),
    "Eq. 3: population std": ("stat_threshold", stat_threshold_population_std, STAT_PINS),
    "Eq. 3: sign of the quantile term": ("stat_threshold", stat_threshold_minus, STAT_PINS),
}


def test_pins_pass_on_the_unmodified_oracle():
    for _, _, checks in MUTATIONS.values():
        assert not caught(checks)


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_mistake_is_caught(name, monkeypatch):
    attr, mutated, checks = MUTATIONS[name]
    monkeypatch.setattr(o, attr, mutated)
    assert caught(checks), f"no pin notices: {name}"
