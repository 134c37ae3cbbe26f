"""GPU parity of bsa_select_kv alone on hand-made pooled inputs: exactly equal scores (the
tie rule of the minimal prefix: ascending block id), duplicated KV blocks, and block counts
that exercise every workgroup shape of the selection kernel (one wavefront up to 1024
blocks, four wavefronts beyond, up to the 8192-block limit).  CSR and transposed CSR are
compared bit for bit with the CPU oracle's Eq. 4."""
from math import sqrt

import numpy as np
import pytest
import torch

from oracle import bsa_oracle as o
from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu


def run(shp: B.Shape, Qbar: np.ndarray, Kbar: np.ndarray, p: float):
    """Qbar, Kbar: [H][N][d] float64 (B = 1).  Returns the host CSR of the GPU path."""
    q = torch.from_numpy(np.ascontiguousarray(Qbar)).cuda().reshape(1, shp.H, shp.N, shp.d)
    k = torch.from_numpy(np.ascontiguousarray(Kbar)).cuda().reshape(1, shp.H, shp.N, shp.d)
    lists = B.select_kv(shp, q, k, p)
    return U.lists_to_host(shp, lists)


def check(shp, host, Qbar, Kbar, p, allow_marginal=False):
    scale = 1.0 / sqrt(shp.d)
    for h in range(shp.H):
        scores = o.block_scores(Qbar[h], Kbar[h], scale)
        ptr, idx, margin = o.select_kv(scores, p)
        tptr, tidx = o.transpose_csr(ptr, idx, shp.N)
        gptr, gidx = U.head_csr(host, shp, 0, h, "q2k")
        if allow_marginal and not (np.array_equal(gptr, ptr) and np.array_equal(gidx, idx)):
            # a differing row must be one whose deciding comparison is within rounding of a tie
            for i in range(shp.N):
                mine, ref = gidx[gptr[i]:gptr[i + 1]], idx[ptr[i]:ptr[i + 1]]
                if not np.array_equal(mine, ref):
                    assert o.select_row(scores[i], p).margin < U.SELECT_MARGIN, (h, i)
            continue
        assert np.array_equal(gptr, ptr) and np.array_equal(gidx, idx), f"head {h}"
        kptr, kidx = U.head_csr(host, shp, 0, h, "k2q")
        assert np.array_equal(kptr, tptr) and np.array_equal(kidx, tidx), f"head {h} transposed"


def select_shape(N: int, H: int, d: int) -> B.Shape:
    """A shape with N blocks of one token each (selection only looks at N and d)."""
    assert N % 8 == 0
    return B.Shape(1, H, 8, N // 8, 1, 1, 1, 1, d, B.F32)


@pytest.mark.parametrize("p", [0.3, 0.5, 0.999, 1.0])
def test_all_scores_equal(p):
    """Constant pooled vectors: every score ties, the prefix is the first ceil-ish(p N) block ids."""
    U.progress(f"select all-equal p={p}")
    N, H, d = 40, 2, 64
    shp = select_shape(N, H, d)
    Qbar = np.full((H, N, d), 0.25)
    Kbar = np.full((H, N, d), -0.5)
    host = run(shp, Qbar, Kbar, p)
    check(shp, host, Qbar, Kbar, p)
    ptr, idx = U.head_csr(host, shp, 0, 0, "q2k")
    k = ptr[1] - ptr[0]
    assert np.array_equal(idx[:k], np.arange(k))  # ascending ids from 0


@pytest.mark.parametrize("N,dup", [(40, 2), (96, 4), (1032, 8)])
def test_duplicated_kv_blocks(N, dup):
    """Every KV vector appears `dup` times: ties inside the prefix and, for most rows, at its end."""
    U.progress(f"select duplicated N={N} dup={dup}")
    H, d = 2, 64
    rng = np.random.default_rng(N)
    shp = select_shape(N, H, d)
    base = rng.standard_normal((H, N // dup, d))
    Kbar = np.repeat(base, dup, axis=1)[:, rng.permutation(N)]
    Qbar = rng.standard_normal((H, N, d))
    for p in (0.5, 0.9):
        host = run(shp, Qbar, Kbar, p)
        check(shp, host, Qbar, Kbar, p)


@pytest.mark.parametrize("N,H", [(8, 1), (520, 2), (1024, 1), (1032, 1), (4096, 1), (4104, 1), (8192, 1)])
def test_block_counts(N, H):
    U.progress(f"select N={N}")
    d = 32
    rng = np.random.default_rng(N + 1)
    shp = select_shape(N, H, d)
    Qbar = rng.standard_normal((H, N, d)) * 1.5
    Kbar = rng.standard_normal((H, N, d)) * 1.5
    host = run(shp, Qbar, Kbar, 0.9)
    check(shp, host, Qbar, Kbar, 0.9, allow_marginal=True)


def test_signed_zero_and_negative_scores():
    """Scores of both signs and exact zeros (+0 and -0 must tie)."""
    U.progress("select signed zeros")
    N, H, d = 64, 1, 8
    shp = select_shape(N, H, d)
    rng = np.random.default_rng(5)
    Qbar = rng.standard_normal((H, N, d))
    Kbar = rng.standard_normal((H, N, d))
    Kbar[0, 10:20] = 0.0      # scores exactly +0 or -0 depending on the signs of Q
    Kbar[0, 30:34] *= -0.0
    host = run(shp, Qbar, Kbar, 0.95)
    check(shp, host, Qbar, Kbar, 0.95)


@pytest.mark.parametrize("N,k,p", [(520, 52, 0.9), (520, 260, 0.5), (520, 5, 1.0), (1032, 100, 0.95), (40, 40, 0.8), (64, 1, 0.9)])
def test_statistical_threshold_filter(N, k, p):
    """Eq. 3 ahead of Eq. 4: candidates are the blocks whose logit reaches mean + std * z."""
    U.progress(f"select stat N={N} k={k} p={p}")
    H, d = 2, 32
    rng = np.random.default_rng(7 * N + k)
    shp = select_shape(N, H, d)
    Qbar = rng.standard_normal((H, N, d)) * 1.5
    Kbar = rng.standard_normal((H, N, d)) * 1.5
    z = o.stat_quantile(k, N)  # an input of the call: the caller supplies Eq. 3's quantile
    q = torch.from_numpy(Qbar).cuda().reshape(1, H, N, d)
    kk = torch.from_numpy(Kbar).cuda().reshape(1, H, N, d)
    host = U.lists_to_host(shp, B.select_kv(shp, q, kk, p, stat_z=z))
    scale = 1.0 / sqrt(d)
    shorter = 0
    for h in range(H):
        scores = o.block_scores(Qbar[h], Kbar[h], scale)
        ptr, idx, margin = o.select_kv(scores, p, z)
        plain, _, _ = o.select_kv(scores, p)
        shorter += int(ptr[-1] < plain[-1])
        gptr, gidx = U.head_csr(host, shp, 0, h, "q2k")
        if not (np.array_equal(gptr, ptr) and np.array_equal(gidx, idx)):
            for i in range(N):  # a differing row must sit within rounding of a deciding comparison
                if not np.array_equal(gidx[gptr[i]:gptr[i + 1]], idx[ptr[i]:ptr[i + 1]]):
                    assert o.select_row(scores[i], p, z).margin < U.SELECT_MARGIN, (h, i)
            continue
        tptr, tidx = o.transpose_csr(ptr, idx, N)
        kptr, kidx = U.head_csr(host, shp, 0, h, "k2q")
        assert np.array_equal(kptr, tptr) and np.array_equal(kidx, tidx)
    if k < N // 2 and p >= 0.9:
        assert shorter == H  # the filter is active in these cases, not vacuous


def test_statistical_threshold_with_no_candidate_keeps_the_best_block():
    U.progress("select stat no candidate")
    N, H, d = 64, 1, 8
    shp = select_shape(N, H, d)
    rng = np.random.default_rng(3)
    Qbar, Kbar = rng.standard_normal((H, N, d)), rng.standard_normal((H, N, d))
    Kbar[0, 5] = Kbar[0, 9]  # an exact tie that may be a row's maximum: lowest id wins
    q = torch.from_numpy(Qbar).cuda().reshape(1, H, N, d)
    k = torch.from_numpy(Kbar).cuda().reshape(1, H, N, d)
    host = U.lists_to_host(shp, B.select_kv(shp, q, k, 0.9, stat_z=float("inf")))
    ptr, idx = U.head_csr(host, shp, 0, 0, "q2k")
    scores = o.block_scores(Qbar[0], Kbar[0], 1.0 / sqrt(d))
    assert np.array_equal(np.diff(ptr), np.ones(N, dtype=np.int32))
    assert np.array_equal(idx, scores.argmax(axis=1))  # argmax returns the first maximum
