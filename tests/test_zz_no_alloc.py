"""bsa_select_kv_static (the selection with the library's built-in scratch, for callers that
cannot allocate) against bsa_select_kv on the same inputs: lists, transposed lists and nnz must
be identical, on two calls in a row, the second with a smaller input (the buffer keeps the first
call's contents).  No device memory may be allocated by the call itself."""
import numpy as np
import pytest
import torch

from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu


def _pooled(H, N, d, seed):
    rng = np.random.default_rng(seed)
    mk = lambda: torch.from_numpy(rng.standard_normal((1, H, N, d)) * 1.5).cuda()
    return mk(), mk()


def _shape(H, grid):
    return B.Shape(1, H, *grid, 4, 4, 4, 32, B.BF16)


def _same(a: B.KvLists, b: B.KvLists, rows: int):
    torch.cuda.synchronize()
    nnz = int(a.nnz.item())
    assert nnz == int(b.nnz.item()) and nnz == int(a.q2k_ptr[rows].item())
    assert torch.equal(a.q2k_ptr, b.q2k_ptr) and torch.equal(a.k2q_ptr, b.k2q_ptr)
    assert torch.equal(a.q2k_idx[:nnz], b.q2k_idx[:nnz]) and torch.equal(a.k2q_idx[:nnz], b.k2q_idx[:nnz])
    return nnz


def test_static_scratch_selection_matches_the_workspace_one_twice_in_a_row():
    # first the largest layer that fits the built-in buffer (33,280 tokens, 12 heads: 26.4 MB of scratch),
    # then a much smaller one whose scratch lies inside what the first call left behind
    for H, grid, thr, seed in ((12, (20, 32, 52), 0.9, 1), (3, (8, 12, 20), 0.7, 2)):
        shp = _shape(H, grid)
        U.progress(f"static select H={H} N={shp.N}")
        assert B.select_workspace_bytes(shp) <= B.STATIC_SELECT_BYTES
        Qbar, Kbar = _pooled(H, shp.N, 32, seed)
        ref = B.select_kv(shp, Qbar, Kbar, thr)
        out = B.alloc_kv_lists(shp, Qbar.device, workspace=False)
        for t in (out.q2k_ptr, out.q2k_idx, out.k2q_ptr, out.k2q_idx):
            t.fill_(-7)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        B.select_kv_static(shp, Qbar, Kbar, thr, out)
        assert torch.cuda.memory_allocated() == before
        nnz = _same(out, ref, shp.rows)
        assert 0 < nnz < shp.rows * shp.N
    # a shape beyond the buffer is refused, and nothing was launched: the outputs are untouched
    big = _shape(40, (20, 44, 80))
    q = torch.zeros(1, device="cuda", dtype=torch.float64)
    with pytest.raises(B.BsaError) as e:
        B.select_kv_static(big, q, q, 0.9, B.KvLists(out.q2k_ptr, torch.empty(big.rows * big.N, dtype=torch.int32, device="cuda"),
                                                     out.k2q_ptr, out.k2q_idx, out.nnz, out.workspace))
    assert e.value.status == -8
