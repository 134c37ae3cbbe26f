"""The library allocates nothing, never synchronises and launches on the stream it is given, so
one whole layer (pooling, selection, pruning, forward, backward) can be recorded into a HIP
graph.  A replay must reproduce the eager launches bit for bit: the kernels are deterministic
(fixed summation orders, no atomics on floating point).  The graph is replayed several times
with eager work and synchronisations of the program in between, and every replay is checked."""
import pytest
import torch

from bsa_workloads import Workload
from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu

CASES = {
    # MFMA path with split units and critical-token windows; the fp32 ALU path on ragged blocks
    "win_split": Workload("win_split", 1, 2, 128, "bf16", (16, 16, 24), (4, 4, 4), threshold=0.7, window=(2, 2, 2), seed=3),
    "ragged_f32": Workload("ragged_f32", 2, 2, 72, "fp32", (6, 6, 10), (3, 2, 5), threshold=0.7, keep_ratio=0.4),
}


@pytest.mark.parametrize("name", list(CASES))
def test_a_captured_layer_replays_the_eager_result(name):
    wl = CASES[name]
    U.progress(f"graph capture {name}")
    shp = U.shape_of(wl)
    dev = torch.device("cuda:0")
    x = U.device_inputs(wl)
    Q, K, V, dO = x["Q"], x["K"], x["V"], x["dO"]
    nk = B.n_keep(shp, wl.keep_ratio)
    Qbar = torch.empty((wl.B, wl.H, shp.N, wl.d), dtype=torch.float64, device=dev)
    Kbar = torch.empty_like(Qbar)
    lists = B.alloc_kv_lists(shp, dev)
    keep = torch.empty((wl.B, wl.H, shp.N, nk), dtype=torch.int32, device=dev)
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    LSE = torch.empty((wl.B, wl.H, wl.L), dtype=torch.float32, device=dev)
    ws = torch.empty(max(1, B.bwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
    fws = torch.empty(max(1, B.fwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
    outs = (O, LSE, dQ, dK, dV, keep, lists.q2k_ptr, lists.k2q_ptr)

    def layer():
        B.pool_blocks(shp, Q, Qbar)
        B.pool_blocks(shp, K, Kbar)
        B.select_kv(shp, Qbar, Kbar, wl.threshold, out=lists)
        B.prune_q(shp, Q, wl.keep_ratio, keep)
        B.attn_fwd(shp, Q, K, V, lists, keep, O=O, LSE=LSE, workspace=fws)
        B.attn_bwd(shp, Q, K, V, O, LSE, dO, lists, keep, dQ=dQ, dK=dK, dV=dV, workspace=ws)

    layer()  # eager: also the first call of every kernel, so that the capture records launches only
    torch.cuda.synchronize()
    nnz = int(lists.nnz.item())
    ref = [t.clone() for t in outs]
    idx_ref = lists.q2k_idx[:nnz].clone()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer()
    torch.cuda.synchronize()

    for replay in range(3):
        for t in outs:
            t.zero_()
        lists.q2k_idx.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert int(lists.nnz.item()) == nnz, f"replay {replay}"
        assert torch.equal(lists.q2k_idx[:nnz], idx_ref), f"replay {replay}: q2k_idx"
        for got, want, label in zip(outs, ref, ("O", "LSE", "dQ", "dK", "dV", "keep", "q2k_ptr", "k2q_ptr")):
            # bit patterns, so that -inf LSE rows and NaN-free equality are both covered
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), f"replay {replay}: {label}"
        layer()  # the program's own eager work between replays
        torch.cuda.synchronize()
