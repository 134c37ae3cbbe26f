"""GPU parity, small shapes: every stage of the HIP path (through the C ABI) against the CPU
oracle, element by element, on seeded inputs.  Index work (pooled sums are compared as
doubles, keep lists, CSR, transposed CSR) must be bit-exact; O / LSE / dQ / dK / dV are held to
the criteria of tests/tolerance.py (fp32: max-abs 1e-4 of the oracle tensor's RMS; bf16: 2e-2
for O plainly, 5e-3 in RMS for every tensor, and the gradients element by element after the
bf16 rounding of their own value and of the MFMA operands)."""
import functools
from math import sqrt

import numpy as np
import pytest
import torch

from bsa_workloads import WORKLOADS, Workload, head_inputs
from oracle import bsa_oracle as o
from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu

CASES = {
    # BASELINE config 0
    "tiny": WORKLOADS["tiny"],
    "tiny_p60": WORKLOADS["tiny"].replace(threshold=0.6, seed=1),
    # the flagship tile shape (4x4x4 blocks, d=128, bf16) on a small grid: several blocks, H=2
    "mini_wan": Workload("mini_wan", 1, 2, 128, "bf16", (8, 8, 12), (4, 4, 4), threshold=0.6),
    "mini_wan_r25": Workload("mini_wan_r25", 1, 2, 128, "bf16", (8, 8, 12), (4, 4, 4), threshold=0.8, keep_ratio=0.25),
    "mini_wan_r100": Workload("mini_wan_r100", 2, 1, 128, "bf16", (4, 8, 12), (4, 4, 4), threshold=0.5, keep_ratio=1.0),
    "mini_wan_d64": Workload("mini_wan_d64", 1, 3, 64, "bf16", (8, 4, 12), (4, 4, 4), threshold=0.7),
    # ragged everything: odd block extents, d not a power of two, batch 2
    "ragged_f32": Workload("ragged_f32", 2, 2, 72, "fp32", (6, 6, 10), (3, 2, 5), threshold=0.7, keep_ratio=0.4),
    "ragged_bf16": Workload("ragged_bf16", 1, 2, 64, "bf16", (4, 8, 16), (2, 4, 4), threshold=0.7, keep_ratio=0.3),
    # more blocks than one mask word, not a multiple of 32
    "n84": Workload("n84", 1, 2, 64, "bf16", (4, 12, 28), (2, 2, 4), threshold=0.5, keep_ratio=0.5),
    # degenerate: a single block; one retained query (the center alone)
    "one_block": Workload("one_block", 1, 1, 64, "fp32", (2, 4, 4), (2, 4, 4), keep_ratio=0.5),
    "keep_one": Workload("keep_one", 1, 2, 64, "fp32", (4, 8, 8), (2, 4, 4), threshold=0.6, keep_ratio=1 / 32),
    # maximum block size and head dimension
    "max_block": Workload("max_block", 1, 1, 256, "fp32", (8, 8, 8), (4, 8, 8), threshold=0.9, keep_ratio=0.3),
    # short launches on the MFMA path: on each XCD the walks of the last units are split over
    # several workgroups and merged by a combine launch (48 units; 60 units, not a multiple of 8,
    # last query-block group ragged, two wavefronts per query block)
    "split_tail": Workload("split_tail", 1, 2, 128, "bf16", (16, 16, 24), (4, 4, 4), threshold=0.7),
    "split_ragged": Workload("split_ragged", 1, 5, 64, "bf16", (12, 12, 20), (4, 4, 4), threshold=0.7, keep_ratio=0.75),
    # window-based critical tokens (Sec. 3.2.2): the paper's (2,2,2) windows in 4x4x4 blocks on the
    # MFMA path, small windows on the fp32 path, and windows that do not tile the block into a
    # power-of-two count (3 windows of a 3x2x4 block)
    "win_tiny": WORKLOADS["tiny"].replace(window=(1, 2, 2), threshold=0.6, seed=2),
    "win_wan": Workload("win_wan", 1, 2, 128, "bf16", (8, 8, 12), (4, 4, 4), threshold=0.6, window=(2, 2, 2)),
    "win_wan_r75": Workload("win_wan_r75", 1, 2, 64, "bf16", (8, 8, 12), (4, 4, 4), threshold=0.7, keep_ratio=0.75, window=(2, 4, 4)),
    "win_split": Workload("win_split", 1, 2, 128, "bf16", (16, 16, 24), (4, 4, 4), threshold=0.7, window=(2, 2, 2), seed=3),
    "win_ragged": Workload("win_ragged", 1, 2, 72, "fp32", (6, 6, 8), (3, 2, 4), threshold=0.7, keep_ratio=0.5, window=(1, 2, 4)),
    # block-major token order (the one-time reorder of Sec. 3.2.1) of the same videos
    "bm_tiny": WORKLOADS["tiny"].replace(block_major=True, threshold=0.6, seed=1),
    "bm_wan": Workload("mini_wan", 1, 2, 128, "bf16", (8, 8, 12), (4, 4, 4), threshold=0.6, block_major=True),
    "bm_win_split": Workload("win_split", 1, 2, 128, "bf16", (16, 16, 24), (4, 4, 4), threshold=0.7, window=(2, 2, 2), seed=3,
                             block_major=True),
    # 16 or fewer retained queries per block: a wavefront carries two query blocks.  A split tail with
    # windows; a block count that is not a multiple of eight (a wavefront with one real and one
    # missing block, a group with missing wavefronts); a single retained query per block
    "pack_win_split": Workload("pack_win_split", 1, 4, 128, "bf16", (16, 16, 24), (4, 4, 4), threshold=0.7, keep_ratio=0.25,
                               window=(2, 2, 2), seed=5),
    "pack_ragged": Workload("pack_ragged", 1, 5, 64, "bf16", (12, 12, 20), (4, 4, 4), threshold=0.7, keep_ratio=0.25),
    "pack_keep_one": Workload("pack_keep_one", 1, 2, 128, "bf16", (4, 8, 12), (4, 4, 4), threshold=0.6, keep_ratio=1 / 64),
    # threshold 1: every block selected
    "p_one": Workload("p_one", 1, 1, 64, "bf16", (4, 8, 8), (2, 4, 4), threshold=1.0, keep_ratio=0.5),
}


@functools.lru_cache(maxsize=None)
def run_case(name: str):
    wl = CASES[name]
    x = U.device_inputs(wl)
    shp, Qbar, Kbar, lists, keep = U.run_indices(wl, x)
    O, LSE = B.attn_fwd(shp, x["Q"], x["K"], x["V"], lists, keep)
    dQ, dK, dV = B.attn_bwd(shp, x["Q"], x["K"], x["V"], O, LSE, x["dO"], lists, keep)
    torch.cuda.synchronize()
    host = U.lists_to_host(shp, lists)
    ref, sigma = {}, {}
    part = U.part_of(wl)
    for b in range(wl.B):
        for h in range(wl.H):
            xi = head_inputs(wl, b, h)
            ref[b, h] = o.bsa_head(xi["Q"], xi["K"], xi["V"], xi["dO"], part, wl.threshold, wl.keep_ratio,
                                   o_storage=U.o_storage_of(wl))
            if wl.dtype == "bf16":
                sigma[b, h] = U.T.rounding_sigma(xi, part, ref[b, h][0], 1 / sqrt(wl.d))
    return dict(wl=wl, shp=shp, part=part, x=x, Qbar=Qbar, Kbar=Kbar, lists=lists, host=host, keep=keep,
                O=O, LSE=LSE, dQ=dQ, dK=dK, dV=dV, ref=ref, sigma=sigma, name=name)


def heads(r):
    return [(b, h) for b in range(r["wl"].B) for h in range(r["wl"].H)]


@pytest.mark.parametrize("name", list(CASES))
def test_pool_is_bit_exact(name):
    r = run_case(name)
    for b, h in heads(r):
        ix = r["ref"][b, h][0]
        assert np.array_equal(r["Qbar"][b, h].cpu().numpy(), ix.Qbar)
        assert np.array_equal(r["Kbar"][b, h].cpu().numpy(), ix.Kbar)


@pytest.mark.parametrize("name", list(CASES))
def test_keep_lists_are_bit_exact(name):
    r = run_case(name)
    for b, h in heads(r):
        assert np.array_equal(r["keep"][b, h].cpu().numpy(), r["ref"][b, h][0].keep_idx)


@pytest.mark.parametrize("name", list(CASES))
def test_kv_lists_and_transpose_are_bit_exact(name):
    r = run_case(name)
    wl = r["wl"]
    for b, h in heads(r):
        ix = r["ref"][b, h][0]
        assert ix.select_margin > U.SELECT_MARGIN  # identity below is meaningful, not luck
        assert U.check_lists_against_oracle(wl, r["shp"], r["host"], b, h, ix) == 0
    assert r["host"]["k2q_ptr"][-1] == r["host"]["nnz"]


@pytest.mark.parametrize("name", list(CASES))
def test_forward_matches_oracle(name):
    r = run_case(name)
    for b, h in heads(r):
        _, O, LSE, *_ = r["ref"][b, h]
        U.check_tensors(name, f"fwd b{b} h{h}", r["wl"].dtype, [("O", U.host_f64(r["O"][b, h]), O)],
                        lse=(U.host_f64(r["LSE"][b, h]), LSE))


@pytest.mark.parametrize("name", list(CASES))
def test_backward_matches_oracle(name):
    r = run_case(name)
    for b, h in heads(r):
        _, _, _, dQ, dK, dV = r["ref"][b, h]
        U.check_tensors(name, f"bwd b{b} h{h}", r["wl"].dtype,
                        [(t, U.host_f64(r[t][b, h]), ref) for t, ref in (("dQ", dQ), ("dK", dK), ("dV", dV))],
                        sigma=r["sigma"].get((b, h)))


@pytest.mark.parametrize("name", ["tiny", "mini_wan", "mini_wan_r25", "mini_wan_r100", "win_wan", "ragged_bf16"])
def test_backward_forms_delta_from_the_output_it_is_handed(name):
    """The backward call receives O (and LSE) as arguments.  Handed a stored O that is visibly not
    the forward's (the oracle's O plus noise of a quarter of its RMS) and the oracle's LSE, it must
    reproduce the oracle's backward for that same O: delta = <g, O> comes from the argument."""
    r = run_case(name)
    wl, shp, x, part = r["wl"], r["shp"], r["x"], r["part"]
    store = U.o_storage_of(wl)
    O2, L2 = torch.empty_like(r["O"]), torch.empty_like(r["LSE"])
    handed = {}
    for b, h in heads(r):
        _, O, LSE, *_ = r["ref"][b, h]
        rng = np.random.default_rng(1000 + 10 * b + h)
        handed[b, h] = np.asarray(store(O + 0.25 * sqrt(np.mean(O * O)) * rng.standard_normal(O.shape)), dtype=np.float64)
        O2[b, h] = torch.from_numpy(handed[b, h]).to(O2.dtype)  # exact: already rounded to the storage type
        L2[b, h] = torch.from_numpy(LSE).to(L2.dtype)
    dQ, dK, dV = B.attn_bwd(shp, x["Q"], x["K"], x["V"], O2, L2, x["dO"], r["lists"], r["keep"])
    torch.cuda.synchronize()
    scale = 1 / sqrt(wl.d)
    for b, h in heads(r):
        xi, ix = head_inputs(wl, b, h), r["ref"][b, h][0]
        rdQ, rdK, rdV = o.attn_bwd(xi["Q"], xi["K"], xi["V"], xi["dO"], part, ix.q2k_ptr, ix.q2k_idx, ix.keep_idx, scale,
                                   O_in=handed[b, h])
        sg = U.T.rounding_sigma(xi, part, ix, scale, own_forward=False, O_in=handed[b, h]) if wl.dtype == "bf16" else None
        U.check_tensors(name, f"bwd handed-O b{b} h{h}", wl.dtype,
                        [("dQ", U.host_f64(dQ[b, h]), rdQ), ("dK", U.host_f64(dK[b, h]), rdK), ("dV", U.host_f64(dV[b, h]), rdV)],
                        sigma=sg)


@pytest.mark.parametrize("name", ["tiny_p60", "mini_wan", "ragged_bf16", "win_tiny", "win_wan", "win_ragged"])
def test_fill_and_zero_rows_are_exact(name):
    r = run_case(name)
    part, tok = r["part"], r["part"].block_tokens()
    cof = part.center_of()
    for b, h in heads(r):
        keep = r["ref"][b, h][0].keep_idx
        O, LSE, dQ = (r[k][b, h].float().cpu().numpy() for k in ("O", "LSE", "dQ"))
        for i in range(part.N):
            pruned = np.setdiff1d(np.arange(part.Bk), keep[i])
            c = tok[i, cof[pruned]]  # each pruned token's window center
            assert np.array_equal(O[tok[i, pruned]], O[c])
            assert np.all(LSE[tok[i, pruned]] == LSE[c])
            assert not dQ[tok[i, pruned]].any()


@pytest.mark.parametrize("name", ["tiny", "mini_wan", "ragged_f32"])
def test_runs_are_deterministic(name):
    r = run_case(name)
    wl, shp, x = r["wl"], r["shp"], r["x"]
    _, _, _, lists, keep = U.run_indices(wl, x)
    O, LSE = B.attn_fwd(shp, x["Q"], x["K"], x["V"], lists, keep)
    dQ, dK, dV = B.attn_bwd(shp, x["Q"], x["K"], x["V"], O, LSE, x["dO"], lists, keep)
    torch.cuda.synchronize()
    nnz = r["host"]["nnz"]
    assert torch.equal(lists.q2k_idx[:nnz], r["lists"].q2k_idx[:nnz]) and torch.equal(lists.k2q_idx[:nnz], r["lists"].k2q_idx[:nnz])
    for a, b_ in ((O, r["O"]), (LSE, r["LSE"]), (dQ, r["dQ"]), (dK, r["dK"]), (dV, r["dV"])):
        assert torch.equal(a, b_)


@pytest.mark.parametrize("name", ["tiny", "mini_wan", "ragged_f32"])
def test_dense_baseline_is_full_attention(name):
    """Eq. 1: the in-repo dense kernel against the oracle at threshold 1, no pruning."""
    r = run_case(name)
    wl, shp, x = r["wl"], r["shp"], r["x"]
    O, LSE = B.dense_attn_fwd(shp, x["Q"], x["K"], x["V"])
    dQ, dK, dV = B.dense_attn_bwd(shp, x["Q"], x["K"], x["V"], O, LSE, x["dO"])
    torch.cuda.synchronize()
    for b, h in heads(r):
        xi = head_inputs(wl, b, h)
        ix, rO, rL, rdQ, rdK, rdV = o.bsa_head(xi["Q"], xi["K"], xi["V"], xi["dO"], r["part"], 1.0, 1.0,
                                               o_storage=U.o_storage_of(wl))
        sg = U.T.rounding_sigma(xi, r["part"], ix, 1 / sqrt(wl.d)) if wl.dtype == "bf16" else None
        U.check_tensors(name + " dense", f"b{b} h{h}", wl.dtype,
                        [(t, U.host_f64(got[b, h]), ref) for t, got, ref in (("O", O, rO), ("dQ", dQ, rdQ), ("dK", dK, rdK), ("dV", dV, rdV))],
                        sigma=sg, lse=(U.host_f64(LSE[b, h]), rL))


def test_sparse_path_at_threshold_one_equals_dense_path():
    r = run_case("p_one")
    shp, x = r["shp"], r["x"]
    assert r["host"]["nnz"] == shp.rows * shp.N
    # with no pruning as well, the sparse kernels compute Eq. 1
    wl = r["wl"].replace(keep_ratio=1.0)
    _, _, _, lists, keep = U.run_indices(wl, x)
    O, LSE = B.attn_fwd(shp, x["Q"], x["K"], x["V"], lists, keep)
    Od, Ld = B.dense_attn_fwd(shp, x["Q"], x["K"], x["V"])
    torch.cuda.synchronize()
    assert U.rel_err(U.host_f64(O), U.host_f64(Od)) < 2e-2
    assert (LSE - Ld).abs().max().item() < 1e-4


@pytest.mark.parametrize("raster,tiled", [("tiny_p60", "bm_tiny"), ("mini_wan", "bm_wan"), ("win_split", "bm_win_split")])
def test_block_major_layout_is_a_pure_permutation_of_the_raster_results(raster, tiled):
    """Same video, two token orders: every output of the block-major run is the raster run's
    output with its rows reordered, bit for bit (same tiles, same arithmetic order)."""
    from bsa_workloads import block_major_order

    a, b = run_case(raster), run_case(tiled)
    wl = a["wl"]
    assert b["wl"].replace(block_major=False) == wl.replace(name=b["wl"].name)
    order = torch.from_numpy(block_major_order(wl.grid, wl.block)).cuda()
    assert torch.equal(a["lists"].q2k_ptr, b["lists"].q2k_ptr) and torch.equal(a["keep"], b["keep"])
    nnz = a["host"]["nnz"]
    assert torch.equal(a["lists"].q2k_idx[:nnz], b["lists"].q2k_idx[:nnz])
    for name in ("O", "dQ", "dK", "dV"):
        assert torch.equal(a[name][:, :, order], b[name]), name
    assert torch.equal(a["LSE"][:, :, order], b["LSE"])


def test_whole_step_is_graph_capturable_and_replays_bit_identically():
    """The library allocates nothing, never synchronises and launches only kernels: one layer
    (all five calls, caller-owned buffers) is captured into a HIP graph; every replay, with
    eager work and synchronisations in between, must reproduce the eager results bit for bit."""
    wl = CASES["win_split"]
    shp = U.shape_of(wl)
    x = U.device_inputs(wl)
    dev = x["Q"].device
    nk = B.n_keep(shp, wl.keep_ratio)
    Qbar = torch.empty((wl.B, wl.H, shp.N, wl.d), dtype=torch.float64, device=dev)
    Kbar = torch.empty_like(Qbar)
    lists = B.alloc_kv_lists(shp, dev)
    keep = torch.empty((wl.B, wl.H, shp.N, nk), dtype=torch.int32, device=dev)
    O, dQ, dK, dV = (torch.empty_like(x["Q"]) for _ in range(4))
    LSE = torch.empty((wl.B, wl.H, wl.L), dtype=torch.float32, device=dev)
    ws = torch.empty(max(1, B.bwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)
    fws = torch.empty(max(1, B.fwd_workspace_bytes(shp, nk)), dtype=torch.uint8, device=dev)

    def step():
        B.pool_blocks(shp, x["Q"], Qbar)
        B.pool_blocks(shp, x["K"], Kbar)
        B.select_kv(shp, Qbar, Kbar, wl.threshold, out=lists)
        B.prune_q(shp, x["Q"], wl.keep_ratio, keep)
        B.attn_fwd(shp, x["Q"], x["K"], x["V"], lists, keep, O=O, LSE=LSE, workspace=fws)
        B.attn_bwd(shp, x["Q"], x["K"], x["V"], O, LSE, x["dO"], lists, keep, dQ=dQ, dK=dK, dV=dV, workspace=ws)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (O, LSE, dQ, dK, dV, lists.q2k_ptr, lists.k2q_ptr, keep)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream, as torch asks
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (O, LSE, dQ, dK, dV, keep):
            t.zero_()  # eager work between the replays
        lists.q2k_ptr.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b_ in zip(ref, (O, LSE, dQ, dK, dV, lists.q2k_ptr, lists.k2q_ptr, keep)):
            assert torch.equal(a, b_), rep
