"""The register-resident matrix-core loop used as the measured MFMA ceiling: it must really
perform the products it is credited with.  Its operands are small exact values, so the sum
every lane reports has a closed form on the host."""
import numpy as np
import pytest
import torch

from paper_2509_01085_amd import binding as B

import gpu_util as U

pytestmark = pytest.mark.gpu


def test_probe_counts_and_computes_what_it_claims():
    U.progress("mfma probe")
    wgs, iters = 8, 300
    sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    flops = B.mfma_probe(wgs, iters, sink)
    assert flops == wgs * 4 * iters * 4 * 2 * 32 * 32 * 16
    got = sink.cpu().numpy().reshape(wgs * 4, 64)
    # A[i][k] = ((i + k) mod 4) / 4, B[k][j] = 2^-10 where (j xor k) is even, else 0 (k taken mod 8)
    A = np.array([[((i + (k % 8)) & 3) * 0.25 for k in range(16)] for i in range(32)])
    Bm = np.array([[0.0 if ((j ^ (k % 8)) & 1) else 2.0 ** -10 for j in range(32)] for k in range(16)])
    Cm = A @ Bm
    expect = np.empty(64)
    for lane in range(64):
        rows = [8 * (r // 4) + 4 * (lane // 32) + r % 4 for r in range(16)]
        expect[lane] = 4 * iters * Cm[rows, lane % 32].sum()
    assert np.array_equal(got, np.broadcast_to(expect.astype(np.float32), got.shape))


def test_probe_rejects_bad_arguments():
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    assert B.lib().bsa_mfma_probe(0, 1, sink.data_ptr(), None) < 0
    assert B.lib().bsa_mfma_probe(1, 0, sink.data_ptr(), None) < 0
    assert B.lib().bsa_mfma_probe(1, 1, None, None) < 0
