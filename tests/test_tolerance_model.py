"""Why the bf16 parity bound has a relative term: storing the EXACT gradient in bfloat16
already moves its largest entries by more than 2e-2 of the tensor's RMS.  Pure CPU, no kernel:
the oracle's fp64 gradients of a flagship-shaped case are rounded to bf16 and compared with
themselves.  The test pins the two facts the GPU parity bound rests on:
  * max |bf16(x) - x| / RMS(x) exceeds 2e-2 for the gradient tensors (heavy tails: the fill
    gradient folds many dO rows into each critical token's row), so a plain 2e-2 * RMS bound
    cannot be met by any implementation that returns bf16;
  * |bf16(x) - x| <= 2^-8 |x| element by element, which is the term the bound adds."""
from math import sqrt

import numpy as np

from bsa_workloads import Workload, bf16_round, head_inputs
from oracle import bsa_oracle as o

CASE = Workload("mini_wan", 1, 2, 128, "bf16", (8, 8, 12), (4, 4, 4), threshold=0.6)


def test_bf16_storage_alone_exceeds_the_plain_relative_rms_figure():
    part = o.Partition(*CASE.grid, *CASE.block)
    worst = {}
    for h in range(CASE.H):
        x = head_inputs(CASE, 0, h)
        _, O, _, dQ, dK, dV = o.bsa_head(x["Q"], x["K"], x["V"], x["dO"], part, CASE.threshold, CASE.keep_ratio)
        for name, t in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
            err = np.abs(bf16_round(t.astype(np.float32)).astype(np.float64) - t)
            assert np.all(err <= 2.0 ** -8 * np.abs(t) + 1e-30)  # round-to-nearest: half an ulp of 8 significant bits
            worst[name] = max(worst.get(name, 0.0), float(err.max() / sqrt(np.mean(t * t))))
    # the outputs are averages of V rows (light tails) and stay below the figure ...
    assert worst["O"] < 2e-2
    # ... the gradients do not
    assert max(worst["dQ"], worst["dK"], worst["dV"]) > 2e-2, worst
