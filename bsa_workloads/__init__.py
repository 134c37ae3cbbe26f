"""Seeded synthetic video-shaped inputs and the named workload table.

This module holds no arithmetic of the attention method itself: it only draws
the Q/K/V/dO tensors (smooth spatiotemporal field + Gaussian noise) and lists
the shapes of the named workloads.  Both the CPU oracle's tests and the HIP
path's tests/benchmark import it; neither of those two imports the other.
"""
from .video_fields import (  # noqa: F401
    Workload,
    WORKLOADS,
    TENSOR_NAMES,
    head_tensor,
    head_inputs,
    block_major_order,
    bf16_round,
    bf16_bits,
    bf16_from_bits,
)
