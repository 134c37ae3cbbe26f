"""Synthetic stand-ins for video-DiT attention activations.

Each of Q, K, V is a smooth spatiotemporal field over the latent grid
(a sum of four unit-amplitude low-frequency sinusoids per channel) plus
white Gaussian noise; dO is white noise.  The smooth part gives neighbouring
tokens similar features (so query pruning has redundancy to remove) and gives
block-level scores structure (so the cumulative-mass selection keeps a
content-dependent subset); the noise level moves the within-block similarity.

Every (tensor, batch, head) slice has its own random stream, so a single head
of a large workload can be generated without drawing the others.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import ceil
from typing import Dict, Tuple

import numpy as np

TENSOR_NAMES = ("Q", "K", "V", "dO")
_N_SINUSOIDS = 4
_MAX_FREQ = 2  # integer frequencies drawn from {0, 1, 2} per axis


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    d: int
    dtype: str  # "fp32" or "bf16"
    grid: Tuple[int, int, int]  # (T, Hs, Ws)
    block: Tuple[int, int, int]  # (Ct, Ch, Cw)
    sigma: float = 0.3
    threshold: float = 0.9
    keep_ratio: float = 0.5
    seed: int = 0
    window: Tuple[int, int, int] = (0, 0, 0)  # critical-token window; zeros = the whole block
    block_major: bool = False  # token order of the tensors: raster, or the tokens of a block adjacent

    @property
    def L(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]

    @property
    def Bk(self) -> int:
        return self.block[0] * self.block[1] * self.block[2]

    @property
    def N(self) -> int:
        return self.L // self.Bk

    @property
    def n_keep(self) -> int:
        wk = (self.window[0] or self.block[0]) * (self.window[1] or self.block[1]) * (self.window[2] or self.block[2])
        return (self.Bk // wk) * int(ceil(self.keep_ratio * wk - 1e-12))

    def replace(self, **kw) -> "Workload":
        from dataclasses import replace as _r

        return _r(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # 256 tokens, 8 blocks of 32: the case the CPU oracle finishes instantly.
    "tiny": Workload("tiny", 1, 2, 64, "fp32", (4, 8, 8), (2, 4, 4)),
    # Wan-1.3B-shaped layer, 33,280 tokens, 520 blocks of 64.
    "wan1p3b": Workload("wan1p3b", 1, 12, 128, "bf16", (20, 32, 52), (4, 4, 4)),
    # the same layer with the paper's default critical-token windows, (2,2,2) inside each block
    "wan1p3b_win": Workload("wan1p3b_win", 1, 12, 128, "bf16", (20, 32, 52), (4, 4, 4), window=(2, 2, 2)),
    # 720p-shaped layer, 70,400 tokens, 1,100 blocks.
    "hd720p": Workload("hd720p", 1, 40, 128, "bf16", (20, 44, 80), (4, 4, 4)),
    # long-sequence layer, 161,280 tokens, 2,520 blocks.
    "long": Workload("long", 1, 12, 128, "bf16", (40, 48, 84), (4, 4, 4)),
}


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 holding the same values."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bfloat16, returned as float32."""
    return bf16_from_bits(bf16_bits(x))


def _smooth_field(rng: np.random.Generator, grid, d: int) -> np.ndarray:
    T, Hs, Ws = grid
    freqs = rng.integers(0, _MAX_FREQ + 1, size=(d, _N_SINUSOIDS, 3))
    # a sinusoid with all-zero frequency would be a constant: redraw those
    while True:
        dead = ~freqs.any(axis=2)
        if not dead.any():
            break
        freqs[dead] = rng.integers(0, _MAX_FREQ + 1, size=(int(dead.sum()), 3))
    phase = rng.uniform(0.0, 2.0 * np.pi, size=(d, _N_SINUSOIDS))
    two_pi_i = 2j * np.pi
    et = np.exp(two_pi_i * np.arange(T)[:, None, None] * freqs[None, :, :, 0] / T)
    eh = np.exp(two_pi_i * np.arange(Hs)[:, None, None] * freqs[None, :, :, 1] / Hs)
    ew = np.exp(two_pi_i * np.arange(Ws)[:, None, None] * freqs[None, :, :, 2] / Ws)
    eth = et[:, None] * eh[None, :] * np.exp(1j * phase)[None, None]  # [T,Hs,d,m]
    field = np.einsum("thcm,wcm->thwc", eth, ew).imag  # sum over the sinusoids
    return field.reshape(T * Hs * Ws, d)


def head_tensor(wl: Workload, which: str, b: int, h: int) -> np.ndarray:
    """One [L, d] float32 slice of tensor `which` in the workload's token order.

    For bf16 workloads the values are already rounded to bfloat16, so what
    the CPU oracle reads equals what the device holds."""
    tid = TENSOR_NAMES.index(which)
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([wl.seed, tid, b, h])))
    if which == "dO":
        x = rng.standard_normal((wl.L, wl.d), dtype=np.float32)
    else:
        field = _smooth_field(rng, wl.grid, wl.d)
        noise = rng.standard_normal((wl.L, wl.d), dtype=np.float32)
        x = (field + np.float64(wl.sigma) * noise).astype(np.float32)
    if wl.dtype == "bf16":
        x = bf16_round(x)
    if wl.block_major:  # the same video, rows reordered so that the tokens of a block are adjacent
        x = np.ascontiguousarray(x[block_major_order(wl.grid, wl.block)])
    return x


def block_major_order(grid: Tuple[int, int, int], block: Tuple[int, int, int]) -> np.ndarray:
    """order[i*Bk + c] = raster index of intra-block token c of block i (blocks and the tokens
    inside a block both numbered raster-wise): a pure index permutation, no arithmetic."""
    T, Hs, Ws = grid
    Ct, Ch, Cw = block
    n = np.arange(T * Hs * Ws, dtype=np.int64).reshape(T // Ct, Ct, Hs // Ch, Ch, Ws // Cw, Cw)
    return n.transpose(0, 2, 4, 1, 3, 5).reshape(-1)


def head_inputs(wl: Workload, b: int, h: int) -> Dict[str, np.ndarray]:
    return {name: head_tensor(wl, name, b, h) for name in TENSOR_NAMES}
