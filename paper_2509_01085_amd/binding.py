"""ctypes binding of libbsa.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device
memory (tensors) and the stream.  The functions mirror the C ABI of include/bsa.h
name for name (without the `bsa_` prefix) and raise BsaError on a negative status.
Importing this module fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from math import sqrt
from typing import Optional

import torch

# BSA_LIB selects another build of the same library (e.g. one compiled with different tuning flags)
_LIB_PATH = os.environ.get("BSA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbsa.so")

F32, BF16 = 0, 1
RASTER, BLOCK_MAJOR = 0, 1
EXPORTS = (
    "bsa_strerror", "bsa_n_keep", "bsa_pool_blocks", "bsa_select_workspace_bytes", "bsa_select_kv",
    "bsa_select_kv_stat", "bsa_select_kv_static", "bsa_prune_q", "bsa_fwd_workspace_bytes", "bsa_attn_fwd", "bsa_bwd_workspace_bytes", "bsa_attn_bwd", "bsa_attn_bwd_stages",
    "bsa_dense_bwd_workspace_bytes", "bsa_dense_attn_fwd", "bsa_dense_attn_bwd", "bsa_mfma_probe",
)


class BsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().bsa_strerror(status).decode()} (status {status})")


class ShapeStruct(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "T", "Hs", "Ws", "Ct", "Ch", "Cw", "d", "dtype", "Wt", "Wh", "Ww", "layout")]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2509_01085_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(_LIB_PATH)
        P, vp, i32, i64, f32, f64, sz = C.POINTER(ShapeStruct), C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_double, C.c_size_t
        L.bsa_strerror.restype, L.bsa_strerror.argtypes = C.c_char_p, [C.c_int]
        L.bsa_n_keep.restype, L.bsa_n_keep.argtypes = C.c_int, [P, f64]
        L.bsa_pool_blocks.restype, L.bsa_pool_blocks.argtypes = C.c_int, [P, vp, vp, vp]
        L.bsa_select_workspace_bytes.restype, L.bsa_select_workspace_bytes.argtypes = sz, [P]
        L.bsa_select_kv.restype = C.c_int
        L.bsa_select_kv.argtypes = [P, vp, vp, f64, f64, vp, vp, i64, vp, vp, vp, vp, sz, vp]
        L.bsa_select_kv_stat.restype = C.c_int
        L.bsa_select_kv_stat.argtypes = [P, vp, vp, f64, f64, f64, vp, vp, i64, vp, vp, vp, vp, sz, vp]
        L.bsa_select_kv_static.restype = C.c_int
        L.bsa_select_kv_static.argtypes = [P, vp, vp, f64, f64, vp, vp, i64, vp, vp, vp, vp]
        L.bsa_prune_q.restype, L.bsa_prune_q.argtypes = C.c_int, [P, vp, f64, vp, vp]
        L.bsa_attn_fwd.restype = C.c_int
        L.bsa_attn_fwd.argtypes = [P, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, vp, sz, vp]
        L.bsa_fwd_workspace_bytes.restype, L.bsa_fwd_workspace_bytes.argtypes = sz, [P, i32]
        L.bsa_bwd_workspace_bytes.restype, L.bsa_bwd_workspace_bytes.argtypes = sz, [P, i32]
        L.bsa_attn_bwd.restype = C.c_int
        L.bsa_attn_bwd.argtypes = [P] + [vp] * 11 + [i32, f32, vp, vp, vp, vp, sz, vp]
        L.bsa_attn_bwd_stages.restype = C.c_int
        L.bsa_attn_bwd_stages.argtypes = [P] + [vp] * 11 + [i32, f32, vp, vp, vp, vp, sz, C.c_uint, vp]
        L.bsa_dense_bwd_workspace_bytes.restype, L.bsa_dense_bwd_workspace_bytes.argtypes = sz, [P]
        L.bsa_dense_attn_fwd.restype = C.c_int
        L.bsa_dense_attn_fwd.argtypes = [P, vp, vp, vp, f32, vp, vp, vp]
        L.bsa_dense_attn_bwd.restype = C.c_int
        L.bsa_dense_attn_bwd.argtypes = [P] + [vp] * 6 + [f32, vp, vp, vp, vp, sz, vp]
        L.bsa_mfma_probe.restype, L.bsa_mfma_probe.argtypes = i64, [i32, i32, vp, vp]
        _lib = L
    return _lib


@dataclass(frozen=True)
class Shape:
    B: int
    H: int
    T: int
    Hs: int
    Ws: int
    Ct: int
    Ch: int
    Cw: int
    d: int
    dtype: int  # F32 or BF16
    Wt: int = 0  # window of the critical-token mechanism; 0, 0, 0 = the whole block
    Wh: int = 0
    Ww: int = 0
    layout: int = 0  # RASTER or BLOCK_MAJOR

    @property
    def L(self) -> int:
        return self.T * self.Hs * self.Ws

    @property
    def Bk(self) -> int:
        return self.Ct * self.Ch * self.Cw

    @property
    def N(self) -> int:
        return self.L // self.Bk

    @property
    def rows(self) -> int:
        return self.B * self.H * self.N

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == F32 else torch.bfloat16

    def c(self) -> ShapeStruct:
        return ShapeStruct(self.B, self.H, self.T, self.Hs, self.Ws, self.Ct, self.Ch, self.Cw, self.d, self.dtype,
                           self.Wt, self.Wh, self.Ww, self.layout)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "libbsa takes contiguous tensors"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status < 0:
        raise BsaError(status, where)


def n_keep(shape: Shape, keep_ratio: float) -> int:
    n = lib().bsa_n_keep(C.byref(shape.c()), keep_ratio)
    _check(n, "bsa_n_keep")
    return n


def pool_blocks(shape: Shape, X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty((shape.B, shape.H, shape.N, shape.d), dtype=torch.float64, device=X.device)
    _check(lib().bsa_pool_blocks(C.byref(shape.c()), _ptr(X), _ptr(out), _stream()), "bsa_pool_blocks")
    return out


@dataclass
class KvLists:
    q2k_ptr: torch.Tensor  # [rows+1] int32
    q2k_idx: torch.Tensor  # [rows*N] int32 (first nnz valid)
    k2q_ptr: Optional[torch.Tensor]
    k2q_idx: Optional[torch.Tensor]
    nnz: torch.Tensor  # int64 device scalar
    workspace: torch.Tensor


def select_workspace_bytes(shape: Shape) -> int:
    return lib().bsa_select_workspace_bytes(C.byref(shape.c()))


STATIC_SELECT_BYTES = 32 << 20  # BSA_STATIC_SELECT_BYTES of the header


def alloc_kv_lists(shape: Shape, device, transpose: bool = True, workspace: bool = True) -> KvLists:
    cap = shape.rows * shape.N
    i32 = dict(dtype=torch.int32, device=device)
    return KvLists(
        torch.empty(shape.rows + 1, **i32), torch.empty(cap, **i32),
        torch.empty(shape.rows + 1, **i32) if transpose else None,
        torch.empty(cap, **i32) if transpose else None,
        torch.zeros(1, dtype=torch.int64, device=device),
        torch.empty(select_workspace_bytes(shape) if workspace else 0, dtype=torch.uint8, device=device))


def select_kv_static(shape: Shape, Qbar: torch.Tensor, Kbar: torch.Tensor, threshold: float, out: KvLists,
                     score_scale: Optional[float] = None) -> KvLists:
    """bsa_select_kv_static: the selection with the library's built-in scratch; `out` (lists and
    the nnz scalar, no workspace needed) comes from the caller, the call allocates nothing."""
    if score_scale is None:
        score_scale = 1.0 / sqrt(shape.d)
    st = lib().bsa_select_kv_static(C.byref(shape.c()), _ptr(Qbar), _ptr(Kbar), threshold, score_scale,
                                    _ptr(out.q2k_ptr), _ptr(out.q2k_idx), out.q2k_idx.numel(), _ptr(out.k2q_ptr),
                                    _ptr(out.k2q_idx), _ptr(out.nnz), _stream())
    _check(st, "bsa_select_kv_static")
    return out


def select_kv(shape: Shape, Qbar: torch.Tensor, Kbar: torch.Tensor, threshold: float,
              score_scale: Optional[float] = None, out: Optional[KvLists] = None,
              transpose: bool = True, stat_z: Optional[float] = None) -> KvLists:
    """stat_z: the quantile U(1 - k/n) of Eq. 3, supplied by the caller; None = plain Eq. 4."""
    if out is None:
        out = alloc_kv_lists(shape, Qbar.device, transpose)
    if score_scale is None:
        score_scale = 1.0 / sqrt(shape.d)
    tail = (_ptr(out.q2k_ptr), _ptr(out.q2k_idx), out.q2k_idx.numel(), _ptr(out.k2q_ptr), _ptr(out.k2q_idx),
            _ptr(out.nnz), _ptr(out.workspace), out.workspace.numel(), _stream())
    if stat_z is None:
        st = lib().bsa_select_kv(C.byref(shape.c()), _ptr(Qbar), _ptr(Kbar), threshold, score_scale, *tail)
    else:
        st = lib().bsa_select_kv_stat(C.byref(shape.c()), _ptr(Qbar), _ptr(Kbar), threshold, stat_z, score_scale, *tail)
    _check(st, "bsa_select_kv")
    return out


def prune_q(shape: Shape, Q: torch.Tensor, keep_ratio: float, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    nk = n_keep(shape, keep_ratio)
    if out is None:
        out = torch.empty((shape.B, shape.H, shape.N, nk), dtype=torch.int32, device=Q.device)
    _check(lib().bsa_prune_q(C.byref(shape.c()), _ptr(Q), keep_ratio, _ptr(out), _stream()), "bsa_prune_q")
    return out


def fwd_workspace_bytes(shape: Shape, n_keep_: int) -> int:
    return lib().bsa_fwd_workspace_bytes(C.byref(shape.c()), n_keep_)


def attn_fwd(shape: Shape, Q, K, V, lists: KvLists, keep_idx: torch.Tensor, sm_scale: Optional[float] = None,
             O: Optional[torch.Tensor] = None, LSE: Optional[torch.Tensor] = None,
             workspace: Optional[torch.Tensor] = None):
    nk = keep_idx.shape[-1]
    if workspace is None:
        workspace = torch.empty(max(1, fwd_workspace_bytes(shape, nk)), dtype=torch.uint8, device=Q.device)
    if sm_scale is None:
        sm_scale = 1.0 / sqrt(shape.d)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((shape.B, shape.H, shape.L), dtype=torch.float32, device=Q.device)
    st = lib().bsa_attn_fwd(C.byref(shape.c()), _ptr(Q), _ptr(K), _ptr(V), _ptr(lists.q2k_ptr), _ptr(lists.q2k_idx),
                            _ptr(keep_idx), nk, sm_scale, _ptr(O), _ptr(LSE), _ptr(workspace), workspace.numel(),
                            _stream())
    _check(st, "bsa_attn_fwd")
    return O, LSE


def bwd_workspace_bytes(shape: Shape, n_keep_: int) -> int:
    return lib().bsa_bwd_workspace_bytes(C.byref(shape.c()), n_keep_)


BWD_PRE, BWD_DQ, BWD_DKV = 1, 2, 4


def attn_bwd(shape: Shape, Q, K, V, O, LSE, dO, lists: KvLists, keep_idx: torch.Tensor,
             sm_scale: Optional[float] = None, dQ=None, dK=None, dV=None, workspace: Optional[torch.Tensor] = None,
             stages: Optional[int] = None):
    if sm_scale is None:
        sm_scale = 1.0 / sqrt(shape.d)
    nk = keep_idx.shape[-1]
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if workspace is None:
        workspace = torch.empty(max(1, bwd_workspace_bytes(shape, nk)), dtype=torch.uint8, device=Q.device)
    args = (C.byref(shape.c()), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO),
            _ptr(lists.q2k_ptr), _ptr(lists.q2k_idx), _ptr(lists.k2q_ptr), _ptr(lists.k2q_idx),
            _ptr(keep_idx), nk, sm_scale, _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), workspace.numel())
    if stages is None:
        st = lib().bsa_attn_bwd(*args, _stream())
    else:
        st = lib().bsa_attn_bwd_stages(*args, stages, _stream())
    _check(st, "bsa_attn_bwd")
    return dQ, dK, dV


def dense_bwd_workspace_bytes(shape: Shape) -> int:
    return lib().bsa_dense_bwd_workspace_bytes(C.byref(shape.c()))


def dense_attn_fwd(shape: Shape, Q, K, V, sm_scale: Optional[float] = None, O=None, LSE=None):
    if sm_scale is None:
        sm_scale = 1.0 / sqrt(shape.d)
    O = torch.empty_like(Q) if O is None else O
    if LSE is None:
        LSE = torch.empty((shape.B, shape.H, shape.L), dtype=torch.float32, device=Q.device)
    st = lib().bsa_dense_attn_fwd(C.byref(shape.c()), _ptr(Q), _ptr(K), _ptr(V), sm_scale, _ptr(O), _ptr(LSE), _stream())
    _check(st, "bsa_dense_attn_fwd")
    return O, LSE


def dense_attn_bwd(shape: Shape, Q, K, V, O, LSE, dO, sm_scale: Optional[float] = None,
                   dQ=None, dK=None, dV=None, workspace=None):
    if sm_scale is None:
        sm_scale = 1.0 / sqrt(shape.d)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if workspace is None:
        workspace = torch.empty(max(1, dense_bwd_workspace_bytes(shape)), dtype=torch.uint8, device=Q.device)
    st = lib().bsa_dense_attn_bwd(C.byref(shape.c()), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO),
                                  sm_scale, _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "bsa_dense_attn_bwd")
    return dQ, dK, dV


def mfma_probe(workgroups: int, iters: int, sink=None) -> int:
    """Enqueue the register-resident matrix-core loop; returns the flops the launch performs."""
    if sink is None:
        sink = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    if sink.numel() < workgroups * 256:
        raise ValueError("sink too small")
    flops = lib().bsa_mfma_probe(workgroups, iters, _ptr(sink), _stream())
    if flops < 0:
        _check(int(flops), "bsa_mfma_probe")
    return int(flops)
