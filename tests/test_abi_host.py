"""Host-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before launching anything (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2509_01085_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOOD = B.Shape(1, 2, 4, 8, 8, 2, 4, 4, 64, B.F32)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bsa.h")).read()
    declared = set(re.findall(r"\b(bsa_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_and_n_keep():
    lib = B.lib()
    assert lib.bsa_strerror(0) == b"ok"
    for st in range(-7, 0):
        assert b"unknown" not in lib.bsa_strerror(st)
    assert B.n_keep(GOOD, 0.5) == 16
    assert B.n_keep(GOOD, 1.0) == 32
    assert B.n_keep(GOOD, 1 / 32) == 1
    assert B.n_keep(B.Shape(1, 12, 20, 32, 52, 4, 4, 4, 128, B.BF16), 0.5) == 32  # Sec. 4.1
    for r in (0.0, -1.0, 1.01, float("nan")):
        with pytest.raises(B.BsaError) as e:
            B.n_keep(GOOD, r)
        assert e.value.status == -3


@pytest.mark.parametrize("field,value,status", [
    ("Ct", 3, -2), ("Cw", 5, -2), ("d", 60, -2), ("d", 264, -2), ("B", 0, -2), ("T", -4, -2),
    ("dtype", 7, -5),
])
def test_shape_validation(field, value, status):
    import dataclasses
    bad = dataclasses.replace(GOOD, **{field: value})
    assert B.lib().bsa_n_keep(C.byref(bad.c()), 0.5) == status
    assert B.lib().bsa_pool_blocks(C.byref(bad.c()), 16, 16, None) == status
    assert B.select_workspace_bytes(bad) == 0


def test_limits_on_block_and_block_count():
    too_big_block = B.Shape(1, 1, 8, 16, 16, 8, 8, 8, 64, B.F32)  # Bk = 512
    assert B.lib().bsa_n_keep(C.byref(too_big_block.c()), 0.5) == -2
    too_many_blocks = B.Shape(1, 1, 32, 32, 32, 1, 1, 2, 64, B.F32)  # N = 16384
    assert B.lib().bsa_n_keep(C.byref(too_many_blocks.c()), 0.5) == -2


def test_null_range_capacity_workspace_errors_come_before_any_launch():
    lib, s = B.lib(), C.byref(GOOD.c())
    p = 4096  # a non-NULL dummy address: these calls must fail validation and never touch it
    assert lib.bsa_pool_blocks(None, p, p, None) == -1
    assert lib.bsa_pool_blocks(s, None, p, None) == -1
    assert lib.bsa_prune_q(s, p, 0.5, None, None) == -1
    assert lib.bsa_prune_q(s, p, 0.0, p, None) == -3
    rows_n = GOOD.rows * GOOD.N
    ws = B.select_workspace_bytes(GOOD)
    assert ws >= GOOD.rows * GOOD.N * 8
    sel = lambda **k: lib.bsa_select_kv(s, k.get("qb", p), p, k.get("thr", 0.9), 0.125, p, p, k.get("cap", rows_n),
                                        k.get("kp", p), k.get("ki", p), None, k.get("ws", p), k.get("wsb", ws), None)
    assert sel(qb=None) == -1
    assert sel(thr=0.0) == -3 and sel(thr=1.5) == -3
    assert sel(cap=rows_n - 1) == -4
    assert sel(ws=None) == -7 and sel(wsb=ws - 1) == -7
    assert sel(kp=None) == -1  # k2q pointers: both or neither
    stat = lambda z, **k: lib.bsa_select_kv_stat(s, k.get("qb", p), p, 0.9, z, 0.125, p, p, k.get("cap", rows_n), p, p, None, p, ws, None)
    assert stat(float("nan")) == -3 and stat(0.5, qb=None) == -1 and stat(float("-inf"), cap=rows_n - 1) == -4
    # the variant with the library's built-in scratch: same checks, in the same order, and a
    # shape whose scratch would not fit is refused before anything touches the device
    stc = lambda sh=s, **k: lib.bsa_select_kv_static(sh, k.get("qb", p), p, k.get("thr", 0.9), 0.125, p, p,
                                                     k.get("cap", rows_n), k.get("kp", p), p, None, None)
    assert stc(qb=None) == -1 and stc(thr=0.0) == -3 and stc(cap=rows_n - 1) == -4 and stc(kp=None) == -1
    hd = B.Shape(1, 40, 20, 44, 80, 4, 4, 4, 128, B.BF16)
    assert B.select_workspace_bytes(hd) > B.STATIC_SELECT_BYTES
    assert stc(C.byref(hd.c()), cap=hd.rows * hd.N) == -8
    assert b"built-in" in lib.bsa_strerror(-8)
    wan = B.Shape(1, 12, 20, 32, 52, 4, 4, 4, 128, B.BF16)
    assert B.select_workspace_bytes(wan) <= B.STATIC_SELECT_BYTES
    assert lib.bsa_attn_fwd(s, p, p, p, p, p, p, 0, 0.125, p, p, None, 0, None) == -3
    assert lib.bsa_attn_fwd(s, p, p, p, p, p, p, 33, 0.125, p, p, None, 0, None) == -3
    assert lib.bsa_attn_fwd(s, p, p, None, p, p, p, 16, 0.125, p, p, None, 0, None) == -1
    # windows of the critical-token mechanism must divide the block; the quota is per window
    wshape = lambda *w: C.byref(B.Shape(1, 2, 4, 8, 8, 2, 4, 4, 64, B.F32, *w).c())
    assert lib.bsa_n_keep(wshape(1, 2, 2), 0.5) == 8 * 2 and lib.bsa_n_keep(wshape(2, 4, 4), 0.5) == 16
    assert lib.bsa_n_keep(wshape(1, 2, 2), 0.3) == 8 * 2  # ceil(0.3 * 4) per window
    assert lib.bsa_n_keep(wshape(1, 3, 2), 0.5) == -2 and lib.bsa_n_keep(wshape(-1, 2, 2), 0.5) == -2
    assert B.fwd_workspace_bytes(GOOD, 16) == 0  # fp32 shapes run the plain kernels: nothing to split
    big = B.Shape(1, 12, 20, 32, 52, 4, 4, 4, 128, B.BF16)  # a short launch on the MFMA path: the tail is split
    fws = B.fwd_workspace_bytes(big, 32)
    assert fws > 0 and B.bwd_workspace_bytes(big, 32) > big.rows * 16640
    sb = C.byref(big.c())
    assert lib.bsa_attn_fwd(sb, p, p, p, p, p, p, 32, 0.125, p, p, None, fws, None) == -7
    assert lib.bsa_attn_fwd(sb, p, p, p, p, p, p, 32, 0.125, p, p, p, fws - 1, None) == -7
    wsb = B.bwd_workspace_bytes(GOOD, 16)
    assert wsb > 0 and B.bwd_workspace_bytes(GOOD, 0) == 0
    bwd = lambda ws, wsbytes, nk=16: lib.bsa_attn_bwd(s, *([p] * 11), nk, 0.125, p, p, p, ws, wsbytes, None)
    assert bwd(None, wsb) == -7 and bwd(p, wsb - 1) == -7 and bwd(p, wsb, 40) == -3
    assert lib.bsa_dense_attn_fwd(s, p, p, None, 0.125, p, p, None) == -1
    dws = B.dense_bwd_workspace_bytes(GOOD)
    assert lib.bsa_dense_attn_bwd(s, *([p] * 6), 0.125, p, p, p, p, dws - 1, None) == -7
    # the matrix-core probe checks its arguments before it launches anything
    assert lib.bsa_mfma_probe(1, 1, None, None) == -1
    assert lib.bsa_mfma_probe(0, 1, p, None) == -3 and lib.bsa_mfma_probe(1, 0, p, None) == -3
