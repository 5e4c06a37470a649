"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before launching anything, and its host-side group
handling agrees with the oracle's independent implementation."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2511_13732_amd as pcg
import workloads as W
from paper_2511_13732_amd.binding import _GroupsStruct

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pcg.h")

OK, NULL_ARG, BAD_SHAPE, BAD_DTYPE, BAD_STRIDE, BAD_TEMP, WS_SMALL, BAD_CSR, HIP, MISALIGNED = \
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(pcg_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"pcg_group_probs", "pcg_verify", "pcg_verify_workspace_bytes",
            "pcg_groups_validate_host", "pcg_groups_canonicalize_host", "pcg_strerror"} <= set(names)
    L = pcg.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in include/pcg.h but not exported"
    assert "gfx950" in pcg.version()


def test_header_constants_match_binding():
    text = open(HEADER).read()
    for name, val in [("PCG_ERR_NULL_ARG", -1), ("PCG_ERR_BAD_SHAPE", -2), ("PCG_ERR_BAD_DTYPE", -3),
                      ("PCG_ERR_BAD_STRIDE", -4), ("PCG_ERR_BAD_TEMPERATURE", -5),
                      ("PCG_ERR_WORKSPACE_TOO_SMALL", -6), ("PCG_ERR_BAD_CSR", -7),
                      ("PCG_ERR_HIP", -8), ("PCG_ERR_MISALIGNED", -9)]:
        assert re.search(rf"{name}\s*=\s*{val}\b", text)
        assert pcg.strerror(val) != "unknown status"
    assert re.search(r"PCG_F32 = 0, PCG_BF16 = 1", text) and (pcg.F32, pcg.BF16) == (0, 1)
    assert C.sizeof(pcg.Diag) == 32 and C.sizeof(_GroupsStruct) == 40


# Fake device addresses: every call below must fail its host-side checks and return before it
# touches them or launches anything.
P = 0x10000


def call_verify(V=64, G=8, nnz=16, dt=0, B=2, K=2, tbs=None, tps=None, dbs=None, dps=None, tau=1.0,
                ws=P, ws_bytes=1 << 30, tgt=P, dft=P, rp=P, mem=P, mult=P, ptok=P, pgrp=P, al=P,
                otok=P, ogrp=P, groups=True):
    gs = _GroupsStruct(V, G, nnz, rp, mem, mult)
    tps = V if tps is None else tps
    dps = V if dps is None else dps
    tbs = (K + 1) * V if tbs is None else tbs
    dbs = K * V if dbs is None else dbs
    return pcg.lib().pcg_verify(C.byref(gs) if groups else None, tgt, dft, dt, B, K, tbs, tps, dbs,
                                dps, tau, ptok, pgrp, 0, 0, al, otok, ogrp, None, ws, ws_bytes, None)


def test_verify_rejects_bad_arguments_on_the_host():
    assert call_verify(groups=False) == NULL_ARG
    assert call_verify(rp=None) == NULL_ARG
    assert call_verify(tgt=None) == NULL_ARG
    assert call_verify(ogrp=None) == NULL_ARG
    assert call_verify(ws=None) == NULL_ARG
    assert call_verify(V=0) == BAD_SHAPE
    assert call_verify(G=0) == BAD_SHAPE
    assert call_verify(nnz=-1) == BAD_SHAPE
    assert call_verify(K=0) == BAD_SHAPE
    assert call_verify(K=65) == BAD_SHAPE
    assert call_verify(B=-1) == BAD_SHAPE
    assert call_verify(dt=2) == BAD_DTYPE
    assert call_verify(tps=63) == BAD_STRIDE
    assert call_verify(dps=0) == BAD_STRIDE
    assert call_verify(tbs=10) == BAD_STRIDE
    assert call_verify(dbs=-5) == BAD_STRIDE
    for tau in (0.0, -1.0, float("nan"), float("inf")):
        assert call_verify(tau=tau) == BAD_TEMP
    assert call_verify(ws=P + 8) == MISALIGNED
    assert call_verify(tgt=P + 2) == MISALIGNED          # fp32 logits on a 2-byte boundary
    assert call_verify(tgt=P + 1, dt=1) == MISALIGNED
    need = pcg.verify_workspace_bytes(64, 8, 2, 2)
    assert need > 0 and need % 256 == 0
    assert call_verify(ws_bytes=need - 1) == WS_SMALL
    assert call_verify(B=0, tgt=None, ws=None) == OK       # an empty batch is a no-op
    assert pcg.verify_workspace_bytes(0, 8, 2, 2) == 0


def test_group_probs_rejects_bad_arguments_on_the_host():
    L = pcg.lib()
    gs = _GroupsStruct(64, 8, 16, P, P, P)
    f = lambda **k: L.pcg_group_probs(k.get("g", C.byref(gs)), k.get("x", P), k.get("dt", 0),
                                      k.get("rows", 4), k.get("stride", 64), k.get("tau", 1.0),
                                      k.get("out", P), k.get("ws", P), k.get("wsb", 1 << 30), None)
    assert f(g=None) == NULL_ARG and f(x=None) == NULL_ARG and f(out=None) == NULL_ARG
    assert f(rows=-1) == BAD_SHAPE and f(dt=7) == BAD_DTYPE and f(stride=32) == BAD_STRIDE
    assert f(tau=0.0) == BAD_TEMP and f(ws=P + 4) == MISALIGNED
    assert f(wsb=pcg.group_probs_workspace_bytes(64, 4) - 1) == WS_SMALL
    assert f(rows=0, x=None) == OK


def test_workspace_sizes_at_the_headline_shape():
    # V = G = 65 536, B = 64, K = 8: parts + row stats + delta rows + residual rows
    n = pcg.verify_workspace_bytes(65536, 65536, 64, 8)
    assert 2 * 64 * 65536 * 4 < n < 2 * 64 * 65536 * 4 + (1 << 20)


@pytest.mark.parametrize("seed", range(4))
def test_host_group_handling_agrees_with_the_oracle(seed):
    V, G = 200 + 37 * seed, 120
    rp, mem = W.random_groups(V, G, 1, 9, seed=seed, cover=False)
    if seed == 3:                          # with repeated entries inside a group
        mem = mem.copy()
        mem[1] = mem[0]
    a = oracle.canonicalize(V, rp, mem)
    rp2, mem2, mult2 = pcg.groups_canonicalize_host(V, rp, mem)
    np.testing.assert_array_equal(a.row_ptr, rp2)
    np.testing.assert_array_equal(a.members, mem2)
    np.testing.assert_array_equal(a.mult, mult2)
    assert pcg.groups_validate_host(V, rp2, mem2, mult2) == OK
    assert len(rp2) - 1 > G                # some tokens were uncovered and became singletons


def test_host_validation_rejects_what_the_oracle_rejects():
    cases = [
        ([1, 2, 4], [0, 1, 2, 3], [1, 1, 1, 1]),
        ([0, 3, 2], [0, 1, 2, 3], [1, 1, 1, 1]),
        ([0, 2, 4], [0, 1, 2, 4], [1, 1, 1, 1]),
        ([0, 2, 4], [0, 1, 2, -1], [1, 1, 1, 1]),
        ([0, 2, 4], [0, 1, 2, 3], [1, 2, 1, 1]),
        ([0, 2, 3], [0, 1, 2], [1, 1, 1, 0]),
    ]
    for rp, mem, mult in cases:
        assert pcg.groups_validate_host(4, rp, mem, mult) == BAD_CSR
        bad = oracle.Groups(4, 2, np.array(rp, np.int32), np.array(mem, np.int32), np.array(mult, np.int32))
        assert oracle.validate(bad) != 0
    assert pcg.groups_validate_host(4, [0, 2, 4], [0, 1, 2, 3], [1, 1, 1, 1]) == OK
    with pytest.raises(pcg.PcgError):
        pcg.groups_canonicalize_host(4, [0, 2, 4], [0, 1, 2, 9])


def test_profile_calls_are_guarded():
    L = pcg.lib()
    ms = (C.c_float * 8)()
    n = C.c_int32()
    assert L.pcg_profile_end(ms, C.byref(n)) == BAD_SHAPE      # nothing was begun
    assert L.pcg_profile_begin(0) == BAD_SHAPE
    assert [pcg.lib().pcg_stage_name(i).decode() for i in range(6)] == \
        ["row_stats", "accept", "table", "gather", "finalize", ""]
