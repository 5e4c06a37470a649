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
                      ("PCG_ERR_HIP", -8), ("PCG_ERR_MISALIGNED", -9), ("PCG_ERR_CAPACITY", -10),
                      ("PCG_ERR_SCRATCH_TOO_SMALL", -11)]:
        assert re.search(rf"{name}\s*=\s*{val}\b", text)
        assert pcg.strerror(val) != "unknown status"
    assert re.search(r"PCG_F32 = 0, PCG_BF16 = 1", text) and (pcg.F32, pcg.BF16) == (0, 1)
    assert C.sizeof(pcg.Diag) == 32 and C.sizeof(_GroupsStruct) == 88 and C.sizeof(pcg.PreparedInfo) == 72


# Fake device addresses: every call below must fail its host-side checks and return before it
# touches them or launches anything.
P = 0x10000


def call_verify(V=64, G=8, nnz=16, dt=0, B=2, K=2, tbs=None, tps=None, dbs=None, dps=None, tau=1.0,
                ws=P, ws_bytes=1 << 30, tgt=P, dft=P, rp=P, mem=P, mult=P, ptok=P, pgrp=P, al=P,
                otok=P, ogrp=P, groups=True):
    gs = _GroupsStruct(V, G, nnz, rp, mem, mult, None, None, None, None, None, None)
    tps = V if tps is None else tps
    dps = V if dps is None else dps
    tbs = (K + 1) * V if tbs is None else tbs
    dbs = K * V if dbs is None else dbs
    return pcg.lib().pcg_verify(C.byref(gs) if groups else None, tgt, dft, dt, B, K, tbs, tps, dbs,
                                dps, tau, ptok, pgrp, 0, 0, al, otok, ogrp, None, ws, ws_bytes, None)


def test_static_scratch_entry_point_refuses_on_the_host_what_does_not_fit():
    """pcg_verify_static looks at the sizes before anything else: a step that needs more scratch
    than the library's own array holds is refused without a GPU being touched."""
    L = pcg.lib()
    cap = pcg.static_scratch_bytes()
    m = re.search(r"#define PCG_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", open(HEADER).read())
    assert m and cap == int(m.group(1)) << int(m.group(2))
    V = G = 65536
    assert L.pcg_verify_workspace_bytes(V, G, 64, 8) <= cap < L.pcg_verify_workspace_bytes(V, G, 128, 8)
    gs = _GroupsStruct(V, G, 32 * V, P, P, P, None, None, None, None, None, None)
    args = lambda B, K: (C.byref(gs), P, P, 1, B, K, (K + 1) * V, V, K * V, V, 1.0, P, P, 0, 0, P, P, P, None, None)
    assert L.pcg_verify_static(*args(128, 8)) == -11
    assert L.pcg_verify_static(None, *args(1, 1)[1:]) == NULL_ARG
    assert L.pcg_verify_static(*args(4, 0)) == BAD_SHAPE
    assert "scratch" in pcg.strerror(-11)


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
    gs = _GroupsStruct(64, 8, 16, P, P, P, None, None, None, None, None, None)
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
    assert 2 * 64 * 65536 * 4 < n < 2 * 64 * 65536 * 4 + (4 << 20)


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
    assert [pcg.lib().pcg_stage_name(i).decode() for i in range(9)] == \
        ["row_stats", "accept_delta", "weights", "gather", "finalize", "accept_thin", "propose", "event_overhead", ""]


# --------------------------------------------------------------------------- prepared layout

def decode_prepared(blob, info, V, G):
    """Rebuild {group: member list} from the prepared blob, following the documented layout."""
    T, BPC = info.ntiles, info.blocks_per_chunk
    desc = blob[info.off_desc:info.off_desc + info.nchunks * T * BPC * 8].view(np.uint32).reshape(
        info.nchunks, T, BPC, 2)
    perm = blob[info.off_perm:info.off_perm + info.nchunks * BPC * 256 * 2].view(np.uint16).reshape(
        info.nchunks, BPC, 4, 64)
    data = blob[info.off_data:info.off_data + (info.bytes - info.off_data) // 16 * 16].view(
        np.uint32).reshape(-1, 4)                    # 16-byte units
    wts = None
    if info.off_weights:
        assert info.off_weights % 256 == 0 and info.bytes - info.off_weights >= 2 * (info.off_weights - info.off_data)
        wts = blob[info.off_weights:info.off_weights + 2 * (info.off_weights - info.off_data)].view(
            np.float32).reshape(-1, 4, 2)            # [unit, r, low / high slot]
    out = {g: [] for g in range(G)}
    wout = {g: [] for g in range(G)}
    padded = 0
    for c in range(info.nchunks):
        for bl in range(BPC):
            for h in range(T):
                off, steps = int(desc[c, h, bl, 0]), int(desc[c, h, bl, 1])
                if steps == 0:
                    continue
                blk = data[off:off + steps * 64].reshape(steps, 64, 4)          # [step, lane, r]
                slots = np.stack([blk & 0xFFFF, blk >> 16], axis=1).reshape(2 * steps, 64, 4)
                if wts is not None:                                             # -> [entry, lane, r]
                    wblk = wts[off:off + steps * 64].reshape(steps, 64, 4, 2).transpose(0, 3, 1, 2).reshape(
                        2 * steps, 64, 4)
                padded += 2 * steps * 256
                for r in range(4):
                    for lane in range(64):
                        k = int(perm[c, bl, r, lane])
                        col = slots[:, lane, r]
                        real = col[col < info.tile_len]
                        assert (col[col >= info.tile_len] < info.tile_len + 32).all()
                        if k == 0xFFFF:
                            assert len(real) == 0
                            continue
                        assert (real < info.tile_len).all()
                        out[c * info.chunk_groups + k] += (real.astype(np.int64) + h * info.tile_len).tolist()
                        if wts is not None:
                            assert (wblk[:, lane, r][col >= info.tile_len] == 0).all()     # padding weighs nothing
                            wout[c * info.chunk_groups + k] += wblk[:, lane, r][col < info.tile_len].tolist()
    if wts is not None:
        return out, padded, wout
    return out, padded


@pytest.mark.parametrize("V,G,smin,smax,chunk", [
    (300, 200, 1, 9, 0),            # one tile, one chunk
    (50000, 9000, 0, 40, 4096),     # two tiles, three chunks, some empty groups
    (90000, 1500, 20, 20, 0),       # three tiles, fixed group size
])
def test_prepared_layout_holds_exactly_the_membership(V, G, smin, smax, chunk):
    rp, mem = W.random_groups(V, G, max(smin, 1), smax, seed=V % 97, cover=False)
    if smin == 0:                    # make a few groups empty
        keep = np.ones(len(mem), bool)
        for g in (3, 700, G - 1):
            keep[rp[g]:rp[g + 1]] = False
        sizes = np.diff(rp)
        sizes[[3, 700, G - 1]] = 0
        mem = mem[keep]
        rp = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rp, mem, _ = pcg.groups_canonicalize_host(V, rp, mem)
    G2 = len(rp) - 1
    blob, info = pcg.groups_prepare_host(V, rp, mem, chunk)
    assert info.V == V and info.G == G2 and info.bytes == len(blob)
    assert info.ntiles * info.tile_len >= V and info.tile_len <= 40704 - 32
    assert info.ntiles == -(-V // (40704 - 32)) and info.nchunks == -(-G2 // info.chunk_groups)
    got, padded = decode_prepared(blob, info, V, G2)
    for g in range(G2):
        assert sorted(got[g]) == sorted(mem[rp[g]:rp[g + 1]].tolist()), g
    # the order inside a list is the builder's choice (bank scheduling); the multiset is not
    print(f"padding overhead {padded / max(1, len(mem)) - 1:.3f}")
    assert padded < 3.0 * len(mem) + 256 * 2 * info.nchunks * info.blocks_per_chunk * info.ntiles


@pytest.mark.parametrize("V,G,smin,smax,chunk", [(300, 200, 1, 9, 0), (50000, 9000, 1, 40, 4096)])
def test_weighted_prepared_layout_carries_every_entrys_weight(V, G, smin, smax, chunk):
    """Sec. 2.2, Eq. (2) and (4): the weight w_{k,t} sits next to the slot of token t in group k's
    list, whatever order the bank scheduling chose; the slot stream equals the unweighted blob's."""
    rp, mem = W.random_groups(V, G, smin, smax, seed=V % 89, cover=False)
    rp, mem, _ = pcg.groups_canonicalize_host(V, rp, mem)
    G2 = len(rp) - 1
    w = W.random_weights(V, mem, seed=5)
    blob, info = pcg.groups_prepare_host(V, rp, mem, chunk, weights=w)
    plain, pinfo = pcg.groups_prepare_host(V, rp, mem, chunk)
    assert info.off_weights == pinfo.bytes and pinfo.off_weights == 0 and info.bytes == len(blob)
    np.testing.assert_array_equal(blob[:pinfo.bytes], plain)
    got, _, wgot = decode_prepared(blob, info, V, G2)
    for g in range(G2):
        assert sorted(zip(got[g], wgot[g])) == sorted(zip(mem[rp[g]:rp[g + 1]].tolist(), w[rp[g]:rp[g + 1]].tolist())), g
    L = pcg.lib()
    n = L.pcg_groups_prepare_weights_bytes(V, G2, rp.ctypes.data, mem.ctypes.data, chunk)
    assert n == len(blob)
    assert L.pcg_groups_prepare_weights_host(V, G2, rp.ctypes.data, mem.ctypes.data, None, chunk,
                                             blob.ctypes.data, n, C.byref(info)) == NULL_ARG
    assert L.pcg_groups_prepare_weights_host(V, G2, rp.ctypes.data, mem.ctypes.data, w.ctypes.data, chunk,
                                             blob.ctypes.data, n - 1, C.byref(info)) == WS_SMALL


def test_prepare_rejects_bad_arguments():
    rp, mem = np.array([0, 2, 4], np.int32), np.array([0, 1, 2, 3], np.int32)
    L = pcg.lib()
    assert L.pcg_groups_prepare_bytes(4, 2, rp.ctypes.data, mem.ctypes.data, 1024) == 0     # not a multiple of 4096
    assert L.pcg_groups_prepare_bytes(4, 2, rp.ctypes.data, mem.ctypes.data, 32768) == 0
    assert L.pcg_groups_prepare_bytes(4, 2, None, mem.ctypes.data, 0) == 0
    n = L.pcg_groups_prepare_bytes(4, 2, rp.ctypes.data, mem.ctypes.data, 0)
    assert n > 0 and n % 256 == 0
    blob = np.zeros(n, np.uint8)
    info = pcg.PreparedInfo()
    assert L.pcg_groups_prepare_host(4, 2, rp.ctypes.data, mem.ctypes.data, 0, blob.ctypes.data, n - 1,
                                     C.byref(info)) == WS_SMALL
    bad = np.array([0, 1, 2, 7], np.int32)
    assert L.pcg_groups_prepare_host(4, 2, rp.ctypes.data, bad.ctypes.data, 0, blob.ctypes.data, n,
                                     C.byref(info)) == BAD_CSR
    # a descriptor that does not belong to the groups is refused before any launch
    blob, info = pcg.groups_prepare_host(4, rp, mem)
    gs = _GroupsStruct(5, 2, 4, P, P, P, P, C.pointer(info), None, None)
    assert pcg.lib().pcg_group_probs(C.byref(gs), P, 0, 1, 5, 1.0, P, P, 1 << 30, None) == BAD_SHAPE
    gs = _GroupsStruct(4, 2, 4, P, P, P, P, None, None, None, None, None)
    assert pcg.lib().pcg_group_probs(C.byref(gs), P, 0, 1, 4, 1.0, P, P, 1 << 30, None) == NULL_ARG


def test_reverse_index_and_thinning_argument_checks():
    V, G = 257, 150
    rp, mem = W.random_groups(V, G, 1, 9, seed=2, cover=False)
    rp, mem, mult = pcg.groups_canonicalize_host(V, rp, mem)
    tok_ptr, tok_groups = pcg.groups_reverse_host(V, rp, mem)
    a = oracle.Groups(V, len(rp) - 1, rp, mem, mult)
    ref_ptr, ref_groups = oracle.reverse_index(a)
    np.testing.assert_array_equal(tok_ptr, ref_ptr)
    np.testing.assert_array_equal(tok_groups, ref_groups)
    np.testing.assert_array_equal(np.diff(tok_ptr), mult)
    L = pcg.lib()
    gs = _GroupsStruct(64, 8, 16, P, P, P, None, None, None, None, None, None)      # no reverse index
    args = lambda g, **k: L.pcg_verify_thinning(C.byref(g), P, P, 0, 2, 2, 192, 64, 128, 64, 1.0, P, P, 0, 0,
                                                P, P, P, k.get("trials", P), None, P, k.get("wsb", 1 << 30), None)
    assert args(gs) == NULL_ARG
    gs = _GroupsStruct(64, 8, 16, P, P, P, None, None, P, P, None, None)
    assert args(gs, trials=None) == NULL_ARG
    assert args(gs, wsb=pcg.verify_thinning_workspace_bytes(64, 2, 2) - 1) == WS_SMALL
    big = _GroupsStruct(5_000_000, 8, 16, P, P, P, None, None, P, P, None, None)    # more parts than the token draw searches
    assert L.pcg_verify_thinning(C.byref(big), P, P, 0, 1, 1, 0, 5_000_000, 0, 5_000_000, 1.0, P, P, 0, 0,
                                 P, P, P, P, None, P, 1 << 40, None) == BAD_SHAPE


def test_propose_argument_checks():
    L = pcg.lib()
    call = lambda g, **k: L.pcg_propose(C.byref(g), k.get("logits", P), k.get("dt", 0), 2, k.get("K", 2),
                                        k.get("pos0", 0), 128, k.get("ps", 64), k.get("tau", 1.0), 0, 0, P, P,
                                        None, P, k.get("wsb", 1 << 30), None)
    rev = _GroupsStruct(64, 8, 16, P, P, P, None, None, P, P, None, None)
    assert call(_GroupsStruct(64, 8, 16, P, P, P, None, None, None, None, None, None)) == NULL_ARG   # no reverse index
    assert call(rev, logits=None) == NULL_ARG
    assert call(rev, dt=7) == BAD_DTYPE
    assert call(rev, K=0) == BAD_SHAPE
    assert call(rev, pos0=63) == BAD_SHAPE          # pos0 + K beyond PCG_MAX_K
    assert call(rev, ps=10) == BAD_STRIDE
    assert call(rev, tau=0.0) == BAD_TEMP
    assert call(rev, logits=P + 2) == MISALIGNED
    assert call(rev, wsb=pcg.propose_workspace_bytes(64, 2, 2) - 1) == WS_SMALL
    assert pcg.propose_workspace_bytes(0, 1, 1) == 0


def test_weights_host_helpers_match_the_oracle_and_are_checked():
    V, G = 300, 200
    rp, mem = W.random_groups(V, G, 1, 9, seed=4, cover=False)
    rp, mem, mult = pcg.groups_canonicalize_host(V, rp, mem)
    rng = np.random.default_rng(0)
    raw = rng.gamma(0.7, size=len(mem))
    tot = np.zeros(V)
    np.add.at(tot, mem, raw)
    w = (raw / tot[mem]).astype(np.float32)
    assert pcg.groups_validate_weights_host(V, rp, mem, w) == OK
    for j, val in ((3, -0.1), (5, np.nan), (7, 1.5)):
        bad = w.copy()
        bad[j] = val
        assert pcg.groups_validate_weights_host(V, rp, mem, bad) == BAD_CSR
    assert pcg.groups_validate_weights_host(V, rp, mem, w * np.float32(0.99)) == BAD_CSR
    og = oracle.with_weights(oracle.Groups(V, len(rp) - 1, rp, mem, mult), w)
    np.testing.assert_array_equal(pcg.groups_reverse_weights_host(V, rp, mem, w), og.tok_weights)
    # weights need a prepared form built with them; thinning and proposals need tok_weights
    L = pcg.lib()
    info = pcg.PreparedInfo()
    both = _GroupsStruct(64, 8, 16, P, P, P, P, C.pointer(info), None, None, P, None)
    assert L.pcg_group_probs(C.byref(both), P, 0, 1, 64, 1.0, P, P, 1 << 30, None) == BAD_SHAPE
    half = _GroupsStruct(64, 8, 16, P, P, P, None, None, P, P, P, None)
    assert L.pcg_propose(C.byref(half), P, 0, 2, 2, 0, 128, 64, 1.0, 0, 0, P, P, None, P, 1 << 30, None) == NULL_ARG
    assert L.pcg_verify_thinning(C.byref(half), P, P, 0, 2, 2, 192, 64, 128, 64, 1.0, P, P, 0, 0,
                                 P, P, P, P, None, P, 1 << 30, None) == NULL_ARG


def test_asg_argument_checks():
    L = pcg.lib()
    g, n, m = C.c_int32(), C.c_int64(), C.c_int32()
    build = lambda **k: L.pcg_asg_build(k.get("unit", P), k.get("V", 256), k.get("d", 128), k.get("theta", 0.4),
                                        k.get("cap", 64), P, P, k.get("room", 1000), P, None, C.byref(g),
                                        C.byref(n), C.byref(m), k.get("ws", P), k.get("wsb", 1 << 30), None)
    assert build(unit=None) == NULL_ARG
    assert build(d=100) == BAD_SHAPE                  # d must be a multiple of 64
    assert build(cap=0) == BAD_SHAPE and build(cap=5000) == BAD_SHAPE
    assert build(theta=float("nan")) == BAD_SHAPE
    assert build(V=1 << 22, d=1024) == BAD_SHAPE      # V * d beyond 2^31
    assert build(unit=P + 2) == MISALIGNED
    assert build(wsb=pcg.lib().pcg_asg_build_workspace_bytes(256, 64) - 1) == WS_SMALL
    assert L.pcg_asg_normalize(None, 4, 4, P, None) == NULL_ARG
    assert L.pcg_asg_normalize(P, 0, 4, P, None) == BAD_SHAPE
    assert pcg.lib().pcg_asg_build_workspace_bytes(256, 5000) == 0
    exact = lambda **k: L.pcg_asg_build_exact(k.get("emb", P), k.get("V", 256), k.get("d", 128), k.get("theta", 0.4),
                                              k.get("cap", 64), P, P, k.get("room", 1000), P, None, C.byref(g),
                                              C.byref(n), C.byref(m), k.get("ws", P), k.get("wsb", 1 << 30), None)
    assert exact(emb=None) == NULL_ARG
    assert exact(d=96) == BAD_SHAPE and exact(cap=0) == BAD_SHAPE and exact(theta=float("inf")) == BAD_SHAPE
    assert exact(emb=P + 4) == MISALIGNED and exact(ws=P + 64) == MISALIGNED
    need = L.pcg_asg_build_exact_workspace_bytes(256, 128, 64)
    assert need >= L.pcg_asg_build_workspace_bytes(256, 64) + 256 * 128 * 2 + 256 * 8      # unit vectors, norms
    assert exact(wsb=need - 1) == WS_SMALL
    assert L.pcg_asg_build_exact_workspace_bytes(1 << 22, 1024, 64) == 0
