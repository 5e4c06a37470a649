"""ctypes front end of the CPU oracle (``pcg_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the CPU-baseline leg
of the benchmark call this; the product path never does and shares no code
with it.  Arrays are numpy, on the host.  Logits are ``float32`` arrays, or
``uint16`` arrays holding bfloat16 bit patterns (``bf16_bits`` converts a torch
bf16 tensor).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcg_oracle.c")
_LIB = os.path.join(_HERE, "libpcg_oracle.so")
_LIB_SAN = os.path.join(_HERE, "libpcg_oracle_san.so")

F32, BF16 = 0, 1
NEAR_TIE = 1e-6


def _sanitize() -> bool:
    return os.environ.get("PCG_SANITIZE", "") not in ("", "0")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP only for the batch loop).  With
    PCG_SANITIZE=1: with ROCm's clang, AddressSanitizer and UndefinedBehaviorSanitizer on, into a
    library of its own (the same compiler and sanitizer runtime as the sanitized libpcg, so that
    one preloaded runtime serves both)."""
    lib = _LIB_SAN if _sanitize() else _LIB
    stale = (not os.path.exists(lib)
             or os.path.getmtime(lib) < max(os.path.getmtime(_SRC),
                                            os.path.getmtime(os.path.join(_HERE, "pcg_oracle.h"))))
    if force or stale:
        if _sanitize():
            subprocess.check_call(["/opt/rocm/llvm/bin/clang", "-O1", "-g", "-std=c11", "-Wall", "-Wextra",
                                   "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
                                   "-fno-sanitize-recover=undefined", "-shared-libsan",
                                   "-fno-omit-frame-pointer", _SRC, "-o", lib, "-lm"])
        else:
            subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fPIC",
                                   "-shared", _SRC, "-o", lib, "-lm"])
    return lib


class _Trace(C.Structure):
    _fields_ = [("T_prop", C.c_void_p), ("D_prop", C.c_void_p), ("near_acc", C.c_void_p),
                ("near_grp", C.c_void_p), ("near_tok", C.c_void_p), ("flags", C.c_void_p),
                ("res_S", C.c_void_p), ("res_lo", C.c_void_p), ("res_hi", C.c_void_p),
                ("R_norm", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.pcg_ref_philox4x32_10.restype = None
        _lib.pcg_ref_uniforms.restype = None
        _lib.pcg_ref_uniforms.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32,
                                          C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.pcg_ref_trial_uniforms.restype = None
        _lib.pcg_ref_trial_uniforms.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32,
                                                C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p]
        for name in ("pcg_ref_softmax_row", "pcg_ref_count_mult", "pcg_ref_canonicalize",
                     "pcg_ref_validate", "pcg_ref_group_probs", "pcg_ref_verify_u",
                     "pcg_ref_verify", "pcg_ref_reverse_index", "pcg_ref_thin_trial",
                     "pcg_ref_verify_thinning"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def bf16_bits(t) -> np.ndarray:
    """torch.bfloat16 CPU tensor -> uint16 numpy array of its bit patterns."""
    import torch
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _logits(a) -> tuple[np.ndarray, int]:
    """Accept float32 / uint16(bf16 bits) numpy arrays or torch CPU tensors."""
    if not isinstance(a, np.ndarray):
        import torch
        if isinstance(a, torch.Tensor):
            a = bf16_bits(a) if a.dtype == torch.bfloat16 else a.detach().cpu().numpy()
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return np.ascontiguousarray(a), BF16
    if a.dtype == np.float32:
        return np.ascontiguousarray(a), F32
    raise TypeError(f"logits must be float32 or uint16 (bf16 bits), got {a.dtype}")


class OracleError(RuntimeError):
    pass


def _check(rc: int, what: str):
    if rc != 0:
        raise OracleError(f"{what} failed with code {rc}")


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().pcg_ref_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniforms(seed: int, offset: int, b: int, i: int) -> tuple[float, float, float]:
    ua, ug, ut = C.c_double(), C.c_double(), C.c_double()
    lib().pcg_ref_uniforms(C.c_uint64(seed), C.c_uint64(offset), C.c_uint32(b), C.c_uint32(i),
                           C.byref(ua), C.byref(ug), C.byref(ut))
    return ua.value, ug.value, ut.value


def softmax_row(logits, temperature: float = 1.0) -> np.ndarray:
    a, dt = _logits(logits)
    assert a.ndim == 1
    out = np.empty(a.shape[0], dtype=np.float64)
    _check(lib().pcg_ref_softmax_row(_p(a), C.c_int(dt), C.c_int64(a.shape[0]),
                                     C.c_double(temperature), _p(out)), "softmax_row")
    return out


@dataclass
class Groups:
    """Canonical group membership: CSR group -> tokens plus per-token multiplicity."""
    V: int
    G: int
    row_ptr: np.ndarray   # int32 [G+1]
    members: np.ndarray   # int32 [nnz]
    mult: np.ndarray      # int32 [V]
    weights: Optional[np.ndarray] = None       # float32 [nnz] general weights (Eq. 2); None = equal split
    tok_weights: Optional[np.ndarray] = None   # float32 [nnz] the same in reverse-index order

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


class _Weights(C.Structure):
    _fields_ = [("weights", C.c_void_p), ("tok_weights", C.c_void_p)]


def _wt(g: "Groups"):
    """Pointer to the weights argument of the _w entry points (NULL = equal split)."""
    if g.weights is None:
        return None
    return C.byref(_Weights(g.weights.ctypes.data,
                            None if g.tok_weights is None else g.tok_weights.ctypes.data))


def validate_weights(g: "Groups", weights, tol: float = 1e-6) -> int:
    w = np.ascontiguousarray(weights, dtype=np.float32)
    return lib().pcg_ref_validate_weights(C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members),
                                          _p(w), C.c_double(tol))


def with_weights(g: "Groups", weights, tol: float = 1e-6) -> "Groups":
    """The same membership with general per-entry weights (validated), and their reverse-index
    order for thinning and proposals."""
    w = np.ascontiguousarray(weights, dtype=np.float32)
    assert w.shape == (g.nnz,)
    _check(validate_weights(g, w, tol), "validate_weights")
    tw = np.empty(max(1, g.nnz), dtype=np.float32)
    _check(lib().pcg_ref_reverse_weights(C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members),
                                         _p(w), _p(tw)), "reverse_weights")
    return Groups(g.V, g.G, g.row_ptr, g.members, g.mult, w, tw[:g.nnz])


def count_mult(V: int, row_ptr, members) -> np.ndarray:
    row_ptr, members = _i32(row_ptr), _i32(members)
    mult = np.empty(V, dtype=np.int32)
    _check(lib().pcg_ref_count_mult(C.c_int32(V), C.c_int32(len(row_ptr) - 1), _p(row_ptr),
                                    _p(members), _p(mult)), "count_mult")
    return mult


def canonicalize(V: int, row_ptr, members) -> Groups:
    """Append a singleton group for every token that is in no group; fill mult."""
    row_ptr, members = _i32(row_ptr), _i32(members)
    G = len(row_ptr) - 1
    # the C routine learns the number of entries from row_ptr[G]; only here is the array's length known
    if G < 0 or not 0 <= int(row_ptr[-1]) <= len(members):
        raise OracleError("canonicalize: row_ptr[G] does not fit the members array")
    oG, onnz = C.c_int32(), C.c_int64()
    _check(lib().pcg_ref_canonicalize(C.c_int32(V), C.c_int32(G), _p(row_ptr), _p(members),
                                      C.byref(oG), C.byref(onnz), None, None, None),
           "canonicalize(size)")
    rp = np.empty(oG.value + 1, dtype=np.int32)
    mem = np.empty(max(onnz.value, 1), dtype=np.int32)
    mult = np.empty(V, dtype=np.int32)
    _check(lib().pcg_ref_canonicalize(C.c_int32(V), C.c_int32(G), _p(row_ptr), _p(members),
                                      C.byref(oG), C.byref(onnz), _p(rp), _p(mem), _p(mult)),
           "canonicalize")
    return Groups(V, oG.value, rp, mem[:onnz.value], mult)


def validate(g: Groups) -> int:
    return lib().pcg_ref_validate(C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members),
                                  _p(g.mult))


def group_probs(g: Groups, logits, temperature: float = 1.0) -> np.ndarray:
    """[rows, V] logits -> [rows, G] float64 group probabilities (Eq. 5)."""
    a, dt = _logits(logits)
    assert a.ndim == 2 and a.shape[1] == g.V
    out = np.empty((a.shape[0], g.G), dtype=np.float64)
    _check(lib().pcg_ref_group_probs_w(C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr),
                                     _p(g.members), _p(g.mult), _wt(g), _p(a), C.c_int(dt),
                                     C.c_int64(a.shape[0]), C.c_int64(a.shape[1]),
                                     C.c_double(temperature), _p(out)), "group_probs")
    return out


@dataclass
class VerifyResult:
    accept_len: np.ndarray     # int32 [B]
    out_tokens: np.ndarray     # int32 [B, K+1], unused tail = -1
    out_groups: np.ndarray     # int32 [B, K+1]
    T_prop: np.ndarray         # float64 [B, K]  (NaN where not evaluated)
    D_prop: np.ndarray
    near_acc: np.ndarray       # uint8 [B, K]
    near_grp: np.ndarray       # uint8 [B]
    near_tok: np.ndarray       # uint8 [B]
    flags: np.ndarray          # uint8 [B]
    res_S: np.ndarray          # float64 [B]
    res_lo: np.ndarray
    res_hi: np.ndarray
    R_norm: Optional[np.ndarray]   # float64 [B, G] when requested
    threads: int = 1


def _strides(a: np.ndarray, batch_stride, pos_stride):
    """Element strides of a [B, P, V] array; explicit values override (0 = shared rows)."""
    bs = a.shape[1] * a.shape[2] if batch_stride is None else batch_stride
    ps = a.shape[2] if pos_stride is None else pos_stride
    return C.c_int64(bs), C.c_int64(ps)


def verify(g: Groups, target_logits, draft_logits, prop_tokens, prop_groups, *,
           temperature: float = 1.0, seed: int = 0, offset: int = 0,
           uniforms_explicit: Optional[tuple[np.ndarray, np.ndarray, np.ndarray]] = None,
           B: Optional[int] = None, tgt_batch_stride=None, dft_batch_stride=None,
           want_R: bool = False, nthreads: int = 1) -> VerifyResult:
    """One speculative step (Algorithm 1) for B sequences.

    target_logits [Bt, K+1, V], draft_logits [Bd, >=K, V].  ``B`` together with
    a batch stride of 0 lets many sequences share one set of rows.  With
    ``uniforms_explicit = (u_acc [B,K], u_grp [B,K+1], u_tok [B,K+1])`` the
    draws are taken from the arrays instead of Philox(seed, offset).
    """
    tgt, dt = _logits(target_logits)
    dft, dt2 = _logits(draft_logits)
    assert dt == dt2 and tgt.ndim == 3 and dft.ndim == 3
    K = tgt.shape[1] - 1
    assert dft.shape[1] >= K and tgt.shape[2] == g.V and dft.shape[2] == g.V
    if B is None:
        B = tgt.shape[0]
    ptok = _i32(prop_tokens).reshape(B, K)
    pgrp = _i32(prop_groups).reshape(B, K)
    tbs, tps = _strides(tgt, tgt_batch_stride, None)
    dbs, dps = _strides(dft, dft_batch_stride, None)

    al = np.empty(B, dtype=np.int32)
    otok = np.empty((B, K + 1), dtype=np.int32)
    ogrp = np.empty((B, K + 1), dtype=np.int32)
    res = VerifyResult(al, otok, ogrp,
                       np.empty((B, K)), np.empty((B, K)), np.zeros((B, K), np.uint8),
                       np.zeros(B, np.uint8), np.zeros(B, np.uint8), np.zeros(B, np.uint8),
                       np.empty(B), np.empty(B), np.empty(B),
                       np.empty((B, g.G)) if want_R else None)
    tr = _Trace(res.T_prop.ctypes.data, res.D_prop.ctypes.data, res.near_acc.ctypes.data,
                res.near_grp.ctypes.data, res.near_tok.ctypes.data, res.flags.ctypes.data,
                res.res_S.ctypes.data, res.res_lo.ctypes.data, res.res_hi.ctypes.data,
                res.R_norm.ctypes.data if want_R else None)
    common = [C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members), _p(g.mult), _wt(g),
              _p(tgt), _p(dft), C.c_int(dt), C.c_int32(B), C.c_int32(K), tbs, tps, dbs, dps,
              C.c_double(temperature), _p(ptok), _p(pgrp)]
    outs = [_p(al), _p(otok), _p(ogrp), C.byref(tr)]
    if uniforms_explicit is not None:
        ua, ug, ut = (np.ascontiguousarray(x, dtype=np.float64) for x in uniforms_explicit)
        assert ua.shape == (B, K) and ug.shape == (B, K + 1) and ut.shape == (B, K + 1)
        rc = lib().pcg_ref_verify_u_w(*common, _p(ua), _p(ug), _p(ut), *outs, C.c_int32(nthreads))
    else:
        used = C.c_int32(1)
        rc = lib().pcg_ref_verify_w(*common, C.c_uint64(seed), C.c_uint64(offset), *outs,
                                  C.c_int32(nthreads), C.byref(used))
        res.threads = used.value
    _check(rc, "verify")
    return res


# --------------------------------------------------------------------------- thinning (Eq. 9)

class _Trial(C.Structure):
    _fields_ = [("y", C.c_int32), ("group", C.c_int32), ("accepted", C.c_int32),
                ("token", C.c_int32), ("T", C.c_double), ("D", C.c_double), ("near", C.c_uint8)]


def reverse_index(g: Groups) -> tuple[np.ndarray, np.ndarray]:
    """token -> groups holding it: (tok_ptr [V+1], tok_groups [nnz])."""
    tok_ptr = np.empty(g.V + 1, dtype=np.int32)
    tok_groups = np.empty(max(1, g.nnz), dtype=np.int32)
    _check(lib().pcg_ref_reverse_index(C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members),
                                       _p(tok_ptr), _p(tok_groups)), "reverse_index")
    return tok_ptr, tok_groups[:g.nnz]


def trial_uniforms(seed: int, offset: int, b: int, i: int, trial: int):
    """(u_y, k24, u_a, u_tok) of one thinning trial."""
    uy, ua, ut, k = C.c_double(), C.c_double(), C.c_double(), C.c_uint32()
    lib().pcg_ref_trial_uniforms(C.c_uint64(seed), C.c_uint64(offset), C.c_uint32(b), C.c_uint32(i),
                                 C.c_uint32(trial), C.byref(uy), C.byref(k), C.byref(ua), C.byref(ut))
    return uy.value, k.value, ua.value, ut.value


def thin_trial(g: Groups, rev, q: np.ndarray, p: Optional[np.ndarray], u_y: float, k24: int,
               u_a: float, u_tok: float) -> _Trial:
    """One thinning trial on token distributions q (target) and p (draft; None = bonus row)."""
    tok_ptr, tok_groups = rev
    q = np.ascontiguousarray(q, dtype=np.float64)
    pp = None if p is None else np.ascontiguousarray(p, dtype=np.float64)
    out = _Trial()
    _check(lib().pcg_ref_thin_trial_w(C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members),
                                    _p(g.mult), _wt(g), _p(tok_ptr), _p(tok_groups), _p(q), _p(pp),
                                    C.c_double(u_y), C.c_uint32(k24), C.c_double(u_a),
                                    C.c_double(u_tok), C.byref(out)), "thin_trial")
    return out


@dataclass
class ThinningResult:
    accept_len: np.ndarray     # int32 [B]
    out_tokens: np.ndarray     # int32 [B, K+1]
    out_groups: np.ndarray     # int32 [B, K+1]
    trials: np.ndarray         # int32 [B]  thinning trials run (0 on the bonus position)
    flags: np.ndarray          # uint8 [B]  bit0: a near-tie on the emitted path; bit1: max_trials hit
    near_acc: np.ndarray       # uint8 [B, K]


def verify_thinning(g: Groups, rev, target_logits, draft_logits, prop_tokens, prop_groups, *,
                    temperature: float = 1.0, seed: int = 0, offset: int = 0,
                    B: Optional[int] = None, tgt_batch_stride=None, dft_batch_stride=None,
                    max_trials: int = 1 << 16, nthreads: int = 1) -> ThinningResult:
    """One speculative step with the reject branch drawn by thinning."""
    tgt, dt = _logits(target_logits)
    dft, dt2 = _logits(draft_logits)
    assert dt == dt2 and tgt.ndim == 3 and dft.ndim == 3
    K = tgt.shape[1] - 1
    if B is None:
        B = tgt.shape[0]
    tok_ptr, tok_groups = rev
    ptok = _i32(prop_tokens).reshape(B, K)
    pgrp = _i32(prop_groups).reshape(B, K)
    tbs, tps = _strides(tgt, tgt_batch_stride, None)
    dbs, dps = _strides(dft, dft_batch_stride, None)
    res = ThinningResult(np.empty(B, np.int32), np.empty((B, K + 1), np.int32),
                         np.empty((B, K + 1), np.int32), np.empty(B, np.int32),
                         np.zeros(B, np.uint8), np.zeros((B, K), np.uint8))
    _check(lib().pcg_ref_verify_thinning_w(
        C.c_int32(g.V), C.c_int32(g.G), _p(g.row_ptr), _p(g.members), _p(g.mult), _wt(g), _p(tok_ptr),
        _p(tok_groups), _p(tgt), _p(dft), C.c_int(dt), C.c_int32(B), C.c_int32(K), tbs, tps, dbs,
        dps, C.c_double(temperature), _p(ptok), _p(pgrp), C.c_uint64(seed), C.c_uint64(offset),
        _p(res.accept_len), _p(res.out_tokens), _p(res.out_groups), _p(res.trials), _p(res.flags),
        _p(res.near_acc), C.c_int32(max_trials), C.c_int32(nthreads)), "verify_thinning")
    return res


# --------------------------------------------------------------------------- proposal coupling (Eq. 6)

def propose_uniforms(seed: int, offset: int, b: int, i: int) -> tuple[float, int]:
    ux, k = C.c_double(), C.c_uint32()
    lib().pcg_ref_propose_uniforms(C.c_uint64(seed), C.c_uint64(offset), C.c_uint32(b), C.c_uint32(i),
                                   C.byref(ux), C.byref(k))
    return ux.value, k.value


@dataclass
class Proposals:
    tokens: np.ndarray     # int32 [B, K]
    groups: np.ndarray     # int32 [B, K]
    near: np.ndarray       # uint8 [B, K]  token draw within 1e-6 of an inner bin edge


def propose(g: Groups, rev, draft_logits, *, temperature: float = 1.0, seed: int = 0,
            offset: int = 0, pos0: int = 0, B: Optional[int] = None, dft_batch_stride=None,
            u_x=None, k24=None, nthreads: int = 1) -> Proposals:
    """Draft-side proposals: x ~ p_i, then one of the groups holding x by the weights (Eq. 6).
    With u_x and k24 ([B, K]) the draws are explicit, else Philox(seed, offset)."""
    dft, dt = _logits(draft_logits)
    assert dft.ndim == 3
    K = dft.shape[1]
    if B is None:
        B = dft.shape[0]
    tok_ptr, tok_groups = rev
    dbs, dps = _strides(dft, dft_batch_stride, None)
    res = Proposals(np.empty((B, K), np.int32), np.empty((B, K), np.int32), np.zeros((B, K), np.uint8))
    common = (C.c_int32(g.V), C.c_int32(g.G), _p(g.mult), _wt(g), _p(tok_ptr), _p(tok_groups), _p(dft),
              C.c_int(dt), C.c_int32(B), C.c_int32(K))
    if u_x is not None:
        ux = np.ascontiguousarray(u_x, dtype=np.float64).reshape(B, K)
        kk = np.ascontiguousarray(k24, dtype=np.uint32).reshape(B, K)
        _check(lib().pcg_ref_propose_u_w(*common, dbs, dps, C.c_double(temperature), _p(ux), _p(kk),
                                       _p(res.tokens), _p(res.groups), _p(res.near)), "propose_u")
    else:
        _check(lib().pcg_ref_propose_w(*common, C.c_int32(pos0), dbs, dps, C.c_double(temperature),
                                     C.c_uint64(seed), C.c_uint64(offset), _p(res.tokens),
                                     _p(res.groups), _p(res.near), C.c_int32(nthreads)), "propose")
    return res


# --------------------------------------------------------------------------- similarity groups (Eq. 1)

def asg_normalize(emb) -> np.ndarray:
    """float32 [V, d] embeddings -> unit vectors as bf16 bit patterns (uint16 [V, d])."""
    e = np.ascontiguousarray(emb, dtype=np.float32)
    out = np.empty(e.shape, dtype=np.uint16)
    _check(lib().pcg_ref_asg_normalize(_p(e), C.c_int32(e.shape[0]), C.c_int32(e.shape[1]), _p(out)),
           "asg_normalize")
    return out


def asg_similarity(unit, a: int, b: int) -> float:
    u = np.ascontiguousarray(unit, dtype=np.uint16)
    f = lib().pcg_ref_asg_similarity
    f.restype = C.c_double
    return f(_p(u), C.c_int32(u.shape[1]), C.c_int32(a), C.c_int32(b))


def asg_row(unit, theta: float, t: int) -> tuple[np.ndarray, int]:
    """(members of G(t) ascending, number of near-tie pairs of the row)."""
    u = np.ascontiguousarray(unit, dtype=np.uint16)
    V, d = u.shape
    buf = np.empty(V, dtype=np.int32)
    n, near = C.c_int32(), C.c_int32()
    _check(lib().pcg_ref_asg_row(_p(u), C.c_int32(V), C.c_int32(d), C.c_float(theta), C.c_int32(t),
                                 _p(buf), C.byref(n), C.byref(near)), "asg_row")
    return buf[:n.value].copy(), near.value


def asg_cosine(emb, a: int, b: int) -> float:
    """Cosine of rows a and b of the float32 embeddings, in double (Eq. 1's similarity)."""
    e = np.ascontiguousarray(emb, dtype=np.float32)
    f = lib().pcg_ref_asg_cosine
    f.restype = C.c_double
    return f(_p(e), C.c_int32(e.shape[1]), C.c_int32(a), C.c_int32(b))


def asg_row_exact(emb, theta: float, t: int) -> tuple[np.ndarray, np.ndarray]:
    """(members of G(t) ascending, the row's cosines float64 [V]) by Eq. (1) on the embeddings
    themselves: double throughout, strict ``> theta``, no rounded unit vectors."""
    e = np.ascontiguousarray(emb, dtype=np.float32)
    V, d = e.shape
    buf = np.empty(V, dtype=np.int32)
    cos = np.empty(V, dtype=np.float64)
    n = C.c_int32()
    _check(lib().pcg_ref_asg_row_exact(_p(e), C.c_int32(V), C.c_int32(d), C.c_double(theta),
                                       C.c_int32(t), _p(buf), C.byref(n), _p(cos)), "asg_row_exact")
    return buf[:n.value].copy(), cos


@dataclass
class AsgResult:
    groups: Groups
    seed_of: np.ndarray      # int32 [G] the token whose similarity group each kept row is
    near_rows: np.ndarray    # uint8 [V] rows with a pair within 1e-5 of the threshold


def _asg_build(call, V: int) -> AsgResult:
    cap = 64 * V
    while True:
        rp = np.empty(V + 1, np.int32)
        mem = np.empty(max(1, cap), np.int32)
        mult = np.empty(V, np.int32)
        seed = np.empty(V, np.int32)
        near = np.zeros(V, np.uint8)
        G, nnz = C.c_int32(), C.c_int64()
        rc = call(G, nnz, rp, mem, cap, mult, seed, near)
        if rc == -4 and nnz.value > cap:
            cap = nnz.value
            continue
        _check(rc, "asg_build")
        return AsgResult(Groups(V, G.value, rp[:G.value + 1].copy(), mem[:nnz.value].copy(), mult),
                         seed[:G.value].copy(), near)


def asg_build(unit, theta: float, nthreads: int = 1) -> AsgResult:
    """Distinct similarity groups of all tokens from the bf16 unit vectors, as canonical Groups."""
    u = np.ascontiguousarray(unit, dtype=np.uint16)
    V, d = u.shape

    def call(G, nnz, rp, mem, cap, mult, seed, near):
        return lib().pcg_ref_asg_build(_p(u), C.c_int32(V), C.c_int32(d), C.c_float(theta), C.byref(G),
                                       C.byref(nnz), _p(rp), _p(mem), C.c_int64(cap), _p(mult), _p(seed),
                                       _p(near), C.c_int32(nthreads))
    return _asg_build(call, V)


def asg_build_exact(emb, theta: float, nthreads: int = 1) -> AsgResult:
    """Distinct similarity groups of all tokens by Eq. (1) on the float32 embeddings themselves
    (double throughout, strict ``> theta``); near_rows marks rows with a cosine within 1e-12 of
    theta."""
    e = np.ascontiguousarray(emb, dtype=np.float32)
    V, d = e.shape

    def call(G, nnz, rp, mem, cap, mult, seed, near):
        return lib().pcg_ref_asg_build_exact(_p(e), C.c_int32(V), C.c_int32(d), C.c_double(theta),
                                             C.byref(G), C.byref(nnz), _p(rp), _p(mem), C.c_int64(cap),
                                             _p(mult), _p(seed), _p(near), C.c_int32(nthreads))
    return _asg_build(call, V)
