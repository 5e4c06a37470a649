"""ctypes binding of libpcg.so: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

F32, BF16 = 0, 1
MAX_STAGES = 8
_HERE = os.path.dirname(os.path.abspath(__file__))


class PcgError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} (status {status})")


def lib_path() -> str:
    """libpcg.so, or with PCG_SANITIZE=1 its host-sanitized build libpcg_san.so (CPU test runs)."""
    name = "libpcg_san.so" if os.environ.get("PCG_SANITIZE", "") not in ("", "0") else "libpcg.so"
    return os.path.join(_HERE, name)


class PreparedInfo(C.Structure):
    """Mirror of pcg_prepared (host descriptor of the prepared membership blob)."""
    _fields_ = [("V", C.c_int32), ("G", C.c_int32), ("ntiles", C.c_int32), ("tile_len", C.c_int32),
                ("chunk_groups", C.c_int32), ("nchunks", C.c_int32),
                ("blocks_per_chunk", C.c_int32), ("reserved", C.c_int32),
                ("off_desc", C.c_int64), ("off_perm", C.c_int64), ("off_data", C.c_int64),
                ("off_weights", C.c_int64), ("bytes", C.c_int64)]


class _GroupsStruct(C.Structure):
    _fields_ = [("V", C.c_int32), ("G", C.c_int32), ("nnz", C.c_int64),
                ("row_ptr", C.c_void_p), ("members", C.c_void_p), ("mult", C.c_void_p),
                ("prepared", C.c_void_p), ("prepared_info", C.POINTER(PreparedInfo)),
                ("tok_ptr", C.c_void_p), ("tok_groups", C.c_void_p),
                ("weights", C.c_void_p), ("tok_weights", C.c_void_p)]


class Diag(C.Structure):
    """Mirror of pcg_diag (eight uint32 counters)."""
    _fields_ = [(n, C.c_uint32) for n in
                ("near_accept", "near_group", "near_token", "zero_draft_mass",
                 "residual_fallback", "bad_proposal", "accepted_total", "sequences")]
    NAMES = [n for n, _ in _fields_]


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  There is no fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build it first (python -m paper_2511_13732_amd.build, or "
                "__graft_entry__.build()); this package has no CPU or PyTorch fallback")
        L = C.CDLL(path)
        L.pcg_group_probs_workspace_bytes.restype = C.c_size_t
        L.pcg_group_probs_workspace_bytes.argtypes = [C.c_int32, C.c_int64]
        L.pcg_verify_workspace_bytes.restype = C.c_size_t
        L.pcg_verify_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.pcg_group_probs.restype = C.c_int
        L.pcg_group_probs.argtypes = [C.POINTER(_GroupsStruct), C.c_void_p, C.c_int, C.c_int64,
                                      C.c_int64, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                      C.c_void_p]
        L.pcg_verify.restype = C.c_int
        L.pcg_verify.argtypes = [C.POINTER(_GroupsStruct), C.c_void_p, C.c_void_p, C.c_int,
                                 C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                 C.c_float, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
        L.pcg_verify_static.restype = C.c_int
        L.pcg_verify_static.argtypes = L.pcg_verify.argtypes[:19] + [C.c_void_p]
        L.pcg_static_scratch_bytes.restype = C.c_size_t
        L.pcg_static_scratch_bytes.argtypes = []
        L.pcg_verify_thinning_workspace_bytes.restype = C.c_size_t
        L.pcg_verify_thinning_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.pcg_verify_thinning.restype = C.c_int
        L.pcg_verify_thinning.argtypes = [C.POINTER(_GroupsStruct), C.c_void_p, C.c_void_p, C.c_int,
                                          C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int64,
                                          C.c_int64, C.c_float, C.c_void_p, C.c_void_p, C.c_uint64,
                                          C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pcg_propose_workspace_bytes.restype = C.c_size_t
        L.pcg_propose_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.pcg_propose.restype = C.c_int
        L.pcg_propose.argtypes = [C.POINTER(_GroupsStruct), C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                  C.c_int32, C.c_int64, C.c_int64, C.c_float, C.c_uint64, C.c_uint64,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                  C.c_void_p]
        L.pcg_groups_reverse_host.restype = C.c_int
        L.pcg_groups_reverse_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]
        L.pcg_asg_normalize.restype = C.c_int
        L.pcg_asg_normalize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.pcg_asg_build_workspace_bytes.restype = C.c_size_t
        L.pcg_asg_build_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
        L.pcg_asg_build.restype = C.c_int
        L.pcg_asg_build.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_void_p,
                                    C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                    C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_int32),
                                    C.c_void_p, C.c_size_t, C.c_void_p]
        L.pcg_asg_build_exact_workspace_bytes.restype = C.c_size_t
        L.pcg_asg_build_exact_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.pcg_asg_build_exact.restype = C.c_int
        L.pcg_asg_build_exact.argtypes = L.pcg_asg_build.argtypes
        L.pcg_groups_validate_weights_host.restype = C.c_int
        L.pcg_groups_validate_weights_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                                       C.c_void_p, C.c_double]
        L.pcg_groups_reverse_weights_host.restype = C.c_int
        L.pcg_groups_reverse_weights_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                                      C.c_void_p, C.c_void_p]
        L.pcg_groups_validate_host.restype = C.c_int
        L.pcg_groups_validate_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                               C.c_void_p]
        L.pcg_groups_canonicalize_host.restype = C.c_int
        L.pcg_groups_canonicalize_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                                   C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                                   C.c_void_p, C.c_void_p, C.c_void_p]
        L.pcg_groups_prepare_bytes.restype = C.c_size_t
        L.pcg_groups_prepare_bytes.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]
        L.pcg_groups_prepare_host.restype = C.c_int
        L.pcg_groups_prepare_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                              C.c_void_p, C.c_size_t, C.POINTER(PreparedInfo)]
        L.pcg_groups_prepare_weights_bytes.restype = C.c_size_t
        L.pcg_groups_prepare_weights_bytes.argtypes = L.pcg_groups_prepare_bytes.argtypes
        L.pcg_groups_prepare_weights_host.restype = C.c_int
        L.pcg_groups_prepare_weights_host.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                                      C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t,
                                                      C.POINTER(PreparedInfo)]
        L.pcg_profile_begin.restype = C.c_int
        L.pcg_profile_begin.argtypes = [C.c_int32]
        L.pcg_profile_end.restype = C.c_int
        L.pcg_profile_end.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        L.pcg_stage_name.restype = C.c_char_p
        L.pcg_stage_name.argtypes = [C.c_int32]
        L.pcg_strerror.restype = C.c_char_p
        L.pcg_strerror.argtypes = [C.c_int]
        L.pcg_last_hip_error.restype = C.c_int
        L.pcg_version.restype = C.c_char_p
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().pcg_strerror(status).decode()


def version() -> str:
    return lib().pcg_version().decode()


def _check(status: int, what: str):
    if status != 0:
        raise PcgError(status, what)


# --------------------------------------------------------------------------- groups

def _np_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


ERR_BAD_CSR = -7


def _csr_i32(row_ptr, members):
    """The two CSR arrays as int32, after the one check that only the caller of the C ABI can
    make: the library learns the number of entries from row_ptr[G] and cannot see how long the
    members array really is."""
    rp, mem = _np_i32(row_ptr), _np_i32(members)
    if rp.ndim != 1 or mem.ndim != 1 or len(rp) < 1 or not 0 <= int(rp[-1]) <= len(mem):
        raise PcgError(ERR_BAD_CSR, "row_ptr[G] does not fit the members array")
    return rp, mem


def groups_validate_host(V: int, row_ptr, members, mult) -> int:
    try:
        rp, mem = _csr_i32(row_ptr, members)
    except PcgError as e:
        return e.status
    mu = _np_i32(mult)
    if len(mu) < V:
        return ERR_BAD_CSR
    return lib().pcg_groups_validate_host(V, len(rp) - 1, rp.ctypes.data, mem.ctypes.data,
                                          mu.ctypes.data)


def groups_canonicalize_host(V: int, row_ptr, members):
    """(row_ptr, members, mult) with a singleton group appended for every uncovered token."""
    rp, mem = _csr_i32(row_ptr, members)
    G = len(rp) - 1
    oG, onnz = C.c_int32(), C.c_int64()
    _check(lib().pcg_groups_canonicalize_host(V, G, rp.ctypes.data, mem.ctypes.data, C.byref(oG),
                                              C.byref(onnz), None, None, None), "canonicalize")
    orp = np.empty(oG.value + 1, np.int32)
    omem = np.empty(max(1, onnz.value), np.int32)
    omult = np.empty(V, np.int32)
    _check(lib().pcg_groups_canonicalize_host(V, G, rp.ctypes.data, mem.ctypes.data, C.byref(oG),
                                              C.byref(onnz), orp.ctypes.data, omem.ctypes.data,
                                              omult.ctypes.data), "canonicalize")
    return orp, omem[:onnz.value], omult


def groups_reverse_host(V: int, row_ptr, members):
    """(tok_ptr [V+1], tok_groups [nnz]): the groups holding each token."""
    rp, mem = _csr_i32(row_ptr, members)
    tok_ptr = np.empty(V + 1, np.int32)
    tok_groups = np.empty(max(1, len(mem)), np.int32)
    _check(lib().pcg_groups_reverse_host(V, len(rp) - 1, rp.ctypes.data, mem.ctypes.data,
                                         tok_ptr.ctypes.data, tok_groups.ctypes.data), "reverse")
    return tok_ptr, tok_groups[:len(mem)]


def groups_validate_weights_host(V: int, row_ptr, members, weights, tol: float = 1e-6) -> int:
    rp, mem = _csr_i32(row_ptr, members)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    if w.ndim != 1 or len(w) < int(rp[-1]):
        return ERR_BAD_CSR
    return lib().pcg_groups_validate_weights_host(V, len(rp) - 1, rp.ctypes.data, mem.ctypes.data,
                                                  w.ctypes.data, tol)


def groups_reverse_weights_host(V: int, row_ptr, members, weights) -> np.ndarray:
    """The per-entry weights in the order of the token -> groups index."""
    rp, mem = _csr_i32(row_ptr, members)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    if w.ndim != 1 or len(w) < int(rp[-1]):
        raise PcgError(ERR_BAD_CSR, "fewer weights than row_ptr[G] entries")
    out = np.empty(max(1, len(mem)), np.float32)
    _check(lib().pcg_groups_reverse_weights_host(V, len(rp) - 1, rp.ctypes.data, mem.ctypes.data,
                                                 w.ctypes.data, out.ctypes.data), "reverse_weights")
    return out[:len(mem)]


def suggest_chunk_groups(G: int, batch: int) -> int:
    """Groups per workgroup of the prepared gather for an expected batch (sequences, or rows of
    pcg_group_probs): small enough to give each of the 256 compute units a workgroup, within the
    library's limits (a multiple of 4096 up to 16384)."""
    want = -(-G * max(1, batch) // 256)
    return int(min(16384, max(4096, -(-want // 4096) * 4096)))


def groups_prepare_host(V: int, row_ptr, members, chunk_groups: int = 0, weights=None):
    """(blob uint8 array, PreparedInfo) of a canonical host CSR; see pcg_groups_prepare_host and,
    with ``weights`` (float32 [nnz]), pcg_groups_prepare_weights_host."""
    rp, mem = _csr_i32(row_ptr, members)
    G = len(rp) - 1
    L = lib()
    sizer = L.pcg_groups_prepare_bytes if weights is None else L.pcg_groups_prepare_weights_bytes
    n = sizer(V, G, rp.ctypes.data, mem.ctypes.data, chunk_groups)
    if n == 0:
        raise PcgError(-2, "pcg_groups_prepare_bytes")
    blob = np.zeros(n, dtype=np.uint8)
    info = PreparedInfo()
    if weights is None:
        _check(L.pcg_groups_prepare_host(V, G, rp.ctypes.data, mem.ctypes.data, chunk_groups,
                                         blob.ctypes.data, n, C.byref(info)), "prepare")
    else:
        w = np.ascontiguousarray(weights, dtype=np.float32)
        assert w.shape == (len(mem),), "one weight per entry"
        _check(L.pcg_groups_prepare_weights_host(V, G, rp.ctypes.data, mem.ctypes.data, w.ctypes.data,
                                                 chunk_groups, blob.ctypes.data, n, C.byref(info)),
               "prepare_weights")
    return blob, info


class Groups:
    """Group membership resident on a device (CSR group -> tokens + multiplicity, and
    optionally the prepared layout the fast gather kernel reads)."""

    def __init__(self, V: int, row_ptr: torch.Tensor, members: torch.Tensor, mult: torch.Tensor,
                 nnz: int, prepared: Optional[torch.Tensor] = None,
                 prepared_info: Optional[PreparedInfo] = None,
                 tok_ptr: Optional[torch.Tensor] = None, tok_groups: Optional[torch.Tensor] = None,
                 weights: Optional[torch.Tensor] = None, tok_weights: Optional[torch.Tensor] = None):
        for t in (row_ptr, members, mult):
            assert t.dtype == torch.int32 and t.is_contiguous()
        self.V, self.G, self.nnz = int(V), int(row_ptr.numel() - 1), int(nnz)
        self.row_ptr, self.members, self.mult = row_ptr, members, mult
        self.prepared, self.prepared_info = prepared, prepared_info
        self.tok_ptr, self.tok_groups = tok_ptr, tok_groups
        self.weights, self.tok_weights = weights, tok_weights
        self.device = row_ptr.device

    @classmethod
    def from_csr(cls, V: int, row_ptr, members, device="cuda", prepare: bool = True,
                 chunk_groups: int = 0, reverse: bool = False, weights=None) -> "Groups":
        """Canonicalise and validate a host CSR with the library, then upload it (with the
        prepared layout unless prepare=False, with the token -> groups index if reverse).
        ``weights`` (float32 [nnz], for the canonical CSR's entries) switches from the equal split
        to general per-entry weights, which the prepared layout then carries too."""
        rp, mem, mult = groups_canonicalize_host(V, row_ptr, members)
        _check(groups_validate_host(V, rp, mem, mult), "validate")
        dev = torch.device(device)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        blob_dev, info = None, None
        wd = twd = None
        if weights is not None:
            w = np.ascontiguousarray(weights, dtype=np.float32)
            assert w.shape == (len(mem),), "one weight per entry of the canonical CSR"
            _check(groups_validate_weights_host(V, rp, mem, w), "validate_weights")
            wd = up(w)
        if prepare:
            blob, info = groups_prepare_host(V, rp, mem, chunk_groups, None if weights is None else w)
            blob_dev = up(blob)
        tp = tg = None
        if reverse:
            tok_ptr, tok_groups = groups_reverse_host(V, rp, mem)
            tp, tg = up(tok_ptr), up(tok_groups if len(tok_groups) else np.zeros(1, np.int32))
            if weights is not None:
                twd = up(groups_reverse_weights_host(V, rp, mem, w))
        return cls(V, up(rp), up(mem if len(mem) else np.zeros(1, np.int32)), up(mult), len(mem),
                   blob_dev, info, tp, tg, wd, twd)

    def without_prepared(self) -> "Groups":
        """The same membership, read through the CSR by the generic kernel."""
        return Groups(self.V, self.row_ptr, self.members, self.mult, self.nnz, None, None,
                      self.tok_ptr, self.tok_groups, self.weights, self.tok_weights)

    def struct(self) -> _GroupsStruct:
        return _GroupsStruct(self.V, self.G, self.nnz, self.row_ptr.data_ptr(),
                             self.members.data_ptr(), self.mult.data_ptr(),
                             None if self.prepared is None else self.prepared.data_ptr(),
                             None if self.prepared_info is None else C.pointer(self.prepared_info),
                             None if self.tok_ptr is None else self.tok_ptr.data_ptr(),
                             None if self.tok_groups is None else self.tok_groups.data_ptr(),
                             None if self.weights is None else self.weights.data_ptr(),
                             None if self.tok_weights is None else self.tok_weights.data_ptr())


# --------------------------------------------------------------------------- calls

_workspaces: dict = {}
_retired: list = []


def _workspace(device: torch.device, nbytes: int) -> torch.Tensor:
    """The default scratch tensor of the calling stream (used when no ``workspace=`` is given).
    One per (device, stream), so calls on different streams never share scratch; a buffer that
    has been handed to a call is kept until the process ends, never freed (work that still
    refers to it may be queued or recorded).  While the stream is being captured into a graph the
    caller must bring the workspace (or use ``static_scratch``): a tensor allocated here would
    be tied to the capture."""
    stream = torch.cuda.current_stream(device)
    if torch.cuda.is_current_stream_capturing():
        raise RuntimeError("pass workspace= (or static_scratch=True) when calling under stream capture")
    key = (device, stream.cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            _retired.append(ws)
        ws = torch.empty(max(nbytes, 1 << 20), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def group_probs_workspace_bytes(V: int, rows: int) -> int:
    return lib().pcg_group_probs_workspace_bytes(V, rows)


def verify_workspace_bytes(V: int, G: int, B: int, K: int) -> int:
    return lib().pcg_verify_workspace_bytes(V, G, B, K)


def group_probs(groups: Groups, logits: torch.Tensor, temperature: float = 1.0,
                out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[rows, V] logits -> [rows, G] float32 group probabilities (Eq. 5)."""
    assert logits.dim() == 2 and logits.shape[1] == groups.V and logits.stride(1) == 1
    assert logits.device == groups.device
    rows = logits.shape[0]
    if out is None:
        out = torch.empty((rows, groups.G), dtype=torch.float32, device=logits.device)
    assert out.shape == (rows, groups.G) and out.is_contiguous() and out.dtype == torch.float32
    need = group_probs_workspace_bytes(groups.V, rows)
    ws = _workspace(logits.device, need) if workspace is None else workspace
    gs = groups.struct()
    with torch.cuda.device(logits.device):
        _check(lib().pcg_group_probs(C.byref(gs), logits.data_ptr(), _dtype_code(logits), rows,
                                     logits.stride(0) if rows > 1 else groups.V,
                                     float(temperature), out.data_ptr(), ws.data_ptr(),
                                     ws.numel(), _stream(logits.device)), "pcg_group_probs")
    return out


@dataclass
class VerifyOutput:
    accept_len: torch.Tensor   # int32 [B]
    out_tokens: torch.Tensor   # int32 [B, K+1], unused tail -1
    out_groups: torch.Tensor   # int32 [B, K+1]


def static_scratch_bytes() -> int:
    return lib().pcg_static_scratch_bytes()


def verify(groups: Groups, target_logits: torch.Tensor, draft_logits: torch.Tensor,
           prop_tokens: torch.Tensor, prop_groups: torch.Tensor, *, temperature: float = 1.0,
           seed: int = 0, offset: int = 0, out: Optional[VerifyOutput] = None,
           diag: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
           B: Optional[int] = None, static_scratch: bool = False) -> VerifyOutput:
    """One speculative step (Algorithm 1) for B sequences.

    target_logits [B, K+1, V], draft_logits [B, >=K, V] (float32 or bfloat16, last axis
    contiguous); prop_tokens / prop_groups int32 [B, K].  ``B`` larger than the tensors'
    batch with batch dimension 1 makes all sequences share the same rows (batch stride 0).
    ``diag`` is an optional zero-initialised int32[8] device tensor that receives pcg_diag.
    ``static_scratch`` calls pcg_verify_static: no workspace is passed or allocated, the
    library's own array is used (``out`` must then be given, so that nothing is allocated).
    """
    assert target_logits.dim() == 3 and draft_logits.dim() == 3
    K, V = target_logits.shape[1] - 1, target_logits.shape[2]
    assert V == groups.V and draft_logits.shape[2] == V and draft_logits.shape[1] >= K
    assert target_logits.stride(2) == 1 and draft_logits.stride(2) == 1
    assert target_logits.dtype == draft_logits.dtype
    dev = target_logits.device
    assert dev == groups.device == draft_logits.device
    if B is None:
        B = target_logits.shape[0]
    shared = B != target_logits.shape[0]
    if shared:
        assert target_logits.shape[0] == 1 and draft_logits.shape[0] == 1
    tbs = 0 if shared else (target_logits.stride(0) if B > 1 else 0)
    dbs = 0 if shared else (draft_logits.stride(0) if B > 1 else 0)
    assert prop_tokens.dtype == torch.int32 and prop_groups.dtype == torch.int32
    assert prop_tokens.is_contiguous() and prop_groups.is_contiguous()
    assert prop_tokens.numel() == B * K and prop_groups.numel() == B * K
    if out is None:
        out = VerifyOutput(torch.empty(B, dtype=torch.int32, device=dev),
                           torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                           torch.empty((B, K + 1), dtype=torch.int32, device=dev))
    gs = groups.struct()
    if static_scratch:
        assert workspace is None
        with torch.cuda.device(dev):
            _check(lib().pcg_verify_static(
                C.byref(gs), target_logits.data_ptr(), draft_logits.data_ptr(),
                _dtype_code(target_logits), B, K, tbs, target_logits.stride(1), dbs,
                draft_logits.stride(1) if K > 1 else V, float(temperature), prop_tokens.data_ptr(),
                prop_groups.data_ptr(), seed, offset, out.accept_len.data_ptr(),
                out.out_tokens.data_ptr(), out.out_groups.data_ptr(),
                None if diag is None else diag.data_ptr(), _stream(dev)), "pcg_verify_static")
        return out
    need = verify_workspace_bytes(V, groups.G, B, K)
    ws = _workspace(dev, need) if workspace is None else workspace
    with torch.cuda.device(dev):
        _check(lib().pcg_verify(C.byref(gs), target_logits.data_ptr(), draft_logits.data_ptr(),
                                _dtype_code(target_logits), B, K, tbs, target_logits.stride(1),
                                dbs, draft_logits.stride(1) if K > 1 else V, float(temperature),
                                prop_tokens.data_ptr(), prop_groups.data_ptr(), seed, offset,
                                out.accept_len.data_ptr(), out.out_tokens.data_ptr(),
                                out.out_groups.data_ptr(),
                                None if diag is None else diag.data_ptr(), ws.data_ptr(),
                                ws.numel(), _stream(dev)), "pcg_verify")
    return out


THIN_MAX_TRIALS = 65520      # PCG_THIN_MAX_TRIALS of pcg.h


def verify_thinning_workspace_bytes(V: int, B: int, K: int) -> int:
    return lib().pcg_verify_thinning_workspace_bytes(V, B, K)


def verify_thinning(groups: Groups, target_logits: torch.Tensor, draft_logits: torch.Tensor,
                    prop_tokens: torch.Tensor, prop_groups: torch.Tensor, *,
                    temperature: float = 1.0, seed: int = 0, offset: int = 0,
                    out: Optional[VerifyOutput] = None, trials: Optional[torch.Tensor] = None,
                    diag: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                    B: Optional[int] = None) -> tuple[VerifyOutput, torch.Tensor]:
    """One speculative step with the reject branch drawn by thinning (Eq. 9).  Arguments as for
    ``verify``; ``groups`` must have been built with ``reverse=True``.  Returns the outputs and
    the int32 [B] number of thinning trials per sequence."""
    assert groups.tok_ptr is not None, "build the groups with reverse=True"
    assert target_logits.dim() == 3 and draft_logits.dim() == 3
    K, V = target_logits.shape[1] - 1, target_logits.shape[2]
    assert V == groups.V and draft_logits.shape[2] == V and draft_logits.shape[1] >= K
    assert target_logits.stride(2) == 1 and draft_logits.stride(2) == 1
    assert target_logits.dtype == draft_logits.dtype
    dev = target_logits.device
    if B is None:
        B = target_logits.shape[0]
    shared = B != target_logits.shape[0]
    if shared:
        assert target_logits.shape[0] == 1 and draft_logits.shape[0] == 1
    tbs = 0 if shared else (target_logits.stride(0) if B > 1 else 0)
    dbs = 0 if shared else (draft_logits.stride(0) if B > 1 else 0)
    assert prop_tokens.dtype == torch.int32 and prop_groups.dtype == torch.int32
    assert prop_tokens.numel() == B * K and prop_groups.numel() == B * K
    if out is None:
        out = VerifyOutput(torch.empty(B, dtype=torch.int32, device=dev),
                           torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                           torch.empty((B, K + 1), dtype=torch.int32, device=dev))
    if trials is None:
        trials = torch.empty(B, dtype=torch.int32, device=dev)
    need = verify_thinning_workspace_bytes(V, B, K)
    ws = _workspace(dev, need) if workspace is None else workspace
    gs = groups.struct()
    with torch.cuda.device(dev):
        _check(lib().pcg_verify_thinning(
            C.byref(gs), target_logits.data_ptr(), draft_logits.data_ptr(),
            _dtype_code(target_logits), B, K, tbs, target_logits.stride(1), dbs,
            draft_logits.stride(1) if K > 1 else V, float(temperature), prop_tokens.data_ptr(),
            prop_groups.data_ptr(), seed, offset, out.accept_len.data_ptr(),
            out.out_tokens.data_ptr(), out.out_groups.data_ptr(), trials.data_ptr(),
            None if diag is None else diag.data_ptr(), ws.data_ptr(), ws.numel(), _stream(dev)),
            "pcg_verify_thinning")
    return out, trials


def propose_workspace_bytes(V: int, B: int, K: int) -> int:
    return lib().pcg_propose_workspace_bytes(V, B, K)


def propose(groups: Groups, draft_logits: torch.Tensor, *, temperature: float = 1.0, seed: int = 0,
            offset: int = 0, pos0: int = 0, prop_tokens: Optional[torch.Tensor] = None,
            prop_groups: Optional[torch.Tensor] = None, diag: Optional[torch.Tensor] = None,
            workspace: Optional[torch.Tensor] = None,
            B: Optional[int] = None) -> tuple[torch.Tensor, torch.Tensor]:
    """Draft-side proposals (Eq. 6): a token from each draft row [B, K, V] and one of the groups
    holding it.  ``groups`` must have been built with ``reverse=True``.  With ``B`` given and a
    leading dimension of 1, all B sequences share the rows.  Returns int32 [B, K] tokens and
    groups."""
    assert groups.tok_ptr is not None, "build the groups with reverse=True"
    assert draft_logits.dim() == 3 and draft_logits.stride(2) == 1
    K, V = draft_logits.shape[1], draft_logits.shape[2]
    assert V == groups.V
    dev = draft_logits.device
    if B is None:
        B = draft_logits.shape[0]
    shared = B != draft_logits.shape[0]
    if shared:
        assert draft_logits.shape[0] == 1
    dbs = 0 if shared else (draft_logits.stride(0) if B > 1 else 0)
    if prop_tokens is None:
        prop_tokens = torch.empty((B, K), dtype=torch.int32, device=dev)
    if prop_groups is None:
        prop_groups = torch.empty((B, K), dtype=torch.int32, device=dev)
    assert prop_tokens.dtype == torch.int32 and prop_groups.dtype == torch.int32
    assert prop_tokens.numel() == B * K and prop_groups.numel() == B * K
    need = propose_workspace_bytes(V, B, K)
    ws = _workspace(dev, need) if workspace is None else workspace
    gs = groups.struct()
    with torch.cuda.device(dev):
        _check(lib().pcg_propose(
            C.byref(gs), draft_logits.data_ptr(), _dtype_code(draft_logits), B, K, pos0, dbs,
            draft_logits.stride(1) if K > 1 else V, float(temperature), seed, offset,
            prop_tokens.data_ptr(), prop_groups.data_ptr(),
            None if diag is None else diag.data_ptr(), ws.data_ptr(), ws.numel(), _stream(dev)),
            "pcg_propose")
    return prop_tokens, prop_groups


ERR_CAPACITY = -10


def asg_normalize(emb: torch.Tensor) -> torch.Tensor:
    """float32 [V, d] embeddings -> bfloat16 unit vectors (Sec. 2.1)."""
    assert emb.dim() == 2 and emb.dtype == torch.float32 and emb.is_contiguous()
    unit = torch.empty(emb.shape, dtype=torch.bfloat16, device=emb.device)
    with torch.cuda.device(emb.device):
        _check(lib().pcg_asg_normalize(emb.data_ptr(), emb.shape[0], emb.shape[1], unit.data_ptr(),
                                       _stream(emb.device)), "pcg_asg_normalize")
    return unit


@dataclass
class AsgGroups:
    row_ptr: torch.Tensor    # int32 [G + 1]
    members: torch.Tensor    # int32 [nnz]
    mult: torch.Tensor       # int32 [V]
    seed_of: torch.Tensor    # int32 [G]
    G: int
    nnz: int
    max_size: int            # largest G(t) before identical sets were dropped


def _asg_build(name, call, ws_bytes, V: int, dev, cap: int, members_capacity: Optional[int]) -> AsgGroups:
    cap = min(cap, 4096)
    room = members_capacity or 32 * V
    G, nnz, largest = C.c_int32(), C.c_int64(), C.c_int32()
    while True:
        row_ptr = torch.empty(V + 1, dtype=torch.int32, device=dev)
        members = torch.empty(room, dtype=torch.int32, device=dev)
        mult = torch.empty(V, dtype=torch.int32, device=dev)
        seed_of = torch.empty(V, dtype=torch.int32, device=dev)
        ws = torch.empty(ws_bytes(cap), dtype=torch.uint8, device=dev)
        with torch.cuda.device(dev):
            rc = call(cap, row_ptr.data_ptr(), members.data_ptr(), room, mult.data_ptr(),
                      seed_of.data_ptr(), C.byref(G), C.byref(nnz), C.byref(largest), ws.data_ptr(),
                      ws.numel(), _stream(dev))
        if rc == ERR_CAPACITY and (largest.value > cap or nnz.value > room):
            if largest.value > 4096:
                raise PcgError(rc, f"{name}: a similarity group has more than 4096 members")
            cap = max(cap, min(4096, largest.value))
            room = max(room, nnz.value)
            continue
        _check(rc, name)
        return AsgGroups(row_ptr[:G.value + 1], members[:nnz.value], mult, seed_of[:G.value],
                         G.value, nnz.value, largest.value)


def asg_build(unit: torch.Tensor, theta: float, cap: int = 256,
              members_capacity: Optional[int] = None) -> AsgGroups:
    """The distinct similarity groups of Eq. (1) from bfloat16 unit vectors [V, d], as device
    CSR arrays.  Room for a group (cap) and for all members is enlarged and the call repeated
    when the library reports that it did not suffice."""
    assert unit.dim() == 2 and unit.dtype == torch.bfloat16 and unit.is_contiguous()
    V, d = unit.shape
    L = lib()
    return _asg_build("pcg_asg_build",
                      lambda cap, *rest: L.pcg_asg_build(unit.data_ptr(), V, d, float(theta), cap, *rest),
                      lambda cap: L.pcg_asg_build_workspace_bytes(V, cap), V, unit.device, cap,
                      members_capacity)


def asg_build_exact(emb: torch.Tensor, theta: float, cap: int = 256,
                    members_capacity: Optional[int] = None) -> AsgGroups:
    """The distinct similarity groups of Eq. (1) from the float32 embeddings [V, d] themselves:
    the cosine is decided in double wherever the bfloat16 contraction cannot.  Same outputs and
    retries as asg_build."""
    assert emb.dim() == 2 and emb.dtype == torch.float32 and emb.is_contiguous()
    V, d = emb.shape
    L = lib()
    return _asg_build("pcg_asg_build_exact",
                      lambda cap, *rest: L.pcg_asg_build_exact(emb.data_ptr(), V, d, float(theta), cap, *rest),
                      lambda cap: L.pcg_asg_build_exact_workspace_bytes(V, d, cap), V, emb.device, cap,
                      members_capacity)


def profile_begin(max_calls: int):
    _check(lib().pcg_profile_begin(max_calls), "pcg_profile_begin")


def profile_end() -> tuple[dict, int]:
    """({stage name: mean milliseconds}, number of recorded calls)."""
    ms = (C.c_float * MAX_STAGES)()
    calls = C.c_int32()
    _check(lib().pcg_profile_end(ms, C.byref(calls)), "pcg_profile_end")
    out = {}
    for i in range(MAX_STAGES):
        name = lib().pcg_stage_name(i).decode()
        if name:
            out[name] = float(ms[i])
    return out, calls.value
