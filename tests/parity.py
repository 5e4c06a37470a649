"""Shared helpers of the GPU parity tests: run both sides on the same inputs and
compare under the near-tie rule.

Integer outputs (accept lengths, emitted tokens and groups) must agree exactly.
The only tolerated disagreement is on a draw that the *oracle* flags as lying
within 1e-6 (on the unit interval) of the threshold that decides it: there the
fp32 kernel and the fp64 oracle may legitimately land on different sides.
Every such draw is counted, every tolerated mismatch is counted, and after one
the rest of that sequence's step is excluded from the comparison.
"""
from __future__ import annotations

import json
import os
from dataclasses import dataclass, field

import numpy as np
import torch

import oracle
import paper_2511_13732_amd as pcg

# Every tally is printed; with PCG_PARITY_REPORT set it is also appended to that file (JSON lines).
REPORT = os.environ.get("PCG_PARITY_REPORT", "")


def _append_report(rec: dict):
    if not REPORT:
        return
    try:
        os.makedirs(os.path.dirname(os.path.abspath(REPORT)), exist_ok=True)
        with open(REPORT, "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass


@dataclass
class Tally:
    sequences: int = 0
    flagged_accept: int = 0
    flagged_group: int = 0
    flagged_token: int = 0
    tolerated: int = 0
    detail: list = field(default_factory=list)

    def add(self, other: "Tally"):
        for k in ("sequences", "flagged_accept", "flagged_group", "flagged_token", "tolerated"):
            setattr(self, k, getattr(self, k) + getattr(other, k))
        self.detail += other.detail

    def report(self, name: str):
        rec = {"case": name, "sequences": self.sequences, "flagged_accept": self.flagged_accept,
               "flagged_group": self.flagged_group, "flagged_token": self.flagged_token,
               "tolerated_mismatches": self.tolerated, "detail": self.detail[:20]}
        print("parity", json.dumps(rec), flush=True)
        _append_report(rec)


def report_error(name: str, err: float):
    """Record a measured group-probability error next to the tallies."""
    rec = {"case": name, "max_rel_err": err}
    print("parity", json.dumps(rec), flush=True)
    _append_report(rec)


def oracle_groups(V: int, row_ptr, members) -> oracle.Groups:
    return oracle.canonicalize(V, row_ptr, members)


def device_groups(V: int, row_ptr, members, prepare: bool = True, chunk_groups: int = 0) -> pcg.Groups:
    return pcg.Groups.from_csr(V, row_ptr, members, "cuda", prepare=prepare, chunk_groups=chunk_groups)


def as_oracle_logits(t: torch.Tensor):
    t = t.detach().cpu().contiguous()           # the device side may be a strided view
    return oracle.bf16_bits(t) if t.dtype == torch.bfloat16 else t.numpy()


def compare_verify(gpu: pcg.VerifyOutput, ref: oracle.VerifyResult, og: oracle.Groups,
                   prop_tokens: np.ndarray, prop_groups: np.ndarray) -> Tally:
    al = gpu.accept_len.cpu().numpy()
    tok = gpu.out_tokens.cpu().numpy()
    grp = gpu.out_groups.cpu().numpy()
    B, K1 = tok.shape
    K = K1 - 1
    prop_tokens = np.asarray(prop_tokens).reshape(B, K)
    prop_groups = np.asarray(prop_groups).reshape(B, K)
    t = Tally(sequences=B)
    t.flagged_accept = int(ref.near_acc.sum())
    t.flagged_group = int(ref.near_grp.sum())
    t.flagged_token = int(ref.near_tok.sum())
    for b in range(B):
        n = int(al[b])
        # structure that holds whatever the draws were
        assert 0 <= n <= K, (b, n)
        assert (tok[b, :n] == prop_tokens[b, :n]).all() and (grp[b, :n] == prop_groups[b, :n]).all()
        assert (tok[b, n + 1:] == -1).all() and (grp[b, n + 1:] == -1).all()
        g, z = int(grp[b, n]), int(tok[b, n])
        assert 0 <= g < og.G, (b, g)
        assert z in og.members[og.row_ptr[g]:og.row_ptr[g + 1]], (b, g, z)
        # exact agreement with the oracle, except on flagged draws
        nr = int(ref.accept_len[b])
        if n != nr:
            i = min(n, nr)
            assert ref.near_acc[b, i], f"seq {b}: accept_len {n} vs oracle {nr}, draw not near a tie"
            t.tolerated += 1
            t.detail.append({"b": b, "kind": "accept", "gpu": n, "oracle": nr})
            continue
        if g != int(ref.out_groups[b, n]):
            assert ref.near_grp[b], f"seq {b}: group {g} vs oracle {ref.out_groups[b, n]}, not near a tie"
            t.tolerated += 1
            t.detail.append({"b": b, "kind": "group", "gpu": g, "oracle": int(ref.out_groups[b, n])})
            continue
        if z != int(ref.out_tokens[b, n]):
            assert ref.near_tok[b], f"seq {b}: token {z} vs oracle {ref.out_tokens[b, n]}, not near a tie"
            t.tolerated += 1
            t.detail.append({"b": b, "kind": "token", "gpu": z, "oracle": int(ref.out_tokens[b, n])})
    return t


def run_both(V, row_ptr, members, tgt: torch.Tensor, dft: torch.Tensor, ptok, pgrp, *,
             temperature=1.0, seed=0, offset=0, dg: pcg.Groups = None, og: oracle.Groups = None,
             nthreads=16, static_scratch=False):
    """Run the HIP library and the oracle on the same inputs; returns (gpu, ref, og, diag)."""
    og = og or oracle_groups(V, row_ptr, members)
    dg = dg or device_groups(V, row_ptr, members)
    diag = torch.zeros(8, dtype=torch.int32, device="cuda")
    gpu = pcg.verify(dg, tgt.cuda(), dft.cuda(),
                     torch.from_numpy(np.ascontiguousarray(ptok, dtype=np.int32)).cuda(),
                     torch.from_numpy(np.ascontiguousarray(pgrp, dtype=np.int32)).cuda(),
                     temperature=temperature, seed=seed, offset=offset, diag=diag,
                     static_scratch=static_scratch)
    torch.cuda.synchronize()
    ref = oracle.verify(og, as_oracle_logits(tgt), as_oracle_logits(dft), ptok, pgrp,
                        temperature=temperature, seed=seed, offset=offset, nthreads=nthreads)
    return gpu, ref, og, dict(zip(pcg.Diag.NAMES, diag.cpu().tolist()))


def group_probs_error(gpu: torch.Tensor, ref: np.ndarray) -> float:
    """Largest |gpu - ref| / (ref + floor): relative error with an absolute floor of 1e-30
    for probabilities that underflow in fp32."""
    g = gpu.double().cpu().numpy()
    return float(np.max(np.abs(g - ref) / (ref + 1e-30 / 1e-5)))


def compare_thinning(gpu: pcg.VerifyOutput, gpu_trials: torch.Tensor, ref: oracle.ThinningResult,
                     og: oracle.Groups, prop_tokens: np.ndarray, prop_groups: np.ndarray) -> Tally:
    """As compare_verify, for the thinning sampler: accept length, emitted token and group and
    the number of trials agree exactly unless the oracle flagged a near-tie on that path."""
    al = gpu.accept_len.cpu().numpy()
    tok = gpu.out_tokens.cpu().numpy()
    grp = gpu.out_groups.cpu().numpy()
    ntr = gpu_trials.cpu().numpy()
    B, K1 = tok.shape
    K = K1 - 1
    prop_tokens = np.asarray(prop_tokens).reshape(B, K)
    prop_groups = np.asarray(prop_groups).reshape(B, K)
    t = Tally(sequences=B)
    t.flagged_accept = int(ref.near_acc.sum())
    t.flagged_group = int((ref.flags & 1).sum())
    for b in range(B):
        n = int(al[b])
        assert 0 <= n <= K, (b, n)
        assert (tok[b, :n] == prop_tokens[b, :n]).all() and (grp[b, :n] == prop_groups[b, :n]).all()
        assert (tok[b, n + 1:] == -1).all() and (grp[b, n + 1:] == -1).all()
        g, z = int(grp[b, n]), int(tok[b, n])
        assert 0 <= g < og.G, (b, g)
        assert z in og.members[og.row_ptr[g]:og.row_ptr[g + 1]], (b, g, z)
        assert (ntr[b] == 0) == (n == K), (b, n, ntr[b])
        nr = int(ref.accept_len[b])
        if n != nr:
            assert ref.near_acc[b, min(n, nr)], f"seq {b}: accept_len {n} vs oracle {nr}, no near-tie"
            t.tolerated += 1
            t.detail.append({"b": b, "kind": "accept", "gpu": n, "oracle": nr})
            continue
        got = (g, z, int(ntr[b]))
        want = (int(ref.out_groups[b, n]), int(ref.out_tokens[b, n]), int(ref.trials[b]))
        if got != want:
            assert ref.flags[b] & 1, f"seq {b}: (group, token, trials) {got} vs oracle {want}, no near-tie"
            t.tolerated += 1
            t.detail.append({"b": b, "kind": "thinning", "gpu": got, "oracle": want})
    return t


def run_both_thinning(V, tgt: torch.Tensor, dft: torch.Tensor, ptok, pgrp, *, dg: pcg.Groups,
                      og: oracle.Groups, rev, temperature=1.0, seed=0, offset=0, nthreads=16):
    """The thinning entry point of the HIP library and of the oracle on the same inputs."""
    diag = torch.zeros(8, dtype=torch.int32, device="cuda")
    gpu, trials = pcg.verify_thinning(
        dg, tgt.cuda(), dft.cuda(), torch.from_numpy(np.ascontiguousarray(ptok, dtype=np.int32)).cuda(),
        torch.from_numpy(np.ascontiguousarray(pgrp, dtype=np.int32)).cuda(),
        temperature=temperature, seed=seed, offset=offset, diag=diag)
    torch.cuda.synchronize()
    ref = oracle.verify_thinning(og, rev, as_oracle_logits(tgt), as_oracle_logits(dft), ptok, pgrp,
                                 temperature=temperature, seed=seed, offset=offset,
                                 max_trials=pcg.THIN_MAX_TRIALS, nthreads=nthreads)
    return gpu, trials, ref, dict(zip(pcg.Diag.NAMES, diag.cpu().tolist()))
