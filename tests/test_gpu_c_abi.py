"""The C ABI used from a plain C program (tests/c_abi/verify_from_c.c: HIP runtime for memory,
libpcg for everything else, no Python and no PyTorch in the process).  The test rebuilds the
program's inputs from its generator, hands them to the oracle and compares what the program
printed.  Run with ``-m gpu`` on an MI355X; the program is built by __graft_entry__.build()."""
import os
import subprocess

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
PROGRAM = os.path.join(HERE, "c_abi", "verify_from_c")
V, G0, B, K = 96, 20, 5, 3


class Lcg:
    def __init__(self):
        self.s = 12345

    def next(self):
        self.s = (self.s * 1664525 + 1013904223) & 0xFFFFFFFF
        return self.s >> 8

    def unit(self):
        return np.float32((self.next() & 0xFFFFFF) - 0x800000) * np.float32(1.0 / 8388608.0)


def program_inputs():
    r = Lcg()
    rp, mem = [0], []
    for _ in range(G0):
        n = 2 + r.next() % 5
        m = []
        while len(m) < n:
            t = r.next() % 90
            if t not in m:
                m.append(t)
        mem += sorted(m)
        rp.append(rp[-1] + n)
    og = oracle.canonicalize(V, np.array(rp, np.int32), np.array(mem, np.int32))
    tgt = np.array([np.float32(3.0) * r.unit() for _ in range(B * (K + 1) * V)], np.float32).reshape(B, K + 1, V)
    noise = np.array([np.float32(0.75) * r.unit() for _ in range(B * K * V)], np.float32).reshape(B, K, V)
    dft = (tgt[:, :K] + noise).astype(np.float32)
    ptok, pgrp = np.zeros((B, K), np.int32), np.zeros((B, K), np.int32)
    for b in range(B):
        for i in range(K):
            g = r.next() % og.G
            pgrp[b, i] = g
            ptok[b, i] = og.members[og.row_ptr[g] + r.next() % (og.row_ptr[g + 1] - og.row_ptr[g])]
    return og, tgt, dft, ptok, pgrp


def test_a_c_program_gets_the_oracles_answers():
    if not os.path.exists(PROGRAM):          # built by __graft_entry__.build(); only if that has not run
        import __graft_entry__
        __graft_entry__.build_c_caller()
    run = subprocess.run([PROGRAM], capture_output=True, text=True, timeout=120)
    print(run.stdout, run.stderr, flush=True)
    assert run.returncode == 0
    lines = run.stdout.splitlines()
    og, tgt, dft, ptok, pgrp = program_inputs()
    assert lines[0].startswith("version libpcg")
    assert lines[1].split() == ["groups", str(og.G), str(og.nnz)]
    assert og.G >= G0 + 6                          # tokens 90..95 (and others) became singleton groups
    ref = oracle.verify(og, tgt, dft, ptok, pgrp, temperature=1.0, seed=7, offset=3)
    near = ref.near_acc.any(axis=1) | ref.near_grp.astype(bool) | ref.near_tok.astype(bool)
    accepted = 0
    for b in range(B):
        w = lines[2 + b].split()
        assert w[:3] == ["seq", str(b), "len"]
        n = int(w[3])
        toks = [int(x) for x in w[5:5 + K + 1]]
        grps = [int(x) for x in w[6 + K + 1:6 + 2 * (K + 1)]]
        accepted += n
        if near[b]:
            continue
        assert n == ref.accept_len[b], b
        assert toks == ref.out_tokens[b].tolist() and grps == ref.out_groups[b].tolist(), b
    want = oracle.group_probs(og, np.ascontiguousarray(tgt[:, 0]), 1.0)
    for b in range(B):
        w = lines[2 + B + b].split()
        assert w[:2] == ["probs", str(b)]
        got = np.array([float(x) for x in w[2:]])
        assert got.shape == (og.G,)
        assert np.max(np.abs(got - want[b]) / (want[b] + 1e-25)) <= 1e-5
        assert abs(got.sum() - 1.0) < 2e-6
    assert lines[2 + 2 * B].split() == ["diag", "sequences", str(B), "accepted", str(accepted)]
    assert lines[3 + 2 * B].startswith("K=0 status -") and "status 0" not in lines[3 + 2 * B]
