"""Malformed memberships thrown at the library's host-side helpers: every call must come back
with a status (never read outside the arrays it was given, which the sanitizer build checks:
see tests/conftest.py for its command line), must agree with the oracle's validator on what is
a usable membership, and must leave its outputs consistent when it accepts."""
import ctypes as C

import numpy as np

import oracle
import paper_2511_13732_amd as pcg


def exact(a):
    """A heap array of exactly a's size (so that a read past its end is seen by the sanitizer)."""
    out = np.empty(len(a), dtype=np.int32)
    out[:] = a
    return out


def mutate(rng, V, rp, mem):
    rp, mem = rp.copy(), mem.copy()
    kind = int(rng.integers(0, 8))
    G = len(rp) - 1
    if kind == 0 and len(mem):
        mem[rng.integers(0, len(mem))] = int(rng.choice([-1, V, V + 5, 2**31 - 1, -2**31]))
    elif kind == 1:
        rp[rng.integers(0, G + 1)] = int(rng.choice([-3, len(mem) + 7, 2**31 - 1]))
    elif kind == 2 and G >= 2:
        i = int(rng.integers(1, G))
        rp[i], rp[i + 1] = rp[i + 1], rp[i]                       # may or may not break monotonicity
    elif kind == 3:
        rp[0] = 1
    elif kind == 4:
        rp[G] = max(0, rp[G] - int(rng.integers(1, 4)))           # last pointer short of the entries
    elif kind == 5 and len(mem) >= 2:
        j = int(rng.integers(1, len(mem)))
        mem[j] = mem[j - 1]                                        # a repeated entry: legal (counted twice)
    elif kind == 6:
        rp[:] = 0                                                  # every group empty
    return rp, mem


def test_malformed_memberships_are_refused_not_followed():
    rng = np.random.default_rng(20251113)
    L = pcg.lib()
    refused = accepted = 0
    for case in range(400):
        V = int(rng.integers(1, 60))
        G = int(rng.integers(1, 40))
        sizes = rng.integers(0, min(V, 6) + 1, size=G)
        rp0 = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        mem0 = np.concatenate([np.sort(rng.choice(V, size=s, replace=False)) for s in sizes] + [np.empty(0, np.int64)]).astype(np.int32)
        rp, mem = mutate(rng, V, rp0, mem0)
        rp, mem = exact(rp), exact(mem)
        # the oracle's verdict on the raw membership: usable iff canonicalisation succeeds
        try:
            want = oracle.canonicalize(V, rp, mem)
        except Exception:
            want = None
        try:
            got = pcg.groups_canonicalize_host(V, rp, mem)
        except pcg.PcgError:
            got = None
        assert (got is None) == (want is None), (case, V, rp.tolist(), mem.tolist())
        # The C ABI learns the number of entries from row_ptr[G]: handing it a shorter members
        # array is the caller's fault, which the Python layers catch.  Only memberships whose
        # arrays fit may go to the library directly.
        fits = 0 <= int(rp[-1]) <= len(mem)
        if got is None:
            refused += 1
            if fits:
                n = L.pcg_groups_prepare_bytes(V, G, rp.ctypes.data, mem.ctypes.data if len(mem) else None, 0)
                if n:       # the sizer may answer for shapes alone; the builder itself must refuse
                    blob = np.zeros(n, np.uint8)
                    info = pcg.PreparedInfo()
                    rc = L.pcg_groups_prepare_host(V, G, rp.ctypes.data, mem.ctypes.data if len(mem) else None, 0,
                                                   blob.ctypes.data, n, C.byref(info))
                    assert rc != 0, (case, rc)
                assert pcg.groups_validate_host(V, rp, mem, np.ones(V, np.int32)) != 0
            else:
                assert pcg.groups_validate_host(V, rp, mem, np.ones(V, np.int32)) == -7
            continue
        accepted += 1
        rp2, mem2, mult2 = got
        np.testing.assert_array_equal(rp2, want.row_ptr)
        np.testing.assert_array_equal(mem2, want.members)
        np.testing.assert_array_equal(mult2, want.mult)
        assert pcg.groups_validate_host(V, rp2, mem2, mult2) == 0
        blob, info = pcg.groups_prepare_host(V, exact(rp2), exact(mem2))
        assert info.G == len(rp2) - 1 and info.bytes == len(blob)
        tok_ptr, tok_groups = pcg.groups_reverse_host(V, exact(rp2), exact(mem2))
        rev = oracle.reverse_index(want)
        np.testing.assert_array_equal(tok_ptr, rev[0])
        np.testing.assert_array_equal(tok_groups, rev[1])
        # a wrong multiplicity is caught
        if len(mult2):
            bad = mult2.copy()
            bad[int(rng.integers(0, len(bad)))] += 1
            assert pcg.groups_validate_host(V, rp2, mem2, bad) != 0
    print(f"{refused} memberships refused, {accepted} accepted")
    assert refused > 50 and accepted > 50
