"""Pins for the oracle's similarity-group construction (Sec. 2.1, Eq. 1): the bf16 unit vectors
against an independent rounding in extended precision, the similarity against numpy's dot, the
thresholded sets and their de-duplication against a dense numpy similarity matrix and Python
sets, and what the definition fixes in closed form: self-membership, symmetry, monotonicity in
theta, one group for theta below -1, singletons for theta near 1, merged duplicates, and
clusters recovered exactly from well-separated mixtures."""
import numpy as np
import pytest
import torch

import oracle


def bf16_to_f64(bits):
    return (np.asarray(bits, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)


def embeddings(V, d, seed, centres=0, sigma=0.05):
    rng = np.random.default_rng(seed)
    if centres == 0:
        return rng.standard_normal((V, d)).astype(np.float32)
    c = rng.standard_normal((centres, d))
    assign = rng.integers(0, centres, size=V)
    assign[:centres] = np.arange(centres)                    # every centre is used
    return (c[assign] + sigma * rng.standard_normal((V, d))).astype(np.float32), assign


def dense_sets(unit, theta):
    """Every token's set from a dense float64 similarity matrix."""
    U = bf16_to_f64(unit)
    S = U @ U.T
    np.fill_diagonal(S, 2.0)
    return [np.flatnonzero(S[t] > np.float64(np.float32(theta))).astype(np.int32) for t in range(len(U))], S


def distinct_in_order(sets):
    seen, kept, seeds = set(), [], []
    for t, s in enumerate(sets):
        key = s.tobytes()
        if key not in seen:
            seen.add(key)
            kept.append(s)
            seeds.append(t)
    return kept, seeds


def test_unit_vectors_are_rounded_once_from_the_exact_quotient():
    E = embeddings(64, 48, 1)
    E[5] = 0.0
    unit = oracle.asg_normalize(E)
    assert (unit[5] == 0).all()
    L = E.astype(np.longdouble)
    x = L / np.sqrt((L * L).sum(axis=1, keepdims=True).clip(min=1e-300))
    x[5] = 0
    # the two bf16 neighbours of x by truncating its float32 image, and the nearer one
    f = x.astype(np.float32)
    lo = (f.view(np.uint32) & 0xFFFF0000)
    for _ in range(2):      # the float32 image may have rounded past a bf16 value
        flo = lo.view(np.float32).astype(np.longdouble)
        lo = np.where(np.abs(flo) > np.abs(x), lo - 0x10000, lo).astype(np.uint32)
    hi = (lo + 0x10000).astype(np.uint32)
    dlo = np.abs(x) - np.abs(lo.view(np.float32).astype(np.longdouble))
    dhi = np.abs(hi.view(np.float32).astype(np.longdouble)) - np.abs(x)
    assert (dlo >= 0).all() and (dhi > 0).all()
    want = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where((lo >> 16) & 1, hi, lo))) >> 16
    want[5] = 0
    np.testing.assert_array_equal(unit, want.astype(np.uint16))
    # a library rounding of the float32 quotient agrees except where that quotient is itself a
    # rounding boundary case (double rounding): a handful of elements at most
    t = torch.from_numpy((E.astype(np.float64) / np.linalg.norm(E.astype(np.float64), axis=1, keepdims=True).clip(1e-300)
                          ).astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (t != unit).sum() <= 3
    norms = np.linalg.norm(bf16_to_f64(unit), axis=1)
    np.testing.assert_allclose(np.delete(norms, 5), 1.0, atol=2.0 ** -8)


def test_similarity_is_the_dot_product_of_the_stored_vectors():
    unit = oracle.asg_normalize(embeddings(40, 96, 2))
    U = bf16_to_f64(unit)
    S = U @ U.T
    for a, b in [(0, 0), (3, 17), (17, 3), (39, 1)]:
        assert abs(oracle.asg_similarity(unit, a, b) - S[a, b]) < 1e-15
    assert oracle.asg_similarity(unit, 3, 17) == oracle.asg_similarity(unit, 17, 3)


@pytest.mark.parametrize("V,d,theta,centres", [(300, 32, 0.25, 0), (500, 64, 0.1, 0), (400, 48, 0.6, 12)])
def test_groups_match_dense_thresholding_and_python_sets(V, d, theta, centres):
    E = embeddings(V, d, 3) if centres == 0 else embeddings(V, d, 3, centres, 0.4)[0]
    unit = oracle.asg_normalize(E)
    res = oracle.asg_build(unit, theta, nthreads=4)
    sets, S = dense_sets(unit, theta)
    off = S[~np.eye(V, dtype=bool)]
    assert (np.abs(off - np.float32(theta)) > 1e-9).all()          # no decision hangs on rounding
    kept, seeds = distinct_in_order(sets)
    g = res.groups
    assert g.G == len(kept) and g.nnz == sum(len(s) for s in kept)
    np.testing.assert_array_equal(res.seed_of, seeds)
    for k, s in enumerate(kept):
        np.testing.assert_array_equal(g.members[g.row_ptr[k]:g.row_ptr[k + 1]], s)
    np.testing.assert_array_equal(g.mult, np.bincount(g.members, minlength=V))
    assert oracle.validate(g) == 0 and (g.mult >= 1).all()
    near = (np.abs(S - np.float32(theta)) < 1e-5) & ~np.eye(V, dtype=bool)
    np.testing.assert_array_equal(res.near_rows, near.any(axis=1))
    for t in (0, V // 2, V - 1):
        row, n_near = oracle.asg_row(unit, theta, t)
        np.testing.assert_array_equal(row, sets[t])
        assert n_near == near[t].sum()


def test_what_the_definition_fixes():
    V, d = 200, 40
    E = embeddings(V, d, 7)
    E[150] = E[20]                     # two tokens with the same embedding
    E[151] = 3.0 * E[21]               # and two that differ by a positive factor
    unit = oracle.asg_normalize(E)
    rows = {th: [oracle.asg_row(unit, th, t)[0] for t in range(V)] for th in (0.1, 0.3)}
    for th, rs in rows.items():
        for t, r in enumerate(rs):
            assert t in r and (np.diff(r) > 0).all()                          # self, ascending
        member = np.zeros((V, V), bool)
        for t, r in enumerate(rs):
            member[t, r] = True
        assert (member == member.T).all()                                     # symmetry
    for t in range(V):
        assert set(rows[0.3][t]) <= set(rows[0.1][t])                         # monotone in theta
    assert oracle.asg_build(unit, -1.5).groups.G == 1                         # everything is similar
    assert oracle.asg_build(unit, -1.5).groups.nnz == V
    single = oracle.asg_build(unit, 0.9)
    # near theta = 1 only identical directions group: {20, 150} and {21, 151}, once each
    assert single.groups.G == V - 2 and single.groups.nnz == V
    np.testing.assert_array_equal(single.groups.members[single.groups.row_ptr[20]:single.groups.row_ptr[21]], [20, 150])
    assert 150 not in single.seed_of and 151 not in single.seed_of


def test_well_separated_clusters_are_recovered_exactly():
    V, d, C = 600, 128, 9
    E, assign = embeddings(V, d, 11, centres=C, sigma=0.05)
    res = oracle.asg_build(oracle.asg_normalize(E), 0.5, nthreads=4)
    g = res.groups
    assert g.G == C and g.nnz == V and (g.mult == 1).all()
    for k in range(C):
        seg = g.members[g.row_ptr[k]:g.row_ptr[k + 1]]
        np.testing.assert_array_equal(seg, np.flatnonzero(assign == assign[res.seed_of[k]]))
