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


# --------------------------------------------------------------------------- Eq. (1) itself

def numpy_cosines(E):
    """Cosine matrix of float32 embeddings with numpy in float64 (independent of the oracle)."""
    X = np.asarray(E, dtype=np.float64)
    n = np.sqrt(np.einsum("ij,ij->i", X, X))
    Xn = np.divide(X, n[:, None], out=np.zeros_like(X), where=n[:, None] > 0)
    return Xn @ Xn.T


@pytest.mark.parametrize("V,d,theta,centres", [(300, 32, 0.25, 0), (400, 48, 0.6, 12), (257, 100, -0.05, 0)])
def test_exact_rows_are_the_definition_on_the_embeddings(V, d, theta, centres):
    """pcg_ref_asg_row_exact is Eq. (1) as printed: cosine of the float32 embeddings in double,
    strict > theta, t in G(t).  Pinned against a numpy cosine matrix and Python sets."""
    E = embeddings(V, d, 9) if centres == 0 else embeddings(V, d, 9, centres, 0.4)[0]
    E[7] = 0.0                                                    # a zero row: cosine 0 with everything
    S = numpy_cosines(E)
    for a, b in [(0, 1), (5, 200), (200, 5), (7, 3), (3, 7), (V - 1, V - 2)]:
        assert abs(oracle.asg_cosine(E, a, b) - S[a, b]) < 1e-14
    assert oracle.asg_cosine(E, 5, 200) == oracle.asg_cosine(E, 200, 5)
    assert abs(oracle.asg_cosine(E, 11, 11) - 1.0) < 1e-15
    off = S[~np.eye(V, dtype=bool)]
    assert (np.abs(off - theta) > 1e-12).all()                    # no decision hangs on summation order
    for t in (0, 7, 100, V - 1):
        row, cos = oracle.asg_row_exact(E, theta, t)
        want = sorted(set(np.flatnonzero(S[t] > theta).tolist()) | {t})
        np.testing.assert_array_equal(row, want)
        np.testing.assert_allclose(np.delete(cos, t), np.delete(S[t], t), atol=1e-14)
        assert cos[t] == 1.0
    # strictness: a threshold exactly at a pair's cosine excludes that pair, just below includes it
    c = oracle.asg_cosine(E, 0, 1)
    assert 1 not in oracle.asg_row_exact(E, c, 0)[0]
    assert 1 in oracle.asg_row_exact(E, np.nextafter(c, -1.0), 0)[0]
    # positive scaling of an embedding changes nothing (cosine), a sign flip mirrors it
    E2 = E.copy()
    E2[1] *= 4.0
    assert abs(oracle.asg_cosine(E2, 0, 1) - c) < 1e-15
    E2[1] *= -1.0
    assert abs(oracle.asg_cosine(E2, 0, 1) + c) < 1e-15


@pytest.mark.parametrize("V,d,theta,centres", [(300, 32, 0.25, 0), (400, 48, 0.6, 12), (200, 16, 0.9, 5)])
def test_exact_groups_are_the_distinct_sets_of_eq1_in_order_of_first_appearance(V, d, theta, centres):
    """pcg_ref_asg_build_exact: every token's set from a numpy cosine matrix, de-duplicated with
    Python sets in order of first appearance; members ascending, mult the entry counts.  Exact
    duplicates of an embedding (cosine 1 with each other, equal cosines with everyone else) must
    fall into one group."""
    E = embeddings(V, d, 21) if centres == 0 else embeddings(V, d, 21, centres, 0.05)[0]
    E[40] = E[3]                                                  # the same embedding twice
    E[41] = 2.5 * E[3]                                            # and scaled: same direction
    S = numpy_cosines(E)
    np.fill_diagonal(S, 2.0)
    assert (np.abs(S - theta) > 1e-9)[S < 0.999999].all()
    sets = [np.flatnonzero((S[t] > theta) | (S[t] > 0.9999999)).astype(np.int32) for t in range(V)]
    kept, seeds = distinct_in_order(sets)
    for nthreads in (1, 3):
        res = oracle.asg_build_exact(E, theta, nthreads=nthreads)
        g = res.groups
        assert g.G == len(kept) and g.V == V
        np.testing.assert_array_equal(res.seed_of, seeds)
        for k, want in enumerate(kept):
            np.testing.assert_array_equal(g.members[g.row_ptr[k]:g.row_ptr[k + 1]], want)
        np.testing.assert_array_equal(g.mult, np.bincount(np.concatenate(kept), minlength=V))
        assert not res.near_rows.any()
    assert 40 not in seeds and 41 not in seeds                   # merged with token 3's group
    # a threshold placed exactly on a pair's cosine marks both of its rows as near ties
    c = oracle.asg_cosine(E, 0, 1)
    near = oracle.asg_build_exact(E, c, nthreads=2).near_rows
    assert near[0] and near[1]


# The similarity the kernels threshold is the dot product of unit vectors rounded to bfloat16
# (8 significant bits: every component off by at most 2^-9 of itself).  With unit vectors x, y
# and their roundings x(1+e), y(1+f), |e|, |f| <= 2^-9:
#   |sum x_k y_k ((1+e_k)(1+f_k) - 1)| <= (2^-8 + 2^-18) sum |x_k y_k| <= 2^-8 + 2^-18
# (Cauchy-Schwarz).  A membership can therefore differ from Eq. (1) only for a pair whose cosine
# lies within BF16_BAND of theta; the tie band of the bf16 form (1e-5) adds nothing visible.
BF16_BAND = 2.0 ** -8 + 2.0 ** -18


@pytest.mark.parametrize("name,V,d,theta,centres,sigma", [
    ("iid, C4-like (d = 1024, groups of tens)", 1536, 1024, 0.085, 0, 0),
    ("iid, small d", 1200, 64, 0.3, 0, 0),
    ("mixture, threshold inside the clusters' cosines (C5-like, 0.8)", 1500, 512, 0.8, 24, 0.5),
    ("mixture, C3-like", 1024, 768, 0.5, 16, 0.3),
    ("paper's range of theta (0.38 .. 0.45)", 1200, 32, 0.42, 0, 0),
])
def test_bf16_groups_differ_from_eq1_only_inside_the_rounding_band(name, V, d, theta, centres, sigma):
    """How far the bf16 form of the construction (what pcg_asg_normalize + pcg_asg_build compute,
    and what the oracle's asg_row mirrors) is from Eq. (1) on the unrounded embeddings: every
    membership that differs belongs to a pair whose exact cosine is within BF16_BAND of theta,
    and the count is reported."""
    E = embeddings(V, d, 31) if centres == 0 else embeddings(V, d, 31, centres, sigma)[0]
    unit = oracle.asg_normalize(E)
    S = numpy_cosines(E)
    exact = S > theta
    np.fill_diagonal(exact, True)
    U = bf16_to_f64(unit)
    rounded = (U @ U.T) > np.float64(np.float32(theta))
    np.fill_diagonal(rounded, True)
    diff = exact != rounded
    n_diff, n_mem = int(diff.sum()), int(exact.sum())
    worst = float(np.abs(S[diff] - theta).max()) if n_diff else 0.0
    worst_err = float(np.abs(U @ U.T - S)[~np.eye(V, dtype=bool)].max())
    print(f"asg bf16 vs Eq. (1) [{name}]: {n_mem} memberships, {n_diff} differ "
          f"({n_diff / max(1, n_mem):.2e}), farthest from theta {worst:.2e}, "
          f"largest |bf16 similarity - cosine| {worst_err:.2e}, band {BF16_BAND:.2e}")
    assert worst_err <= BF16_BAND
    assert (np.abs(S[diff] - theta) <= BF16_BAND).all()
    assert n_mem > V                                              # the threshold does form groups
    # the oracle's two row routines say the same as the two dense matrices
    for t in (0, V // 3, V - 1):
        np.testing.assert_array_equal(oracle.asg_row_exact(E, theta, t)[0], np.flatnonzero(exact[t]))
        np.testing.assert_array_equal(oracle.asg_row(unit, theta, t)[0], np.flatnonzero(rounded[t]))
