"""Pins for the oracle's general per-entry weights w_{k,t} (Sec. 2.2, Eq. 2 and Eq. 4; the equal
split of Eq. 3 is the special case every other pin file covers): weight validation, reverse
order, Eq. (4) as a sparse mat-vec, and -- with dyadic weights, so that every cell has an exact
rational size -- the laws of the proposal (Eq. 6), of one thinning trial (Eq. 9), of the emitted
group (Proposition) and of the token inside it (Eq. 10) by enumeration through the oracle's own
decisions; chi-square at scale for both residual samplers."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse

import oracle
import workloads as W
from test_oracle_pins import chi2_p, exact_probs, f32, small_case


def dyadic_weights(g, seed, denom=64, zero_rate=0.15):
    """Per token, non-negative multiples of 1/denom that sum to exactly 1 over its entries (some
    of them zero): exact in fp32, so every cell of an enumeration is an exact rational."""
    rng = np.random.default_rng(seed)
    w = np.zeros(g.nnz, np.float32)
    entries = [[] for _ in range(g.V)]
    for j, t in enumerate(g.members):
        entries[t].append(j)
    for t in range(g.V):
        n = len(entries[t])
        parts = rng.multinomial(denom - 1, np.ones(n) / n) if n > 1 else np.array([denom - 1])
        if n > 1 and rng.random() < zero_rate:
            parts[rng.integers(n)] = 0
            parts[np.argmax(parts)] += denom - 1 - parts.sum()
        parts[np.argmax(parts)] += 1
        assert parts.sum() == denom and (parts >= 0).all()
        w[entries[t]] = parts / denom
    return w


def ew(g, j):
    return Fraction(float(g.weights[j]))


def exact_T(g, pr):
    return [sum((pr[g.members[j]] * ew(g, j) for j in range(g.row_ptr[k], g.row_ptr[k + 1])), Fraction(0))
            for k in range(g.G)]


def weighted_case(V, G, seed, K=1):
    g, tgt, dft = small_case(V=V, G=G, seed=seed, K=K)
    return oracle.with_weights(g, dyadic_weights(g, seed)), tgt, dft


def test_weight_validation_and_reverse_order():
    g, _, _ = small_case(V=30, G=20, seed=3)
    w = W.random_weights(g.V, g.members, 1)
    assert oracle.validate_weights(g, w) == 0
    bad = w.copy(); bad[0] = -bad[0]
    assert oracle.validate_weights(g, bad) != 0
    bad = w.copy(); bad[5] *= 1.01
    assert oracle.validate_weights(g, bad) != 0
    bad = w.copy(); bad[7] = np.nan
    assert oracle.validate_weights(g, bad) != 0
    gw = oracle.with_weights(g, w)
    tok_ptr, tok_groups = oracle.reverse_index(g)
    # entry e of token t in reverse order is the e-th CSR entry (ascending position) holding t
    for t in range(g.V):
        pos = [j for j in range(g.nnz) if g.members[j] == t]
        np.testing.assert_array_equal(gw.tok_weights[tok_ptr[t]:tok_ptr[t + 1]], w[pos])
        owner = np.searchsorted(g.row_ptr, pos, side="right") - 1
        np.testing.assert_array_equal(tok_groups[tok_ptr[t]:tok_ptr[t + 1]], owner)
    with pytest.raises(oracle.OracleError):
        oracle.with_weights(g, bad)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_group_probs_with_weights_is_the_sparse_matvec_of_eq_4(dtype):
    V, G = 700, 500
    rp, mem = W.random_groups(V, G, 1, 12, seed=2, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    w = W.random_weights(g.V, g.members, 5)
    gw = oracle.with_weights(g, w)
    rng = np.random.default_rng(6)
    x = f32(3 * rng.standard_normal((4, V)))
    if dtype == "bf16":
        import torch
        t = torch.from_numpy(x).to(torch.bfloat16)
        arg, vals = oracle.bf16_bits(t), t.float().numpy()
    else:
        arg, vals = x, x
    got = oracle.group_probs(gw, arg, 0.9)
    rows = np.repeat(np.arange(g.G), np.diff(g.row_ptr))
    Wm = scipy.sparse.csr_matrix((w.astype(np.float64), (rows, g.members)), shape=(g.G, V))
    np.testing.assert_allclose(np.asarray(Wm.sum(axis=0)).ravel(), 1.0, atol=1e-6)      # Eq. (2)
    for r in range(4):
        q = oracle.softmax_row(vals[r], 0.9)
        np.testing.assert_allclose(got[r], Wm @ q, rtol=1e-13, atol=1e-18)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, atol=1e-6)
    # the equal split written out as weights gives the equal-split result
    eq = oracle.with_weights(g, (1.0 / g.mult[g.members]).astype(np.float32))
    np.testing.assert_allclose(oracle.group_probs(eq, arg, 0.9), oracle.group_probs(g, arg, 0.9), rtol=2e-7)


@pytest.mark.parametrize("seed", range(4))
def test_proposal_label_law_with_weights_by_enumeration(seed):
    """Cells (token bin) x (entry slice of the token's weight CDF): the label lands on group k
    with mass D[k] = sum_t p(t) w_{k,t} exactly (Eq. 6)."""
    g, _, dft = weighted_case(8, 6, 50 + seed)
    rev = oracle.reverse_index(g)
    tok_ptr, tok_groups = rev
    p = exact_probs(dft[0, 0])
    total = sum(p, Fraction(0))
    D = exact_T(g, p)
    mass = [Fraction(0)] * g.G
    cum = Fraction(0)
    for x in range(g.V):
        ux = float((cum + p[x] / 2) / total)
        c = Fraction(0)
        for e in range(int(g.mult[x])):
            we = Fraction(float(g.tok_weights[tok_ptr[x] + e]))
            if we > 0:
                lo, hi = int(c * 2 ** 24), int((c + we) * 2 ** 24)          # k24 cells of entry e
                for k24 in (lo, (lo + hi) // 2, hi - 1):
                    r = oracle.propose(g, rev, dft, u_x=[[ux]], k24=[[k24]])
                    assert (int(r.tokens[0, 0]), int(r.groups[0, 0])) == (x, int(tok_groups[tok_ptr[x] + e]))
                mass[int(tok_groups[tok_ptr[x] + e])] += p[x] / total * Fraction(hi - lo, 2 ** 24)
            c += we
        assert c == 1
        cum += p[x]
    assert mass == [d / total for d in D]


@pytest.mark.parametrize("seed", range(4))
def test_emitted_group_law_with_weights_by_enumeration(seed):
    """Eq. (11) with general weights, K = 1, through the oracle's own ratio and residual bins."""
    g, tgt, dft = weighted_case(6 + seed % 3, 5, 60 + seed)
    q, p = exact_probs(tgt[0, 0]), exact_probs(dft[0, 0])
    T, D = exact_T(g, q), exact_T(g, p)
    assert sum(T) == sum(q) and sum(D) == sum(p)              # Eq. (2): no mass lost
    law = np.zeros(g.G)
    rejects = 0
    half = np.full((1, 2), 0.5)
    for k in range(g.G):
        if D[k] == 0:
            continue
        res = oracle.verify(g, tgt, dft, [[0]], [[k]], want_R=True,
                            uniforms_explicit=(np.array([[1 - 2.0 ** -24]]), half, half))
        assert abs(res.T_prop[0, 0] - float(T[k])) < 1e-15 and abs(res.D_prop[0, 0] - float(D[k])) < 1e-15
        r = min(1.0, float(T[k] / D[k]))
        if r < 1.0:
            for ua, want in ((r * (1 - 1e-9), 1), (r * (1 + 1e-9), 0)):
                got = oracle.verify(g, tgt, dft, [[0]], [[k]], uniforms_explicit=(np.array([[ua]]), half, half))
                assert got.accept_len[0] == want
            bins = res.R_norm[0]
            pos = [max(Fraction(0), t - d) for t, d in zip(T, D)]
            np.testing.assert_allclose(bins, [float(x / sum(pos)) for x in pos], rtol=0, atol=1e-14)   # Eq. (8)
            law += float(D[k]) * (1 - r) * bins
            rejects += 1
        law[k] += float(D[k]) * r
    assert rejects > 0
    np.testing.assert_allclose(law, [float(t) for t in T], rtol=0, atol=1e-14)


@pytest.mark.parametrize("seed", range(3))
def test_one_thinning_trial_with_weights_by_enumeration(seed):
    """Cells (token y) x (entry slice by y's weights) x (accept interval): the mass on group k is
    [T_k - D_k]_+ exactly, and the token inside an accepted group follows q(t) w_{k,t} / T_k."""
    g, tgt, dft = weighted_case(7, 5, 90 + seed)
    rev = oracle.reverse_index(g)
    tok_ptr, tok_groups = rev
    qf, pf = oracle.softmax_row(tgt[0, 0]), oracle.softmax_row(dft[0, 0])
    q, p = exact_probs(tgt[0, 0]), exact_probs(dft[0, 0])
    T, D = exact_T(g, q), exact_T(g, p)
    mass = [Fraction(0)] * g.G
    cum = Fraction(0)
    for y in range(g.V):
        uy = float(cum + q[y] / 2)
        c = Fraction(0)
        for e in range(int(g.mult[y])):
            we = Fraction(float(g.tok_weights[tok_ptr[y] + e]))
            if we > 0:
                k24 = int((c + we / 2) * 2 ** 24)
                k = int(tok_groups[tok_ptr[y] + e])
                tr = oracle.thin_trial(g, rev, qf, pf, uy, k24, 0.5, 0.5)
                assert (tr.y, tr.group) == (y, k)
                assert abs(tr.T - float(T[k])) < 1e-15 and abs(tr.D - float(D[k])) < 1e-15
                a = max(Fraction(0), 1 - D[k] / T[k])
                if a > 0:
                    assert oracle.thin_trial(g, rev, qf, pf, uy, k24, float(a) * (1 - 1e-9), 0.5).accepted == 1
                    assert oracle.thin_trial(g, rev, qf, pf, uy, k24, float(a) * (1 + 1e-9), 0.5).accepted == 0
                mass[k] += q[y] * we * a
                # Eq. (10): the token bins inside group k
                lo = Fraction(0)
                for j in range(g.row_ptr[k], g.row_ptr[k + 1]):
                    cj = q[g.members[j]] * ew(g, j)
                    if cj > 0:
                        ut = float((lo + cj / 2) / T[k])
                        assert oracle.thin_trial(g, rev, qf, pf, uy, k24, 0.0, ut).token == g.members[j]
                    lo += cj
                assert lo == T[k]
            c += we
        cum += q[y]
    assert mass == [max(Fraction(0), t - d) for t, d in zip(T, D)]


def test_weighted_samplers_at_scale_chi_square():
    """300 000 sequences sharing one set of rows, arbitrary (non-dyadic) weights: proposals by the
    oracle's coupling, then both residual samplers; first emitted group ~ T, rejected groups ~ R/S
    for both, token inside a resampled group by Eq. (10), bonus token ~ q_K with its group ~ T_K."""
    V, G, K, B, tau = 48, 36, 1, 300_000, 0.8
    rp, mem = W.random_groups(V, G, 2, 6, seed=71, cover=False)
    g0 = oracle.canonicalize(V, rp, mem)
    g = oracle.with_weights(g0, W.random_weights(g0.V, g0.members, 9))
    rev = oracle.reverse_index(g)
    rng = np.random.default_rng(5)
    tgt = f32(2 * rng.standard_normal((1, K + 1, V)))
    dft = f32(tgt[:, :K] + 0.7 * rng.standard_normal((1, K, V)))
    kw = dict(temperature=tau, seed=12, offset=5, B=B, nthreads=8)
    pr = oracle.propose(g, rev, dft, dft_batch_stride=0, **kw)
    T, D = oracle.group_probs(g, tgt[0], tau), oracle.group_probs(g, dft[0], tau)
    assert chi2_p(np.bincount(pr.groups[:, 0], minlength=g.G), D[0], B) > 1e-3
    kw.update(tgt_batch_stride=0, dft_batch_stride=0)
    enum = oracle.verify(g, tgt, dft, pr.tokens, pr.groups, **kw)
    thin = oracle.verify_thinning(g, rev, tgt, dft, pr.tokens, pr.groups, max_trials=65520, **kw)
    np.testing.assert_array_equal(thin.accept_len, enum.accept_len)
    R = np.maximum(0.0, T[0] - D[0])
    rej = enum.accept_len == 0
    assert rej.sum() > 5e4
    for res in (enum, thin):
        assert chi2_p(np.bincount(res.out_groups[:, 0], minlength=g.G), T[0], B) > 1e-3
        assert chi2_p(np.bincount(res.out_groups[rej, 0], minlength=g.G), R / R.sum(), rej.sum()) > 1e-3
        cnt = np.bincount(res.out_groups[rej, 0], minlength=g.G) * (np.diff(g.row_ptr) >= 3)
        k = int(cnt.argmax())
        seg = slice(g.row_ptr[k], g.row_ptr[k + 1])
        q0 = oracle.softmax_row(tgt[0, 0], tau)
        cond = q0[g.members[seg]] * g.weights[seg]
        toks = res.out_tokens[rej & (res.out_groups[:, 0] == k), 0]
        assert chi2_p(np.array([(toks == t).sum() for t in g.members[seg]]), cond / cond.sum(), len(toks)) > 1e-3
        bon = res.accept_len == K
        qK = oracle.softmax_row(tgt[0, K], tau)
        assert chi2_p(np.bincount(res.out_tokens[bon, K], minlength=V), qK, bon.sum()) > 1e-3
        assert chi2_p(np.bincount(res.out_groups[bon, K], minlength=g.G), T[K], bon.sum()) > 1e-3
    tv = 0.5 * np.abs(T[0] - D[0]).sum()
    tr = thin.trials[rej].astype(np.float64)
    assert abs(tr.mean() - 1 / tv) < 4 * np.sqrt((1 - tv) / tv ** 2 / rej.sum())
