"""Pins for the oracle's thinning sampler (Sec. 2.2 "Residual sampling via thinning", Eq. 9):
reverse index against numpy, one trial's law by exact enumeration of its (token, group) cells,
the emitted law against the enumerated residual (itself pinned in test_oracle_pins.py), the
expected number of trials 1 / TV, and the bonus position."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats

import oracle
import workloads as W
from test_oracle_pins import chi2_p, exact_group_probs, exact_probs, f32, small_case


def test_reverse_index_matches_numpy_and_counts():
    V, G = 300, 200
    rp, mem = W.random_groups(V, G, 1, 9, seed=1, cover=False)
    mem = mem.copy()
    mem[1] = mem[0]                                   # a token twice in one group
    g = oracle.canonicalize(V, rp, mem)
    tok_ptr, tok_groups = oracle.reverse_index(g)
    want_ptr, want_groups = W.reverse_index(V, g.row_ptr, g.members)
    np.testing.assert_array_equal(tok_ptr, want_ptr)
    np.testing.assert_array_equal(tok_groups, want_groups)
    np.testing.assert_array_equal(np.diff(tok_ptr), g.mult)          # N(t) = |S(t)| with repeats
    for t in (0, 17, V - 1):
        for k in tok_groups[tok_ptr[t]:tok_ptr[t + 1]]:
            assert t in g.members[g.row_ptr[k]:g.row_ptr[k + 1]]


def test_trial_uniform_layout():
    seed, offset = 0xABCDEF0123456789, 77
    for b, i, trial in [(0, 0, 0), (9, 3, 5), (70000, 64, 65534)]:
        w = oracle.philox4x32_10([offset & 0xFFFFFFFF, offset >> 32, b, i | ((trial + 1) << 16)],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        uy, k24, ua, ut = oracle.trial_uniforms(seed, offset, b, i, trial)
        assert (uy, k24, ua, ut) == (float(int(w[0]) >> 8) / 2 ** 24, int(w[1]) >> 8,
                                     float(int(w[2]) >> 8) / 2 ** 24, float(int(w[3]) >> 8) / 2 ** 24)
    # the accept block of a position (trial bits zero) is a different block
    assert oracle.trial_uniforms(1, 2, 3, 4, 0)[0] != oracle.uniforms(1, 2, 3, 4)[0]


@pytest.mark.parametrize("seed", range(4))
def test_one_trial_emits_the_positive_part_of_T_minus_D(seed):
    """Enumerate the cells of one trial: token y (length q(y)), membership entry of y (1/N(y) each),
    accept interval [0, a(K)).  Mass that lands on group k must be [T_k - D_k]_+ exactly, and the
    total acceptance mass TV(T, D) -- through the implementation's own decisions."""
    g, tgt, dft = small_case(V=7, G=5, seed=80 + seed, K=1)
    rev = oracle.reverse_index(g)
    qf, pf = oracle.softmax_row(tgt[0, 0]), oracle.softmax_row(dft[0, 0])
    q, p = exact_probs(tgt[0, 0]), exact_probs(dft[0, 0])
    T, D = exact_group_probs(g, q), exact_group_probs(g, p)
    mass = [Fraction(0)] * g.G
    cum = Fraction(0)
    for y in range(g.V):
        if q[y] == 0:
            continue
        uy = float(cum + q[y] / 2)
        n = int(g.mult[y])
        for e in range(n):
            k24 = ((2 * e + 1) << 24) // (2 * n)               # middle of entry e's slice
            tr = oracle.thin_trial(g, rev, qf, pf, uy, k24, 0.5, 0.5)
            k = int(rev[1][rev[0][y] + e])
            assert (tr.y, tr.group) == (y, k)
            assert abs(tr.T - float(T[k])) < 1e-15 and abs(tr.D - float(D[k])) < 1e-15
            a = max(Fraction(0), 1 - D[k] / T[k])
            if a > 0:    # the decision flips at a (a < 1 always: D > 0 on these rows)
                assert oracle.thin_trial(g, rev, qf, pf, uy, k24, float(a) * (1 - 1e-9), 0.5).accepted == 1
                assert oracle.thin_trial(g, rev, qf, pf, uy, k24, float(a) * (1 + 1e-9), 0.5).accepted == 0
            else:
                assert oracle.thin_trial(g, rev, qf, pf, uy, k24, 0.0, 0.5).accepted == 0
            mass[k] += q[y] / n * a
        cum += q[y]
    pos = [max(Fraction(0), t - d) for t, d in zip(T, D)]
    assert mass == pos                                          # Eq. (8) per trial, exactly
    # total acceptance mass = TV(T, D) (exact up to sum q != sum p in the last bit)
    assert abs(float(sum(mass)) - float(sum(abs(t - d) for t, d in zip(T, D)) / 2)) < 1e-15
    # bin edges of the token draw are where the implementation says they are
    edges = np.cumsum([float(x) for x in q])
    for y in range(g.V - 1):
        if q[y] > 1e-6 and q[y + 1] > 1e-6:
            assert oracle.thin_trial(g, rev, qf, pf, edges[y] - 1e-9, 0, 0.5, 0.5).y == y
            assert oracle.thin_trial(g, rev, qf, pf, edges[y] + 1e-9, 0, 0.5, 0.5).y == y + 1
            assert oracle.thin_trial(g, rev, qf, pf, edges[y] + 5e-7, 0, 0.5, 0.5).near & 1
            assert not oracle.thin_trial(g, rev, qf, pf, edges[y] + q_mid(q, y + 1), 0, 0.5, 0.5).near & 1


def q_mid(q, y):
    return float(q[y]) / 2


def test_thinning_matches_the_enumerated_residual_in_law():
    """Emitted group ~ R / S (the enumerated residual of the pinned oracle), token inside it by
    Eq. (10), E[trials] = 1 / TV(T, D); accept lengths identical to the enumerated path."""
    V, G, K, B = 48, 36, 1, 300_000
    rp, mem = W.random_groups(V, G, 2, 6, seed=71, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rev = oracle.reverse_index(g)
    rng = np.random.default_rng(5)
    tau = 0.8
    tgt = f32(2 * rng.standard_normal((1, K + 1, V)))
    dft = f32(tgt[:, :K] + 0.7 * rng.standard_normal((1, K, V)))
    p = oracle.softmax_row(dft[0, 0], tau)
    x = rng.choice(V, size=B, p=p)
    k = rev[1][rev[0][x] + (rng.random(B) * g.mult[x]).astype(np.int64)]
    kw = dict(temperature=tau, seed=11, offset=5, B=B, tgt_batch_stride=0, dft_batch_stride=0, nthreads=8)
    thin = oracle.verify_thinning(g, rev, tgt, dft, x.reshape(B, 1), k.reshape(B, 1), **kw)
    enum = oracle.verify(g, tgt, dft, x.reshape(B, 1), k.reshape(B, 1), want_R=False, **kw)
    np.testing.assert_array_equal(thin.accept_len, enum.accept_len)
    acc = thin.accept_len == 1
    np.testing.assert_array_equal(thin.out_groups[acc, 0], enum.out_groups[acc, 0])
    rej = ~acc
    assert rej.sum() > 5e4 and (thin.trials[acc] == 0).all() and (thin.trials[rej] >= 1).all()
    T = oracle.group_probs(g, tgt[0], tau)
    D = oracle.group_probs(g, dft[0], tau)
    R = np.maximum(0.0, T[0] - D[0])
    tv = 0.5 * np.abs(T[0] - D[0]).sum()
    assert chi2_p(np.bincount(thin.out_groups[rej, 0], minlength=g.G), R / R.sum(), rej.sum()) > 1e-3
    # geometric number of trials with success probability TV
    tr = thin.trials[rej].astype(np.float64)
    assert abs(tr.mean() - 1 / tv) < 4 * np.sqrt((1 - tv) / tv ** 2 / rej.sum())
    assert abs((tr == 1).mean() - tv) < 4 * np.sqrt(tv * (1 - tv) / rej.sum())
    # token inside the most frequent resampled group
    q0 = oracle.softmax_row(tgt[0, 0], tau)
    cnt = np.bincount(thin.out_groups[rej, 0], minlength=g.G) * (np.diff(g.row_ptr) >= 3)
    gbig = int(cnt.argmax())
    assert cnt[gbig] > 2000
    seg = g.members[g.row_ptr[gbig]:g.row_ptr[gbig + 1]]
    cond = q0[seg] / g.mult[seg]
    toks = thin.out_tokens[rej & (thin.out_groups[:, 0] == gbig), 0]
    assert chi2_p(np.array([(toks == t).sum() for t in seg]), cond / cond.sum(), len(toks)) > 1e-3
    # bonus position: token ~ q_K, group uniform over the groups that hold it (Eq. 6)
    bon = thin.accept_len == K
    qK = oracle.softmax_row(tgt[0, K], tau)
    assert chi2_p(np.bincount(thin.out_tokens[bon, K], minlength=V), qK, bon.sum()) > 1e-3
    assert chi2_p(np.bincount(thin.out_groups[bon, K], minlength=g.G), T[K], bon.sum()) > 1e-3
    for t, kk in zip(thin.out_tokens[bon, K][:300], thin.out_groups[bon, K][:300]):
        assert t in g.members[g.row_ptr[kk]:g.row_ptr[kk + 1]]


def test_thinning_trial_cap_and_structure():
    g, tgt, dft = small_case(V=9, G=6, seed=3, K=2)
    rev = oracle.reverse_index(g)
    B = 400
    rng = np.random.default_rng(0)
    ptok = rng.integers(0, g.V, (B, 2)).astype(np.int32)
    pgrp = rng.integers(0, g.G, (B, 2)).astype(np.int32)
    a = oracle.verify_thinning(g, rev, tgt, dft, ptok, pgrp, seed=4, B=B, tgt_batch_stride=0,
                               dft_batch_stride=0)
    capped = oracle.verify_thinning(g, rev, tgt, dft, ptok, pgrp, seed=4, B=B, tgt_batch_stride=0,
                                    dft_batch_stride=0, max_trials=1)
    assert (capped.trials <= 1).all() and (capped.flags[a.trials > 1] & 2).all()
    assert not (a.flags & 2).any()
    one = a.trials <= 1
    np.testing.assert_array_equal(a.out_groups[one], capped.out_groups[one])
    for s in range(B):
        n = a.accept_len[s]
        assert (a.out_tokens[s, :n] == ptok[s, :n]).all() and (a.out_groups[s, n + 1:] == -1).all()
        kk, t = a.out_groups[s, n], a.out_tokens[s, n]
        assert t in g.members[g.row_ptr[kk]:g.row_ptr[kk + 1]]
