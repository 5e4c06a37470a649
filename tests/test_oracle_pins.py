"""Pins for the CPU oracle: everything here checks ``oracle/`` against something
other than itself -- library routines, closed forms, exact rational enumeration,
textbook special cases and sampling statistics.  No GPU needed."""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp
import scipy.special
import scipy.stats
import torch

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- helpers

def f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def to_bf16_bits(a):
    return oracle.bf16_bits(torch.from_numpy(f32(a)).to(torch.bfloat16))


def small_case(V=12, G=9, seed=0, K=2, sigma_t=1.5, sigma_d=1.0):
    rp, mem = W.random_groups(V, G, 1, 5, seed, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rng = np.random.default_rng(seed + 1000)
    tgt = f32(sigma_t * rng.standard_normal((1, K + 1, V)))
    dft = f32(tgt[:, :K] + sigma_d * rng.standard_normal((1, K, V)))
    return g, tgt, dft


def exact_probs(row, temperature=1.0):
    """The oracle's softmax output as exact rationals (the softmax itself is
    pinned to scipy separately); downstream arithmetic is then exact."""
    return [Fraction(float(x)) for x in oracle.softmax_row(row, temperature)]


def exact_group_probs(g, pr):
    return [sum((pr[t] / int(g.mult[t]) for t in g.members[g.row_ptr[k]:g.row_ptr[k + 1]]),
                Fraction(0)) for k in range(g.G)]


def chi2_p(counts, probs, n):
    probs = np.asarray(probs, dtype=np.float64)
    keep = probs * n >= 5
    obs = np.append(counts[keep], counts[~keep].sum())
    exp = np.append(probs[keep], probs[~keep].sum()) * n
    if exp[-1] == 0:
        obs, exp = obs[:-1], exp[:-1]
    return scipy.stats.chisquare(obs, exp * obs.sum() / exp.sum()).pvalue


# --------------------------------------------------------------------------- Philox

def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def test_uniform_layout():
    seed, offset = 0x1234567890ABCDEF, 0x0FEDCBA987654321
    for b, i in [(0, 0), (5, 3), (70000, 8)]:
        w = oracle.philox4x32_10([offset & 0xFFFFFFFF, offset >> 32, b, i],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        ua, ug, ut = oracle.uniforms(seed, offset, b, i)
        assert (ua, ug, ut) == tuple(float(int(x) >> 8) / 2 ** 24 for x in w[:3])
        for u in (ua, ug, ut):
            assert 0.0 <= u < 1.0 and np.float32(u) == u     # exact in fp32


def test_uniforms_are_uniform():
    us = np.array([oracle.uniforms(7, 3, b, i) for b in range(4000) for i in range(5)]).ravel()
    assert scipy.stats.kstest(us, "uniform").pvalue > 1e-3


# --------------------------------------------------------------------------- softmax

@pytest.mark.parametrize("tau", [1.0, 0.7, 0.8, 2.5])
def test_softmax_matches_library(tau):
    rng = np.random.default_rng(1)
    x = f32(4 * rng.standard_normal(1000))
    ref = scipy.special.softmax(x.astype(np.float64) / tau)
    np.testing.assert_allclose(oracle.softmax_row(x, tau), ref, rtol=1e-13, atol=0)
    bits = to_bf16_bits(x)
    xb = oracle.bf16_bits_to_f32(bits)
    ref = scipy.special.softmax(xb.astype(np.float64) / tau)
    np.testing.assert_allclose(oracle.softmax_row(bits, tau), ref, rtol=1e-13, atol=0)
    ref = torch.softmax(torch.from_numpy(xb).double() / tau, 0).numpy()
    np.testing.assert_allclose(oracle.softmax_row(bits, tau), ref, rtol=1e-12, atol=0)


def test_softmax_extremes():
    x = f32([-np.inf, 80.0, -80.0, 79.0, -np.inf])
    p = oracle.softmax_row(x)
    assert p[0] == 0 and p[4] == 0 and abs(p.sum() - 1) < 1e-15
    assert p[2] > 0                        # exp(-160) is representable in double
    np.testing.assert_allclose(p[1] / p[3], np.e, rtol=1e-14)
    x = f32([1e4, 1e4 - 1, -1e4])
    np.testing.assert_allclose(oracle.softmax_row(x)[:2], [1 / (1 + np.exp(-1)), 1 / (1 + np.e)])
    with pytest.raises(oracle.OracleError):
        oracle.softmax_row(f32([-np.inf, -np.inf]))
    with pytest.raises(oracle.OracleError):
        oracle.softmax_row(f32([0.0, np.nan]))
    with pytest.raises(oracle.OracleError):
        oracle.softmax_row(f32([0.0, 1.0]), 0.0)


# --------------------------------------------------------------------------- groups

def test_canonicalize_uncovered_tokens_become_singletons():
    # tokens 1 and 4 are in no group
    g = oracle.canonicalize(6, [0, 2, 4, 5], [0, 2, 2, 3, 5])
    assert g.G == 5
    assert g.row_ptr.tolist() == [0, 2, 4, 5, 6, 7]
    assert g.members.tolist() == [0, 2, 2, 3, 5, 1, 4]
    assert g.mult.tolist() == [1, 1, 2, 1, 1, 1]
    assert oracle.validate(g) == 0
    np.testing.assert_array_equal(oracle.count_mult(6, [0, 2, 4, 5], [0, 2, 2, 3, 5]),
                                  [1, 0, 2, 1, 0, 1])


def test_validate_rejects_bad_membership():
    good = oracle.canonicalize(4, [0, 2, 4], [0, 1, 2, 3])
    assert oracle.validate(good) == 0
    for rp, mem, mult in [
        ([1, 2, 4], [0, 1, 2, 3], [1, 1, 1, 1]),       # row_ptr[0] != 0
        ([0, 3, 2], [0, 1, 2, 3], [1, 1, 1, 1]),       # not monotone
        ([0, 2, 4], [0, 1, 2, 4], [1, 1, 1, 1]),       # member out of range
        ([0, 2, 4], [0, 1, 2, 3], [1, 2, 1, 1]),       # mult is not the entry count
        ([0, 2, 3], [0, 1, 2], [1, 1, 1, 0]),          # token 3 uncovered
    ]:
        bad = oracle.Groups(4, 2, np.array(rp, np.int32), np.array(mem, np.int32),
                            np.array(mult, np.int32))
        assert oracle.validate(bad) != 0
        with pytest.raises(oracle.OracleError):
            oracle.group_probs(bad, f32(np.zeros((1, 4))))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_group_probs_is_sparse_matvec_and_sums_to_one(dtype):
    V, G = 300, 260
    rp, mem = W.random_groups(V, G, 1, 12, seed=3, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rng = np.random.default_rng(5)
    x = f32(3 * rng.standard_normal((7, V)))
    arg = to_bf16_bits(x) if dtype == "bf16" else x
    xv = oracle.bf16_bits_to_f32(arg) if dtype == "bf16" else x
    tau = 0.8
    out = oracle.group_probs(g, arg, tau)
    # the weights matrix of Eq. (3): W[k, t] = 1{t in G_k} / N(t), columns sum to one (Eq. 2)
    rows = np.repeat(np.arange(g.G), np.diff(g.row_ptr))
    Wm = sp.csr_matrix((1.0 / g.mult[g.members], (rows, g.members)), shape=(g.G, V))
    np.testing.assert_allclose(np.asarray(Wm.sum(axis=0)).ravel(), 1.0, rtol=1e-14)
    prob = scipy.special.softmax(xv.astype(np.float64) / tau, axis=1)
    np.testing.assert_allclose(out, (Wm @ prob.T).T, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(out.sum(axis=1), 1.0, rtol=0, atol=1e-12)   # no renormalisation


def test_group_probs_partition_is_segment_sum():
    V = 64
    rng = np.random.default_rng(2)
    cuts = np.sort(rng.choice(np.arange(1, V), size=9, replace=False))
    rp = np.concatenate([[0], cuts, [V]]).astype(np.int32)
    g = oracle.canonicalize(V, rp, np.arange(V, dtype=np.int32))
    assert (g.mult == 1).all()
    x = f32(rng.standard_normal((3, V)))
    prob = scipy.special.softmax(x.astype(np.float64), axis=1)
    np.testing.assert_allclose(oracle.group_probs(g, x), np.add.reduceat(prob, rp[:-1], axis=1),
                               rtol=1e-13)


def test_group_probs_special_cases():
    V = 10
    x = f32(np.random.default_rng(0).standard_normal((2, V)))
    prob = scipy.special.softmax(x.astype(np.float64), axis=1)
    # one group holding every token
    g = oracle.canonicalize(V, [0, V], np.arange(V))
    np.testing.assert_allclose(oracle.group_probs(g, x), 1.0, atol=1e-15)
    # singleton groups reproduce the token distribution
    g = oracle.canonicalize(V, np.arange(V + 1), np.arange(V))
    np.testing.assert_allclose(oracle.group_probs(g, x), prob, rtol=1e-14)
    # no groups at all: every token becomes its own group
    g = oracle.canonicalize(V, [0], [])
    assert g.G == V
    np.testing.assert_allclose(oracle.group_probs(g, x), prob, rtol=1e-14)
    # a token listed twice in a group carries weight 2/m there
    g = oracle.canonicalize(3, [0, 3, 5], [0, 0, 1, 0, 2])
    assert g.mult.tolist() == [3, 1, 1]
    p3 = scipy.special.softmax(x[0, :3].astype(np.float64))
    np.testing.assert_allclose(oracle.group_probs(g, x[:1, :3])[0],
                               [2 * p3[0] / 3 + p3[1], p3[0] / 3 + p3[2]], rtol=1e-14)
    # swapped operand check: a permuted vocabulary permutes nothing in G but changes values
    g = oracle.canonicalize(4, [0, 2, 4], [0, 1, 2, 3])
    y = f32([[0.0, 0.0, 1.0, 1.0]])
    out = oracle.group_probs(g, y)[0]
    assert out[1] > out[0] and abs(out[1] / out[0] - np.e) < 1e-12


def test_membership_memory_arithmetic():
    # Sec. 2.2 "Complexity and memory": 65 536 tokens x ~140 members ~ 9.2 M indices,
    # ~37 MB as int32, ~19 MB as int16 -- the sizing the CSR layout is built for.
    n = 65536 * 140
    assert round(n / 1e6, 1) == 9.2
    assert round(n * 4 / 1e6) == 37 and round(n * 2 / 1e6) in (18, 19)


# --------------------------------------------------------------------------- accept test

def token_level_speculative_step(q, p, x, ua, ug):
    """Textbook speculative sampling for one position (Leviathan et al. /
    Chen et al.): accept x iff u < min(1, q/p); else draw from norm(max(0, q-p))."""
    if ua < min(1.0, q[x] / p[x]):
        return True, x
    r = np.maximum(0.0, q - p)
    c = np.cumsum(r)
    return False, int(np.searchsorted(c, ug * c[-1], side="right"))


def test_singleton_groups_reduce_to_token_level_speculative_sampling():
    V, K, B = 40, 3, 300
    g = oracle.canonicalize(V, np.arange(V + 1), np.arange(V))
    rng = np.random.default_rng(11)
    tgt = f32(2 * rng.standard_normal((B, K + 1, V)))
    dft = f32(tgt[:, :K] + rng.standard_normal((B, K, V)))
    ptok = rng.integers(0, V, size=(B, K)).astype(np.int32)
    res = oracle.verify(g, tgt, dft, ptok, ptok, seed=9, offset=4)
    n_rej = 0
    for b in range(B):
        exp_tok = []
        for i in range(K):
            q = scipy.special.softmax(tgt[b, i].astype(np.float64))
            p = scipy.special.softmax(dft[b, i].astype(np.float64))
            ua, ug, _ = oracle.uniforms(9, 4, b, i)
            ok, t = token_level_speculative_step(q, p, int(ptok[b, i]), ua, ug)
            exp_tok.append(t)
            if not ok:
                n_rej += 1
                break
        else:
            q = scipy.special.softmax(tgt[b, K].astype(np.float64))
            _, ug, _ = oracle.uniforms(9, 4, b, K)
            exp_tok.append(int(np.searchsorted(np.cumsum(q), ug * np.cumsum(q)[-1], side="right")))
        n = len(exp_tok)
        assert res.accept_len[b] == n - 1
        assert res.out_tokens[b, :n].tolist() == exp_tok
        assert res.out_groups[b, :n].tolist() == exp_tok
        assert (res.out_tokens[b, n:] == -1).all() and (res.out_groups[b, n:] == -1).all()
    assert 50 < n_rej < B


def test_accept_rate_is_one_minus_tv_and_beats_token_level():
    # Proof of the Proposition: Pr(accept) = sum_k min(D_k, T_k) = 1 - TV(T, D);
    # coarse-graining can only shrink the total variation.
    V, G, B = 60, 50, 200000
    rp, mem = W.random_groups(V, G, 2, 8, seed=21, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rng = np.random.default_rng(22)
    tgt = f32(2 * rng.standard_normal((1, 2, V)))
    dft = f32(tgt[:, :1] + rng.standard_normal((1, 1, V)))
    T = oracle.group_probs(g, tgt[0, :1])[0]
    D = oracle.group_probs(g, dft[0, :1])[0]
    q, p = oracle.softmax_row(tgt[0, 0]), oracle.softmax_row(dft[0, 0])
    tv_groups, tv_tokens = 0.5 * np.abs(T - D).sum(), 0.5 * np.abs(q - p).sum()
    assert tv_groups <= tv_tokens + 1e-15
    assert tv_groups < tv_tokens - 1e-3          # and it does shrink on a generic case
    # proposals by the coupling of Eq. (6)
    x = rng.choice(V, size=B, p=p)
    tok_ptr, tok_groups = W.reverse_index(V, g.row_ptr, g.members)
    k = tok_groups[tok_ptr[x] + (rng.random(B) * g.mult[x]).astype(np.int64)]
    res = oracle.verify(g, tgt, dft, x.reshape(B, 1), k.reshape(B, 1), seed=5, B=B,
                        tgt_batch_stride=0, dft_batch_stride=0, nthreads=8)
    rate = (res.accept_len == 1).mean()
    alpha = 1.0 - tv_groups
    assert abs(rate - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / B)
    # and the proposal marginal is D (Eq. 6)
    assert chi2_p(np.bincount(k, minlength=g.G), D, B) > 1e-3


def test_generator_proposals_follow_the_coupling():
    V, G, B = 48, 40, 150000
    rp, mem = W.random_groups(V, G, 2, 7, seed=31, cover=True)
    g = oracle.canonicalize(V, rp, mem)
    rng = np.random.default_rng(32)
    tau = 0.8
    row = f32(2 * rng.standard_normal(V))
    dft = torch.from_numpy(np.broadcast_to(row, (B, 1, V)).copy())
    tok, grp = W.proposals(dft, tau, g.row_ptr, g.members, rng)
    D = oracle.group_probs(g, row[None], tau)[0]
    p = oracle.softmax_row(row, tau)
    assert scipy.stats.chisquare(np.bincount(grp.ravel(), minlength=g.G), D * B).pvalue > 1e-3
    assert scipy.stats.chisquare(np.bincount(tok.ravel(), minlength=V), p * B).pvalue > 1e-3
    # the proposed token is a member of the proposed group
    for t, k in zip(tok.ravel()[:500], grp.ravel()[:500]):
        assert t in g.members[g.row_ptr[k]:g.row_ptr[k + 1]]


# --------------------------------------------------------------------------- exact enumeration

def run_one(g, tgt, dft, pgrp, ua, ug, ut, ptok=None, want_R=False):
    K = tgt.shape[1] - 1
    pgrp = np.asarray(pgrp, np.int32).reshape(1, K)
    ptok = pgrp * 0 if ptok is None else np.asarray(ptok, np.int32).reshape(1, K)
    return oracle.verify(g, tgt, dft, ptok, pgrp,
                         uniforms_explicit=(np.reshape(ua, (1, K)), np.reshape(ug, (1, K + 1)),
                                            np.reshape(ut, (1, K + 1))), want_R=want_R)


@pytest.mark.parametrize("seed", range(6))
def test_emitted_group_law_is_exactly_target_by_enumeration(seed):
    """Eq. (11) through the implementation's own thresholds, V <= 8, K = 1:
    sum over proposals of [accept mass on g] + [reject mass] x [residual bin of g] = T[g]."""
    V = 5 + seed % 4
    g, tgt, dft = small_case(V=V, G=4 + seed % 3, seed=seed, K=1)
    q, p = exact_probs(tgt[0, 0]), exact_probs(dft[0, 0])
    T, D = exact_group_probs(g, q), exact_group_probs(g, p)
    assert sum(T) == sum(q) and sum(D) == sum(p)           # Eq. (2) => no mass lost
    # proposal law by enumerating (x, k in S(x)) with weight p(x)/m(x)   (Eq. 6)
    prop = [Fraction(0)] * g.G
    for k in range(g.G):
        for t in g.members[g.row_ptr[k]:g.row_ptr[k + 1]]:
            prop[k] += p[t] / int(g.mult[t])
    assert prop == D
    law = np.zeros(g.G)
    n_reject_paths = 0
    for k in range(g.G):
        if D[k] == 0:
            continue
        res = run_one(g, tgt, dft, [k], [0.999999], [0.5, 0.5], [0.5, 0.5], want_R=True)
        r = min(1.0, res.T_prop[0, 0] / res.D_prop[0, 0])
        assert abs(res.T_prop[0, 0] - float(T[k])) < 1e-15 and abs(res.D_prop[0, 0] - float(D[k])) < 1e-15
        # the decision flips exactly at r
        if r < 1.0:
            assert run_one(g, tgt, dft, [k], [r * (1 - 1e-9)], [0.5] * 2, [0.5] * 2).accept_len[0] == 1
            assert run_one(g, tgt, dft, [k], [r * (1 + 1e-9)], [0.5] * 2, [0.5] * 2).accept_len[0] == 0
            assert res.accept_len[0] == 0
            bins = res.R_norm[0]
            n_reject_paths += 1
            # the residual bins are where the implementation says they are
            edges = np.concatenate([[0.0], np.cumsum(bins)])
            for gg in range(g.G):
                if bins[gg] > 1e-9:
                    for u in (edges[gg] + 1e-12, 0.5 * (edges[gg] + edges[gg + 1]), edges[gg + 1] - 1e-12):
                        rr = run_one(g, tgt, dft, [k], [0.999999], [u, 0.5], [0.5] * 2)
                        assert rr.out_groups[0, 0] == gg
                else:
                    assert bins[gg] == 0.0 or T[gg] - D[gg] < 1e-9
            law += float(D[k]) * (1 - r) * bins
            law[k] += float(D[k]) * r
        else:
            assert run_one(g, tgt, dft, [k], [1 - 2.0 ** -24], [0.5] * 2, [0.5] * 2).accept_len[0] == 1
            law[k] += float(D[k])
    assert n_reject_paths > 0
    np.testing.assert_allclose(law, [float(t) for t in T], rtol=0, atol=1e-14)
    # independent closed form of the residual bins (Eq. 8)
    pos = [max(Fraction(0), t - d) for t, d in zip(T, D)]
    np.testing.assert_allclose(bins, [float(x / sum(pos)) for x in pos], rtol=0, atol=1e-14)


@pytest.mark.parametrize("seed", range(3))
def test_two_positions_law_and_accept_length(seed):
    """K = 2: given an accept at position 1, position 2 is again exactly
    target-distributed; Pr(accept_len = j) = prod_{i<j} alpha_i (1 - alpha_j)."""
    g, tgt, dft = small_case(V=7, G=5, seed=40 + seed, K=2)
    T = [exact_group_probs(g, exact_probs(tgt[0, i])) for i in range(3)]
    D = [exact_group_probs(g, exact_probs(dft[0, i])) for i in range(2)]
    alpha = [float(sum(min(t, d) for t, d in zip(T[i], D[i]))) for i in range(2)]
    k0 = int(np.argmax([float(t / d) if d else 0 for t, d in zip(T[0], D[0])]))
    assert T[0][k0] >= D[0][k0]            # a first-position proposal that is always accepted
    law = np.zeros(g.G)
    acc2 = 0.0
    for k in range(g.G):
        if D[1][k] == 0:
            continue
        res = run_one(g, tgt, dft, [k0, k], [0.5, 0.999999], [0.5] * 3, [0.5] * 3, want_R=True)
        r = min(1.0, float(T[1][k] / D[1][k]))
        assert abs(min(1.0, res.T_prop[0, 1] / res.D_prop[0, 1]) - r) < 1e-14
        acc2 += float(D[1][k]) * r
        law[k] += float(D[1][k]) * r
        if r < 1:
            assert res.accept_len[0] == 1 and res.out_groups[0, 0] == k0
            law += float(D[1][k]) * (1 - r) * res.R_norm[0]
        else:
            assert res.accept_len[0] == 2
    np.testing.assert_allclose(law, [float(t) for t in T[1]], atol=1e-14)
    assert abs(acc2 - alpha[1]) < 1e-14
    # all accepted -> the bonus position draws from T of row K (residual with D = 0)
    kk = int(np.argmax([float(t / d) if d else 0 for t, d in zip(T[1], D[1])]))
    res = run_one(g, tgt, dft, [k0, kk], [0.5, 0.5], [0.5] * 3, [0.5] * 3, want_R=True)
    assert res.accept_len[0] == 2
    np.testing.assert_allclose(res.R_norm[0], [float(t) for t in T[2]], atol=1e-15)
    assert abs(res.res_S[0] - 1.0) < 1e-14


@pytest.mark.parametrize("seed", range(3))
def test_token_in_group_and_bonus_marginal_by_enumeration(seed):
    """Eq. (10) through the implementation: cells of the (u_grp, u_tok) square
    map to (group, token) with measure T[g] * q(t)/(m(t) T[g]); summed over
    groups that is q(t) -- the bonus token's marginal (Algorithm 1, last step)."""
    g, tgt, dft = small_case(V=8, G=6, seed=60 + seed, K=1)
    q = exact_probs(tgt[0, 1])
    T = exact_group_probs(g, q)
    D0 = exact_group_probs(g, exact_probs(dft[0, 0]))
    T0 = exact_group_probs(g, exact_probs(tgt[0, 0]))
    k0 = int(np.argmax([float(t / d) if d else 0 for t, d in zip(T0, D0)]))   # accepted for sure
    marg = [Fraction(0)] * g.V
    cumg = Fraction(0)
    for gg in range(g.G):
        if T[gg] == 0:
            continue
        ug_mid = float(cumg + T[gg] / 2)
        cumt = Fraction(0)
        for j in range(g.row_ptr[gg], g.row_ptr[gg + 1]):
            t = int(g.members[j])
            c = q[t] / int(g.mult[t])
            for ut in (float((cumt + c / 1000) / T[gg]), float((cumt + c / 2) / T[gg]),
                       float((cumt + c * 999 / 1000) / T[gg])):
                res = run_one(g, tgt, dft, [k0], [0.0], [0.5, ug_mid], [0.5, ut], ptok=[3])
                assert res.accept_len[0] == 1 and res.out_tokens[0, 0] == 3
                assert (res.out_groups[0, 1], res.out_tokens[0, 1]) == (gg, t)
            marg[t] += T[gg] * (c / T[gg])
            cumt += c
        assert cumt == T[gg]
        cumg += T[gg]
    assert marg == q


# --------------------------------------------------------------------------- sampling at scale

def test_chi_square_one_million_steps():
    """10^6 sampled steps: first emitted group ~ T_0; the second ~ T_1 given an
    accept; bonus token ~ q_K; token inside a resampled group follows Eq. (10)."""
    V, G, K, B = 48, 36, 2, 1_000_000
    rp, mem = W.random_groups(V, G, 2, 6, seed=71, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rng = np.random.default_rng(72)
    tau = 0.8
    tgt = f32(2 * rng.standard_normal((1, K + 1, V)))
    dft = f32(tgt[:, :K] + 0.7 * rng.standard_normal((1, K, V)))
    tok_ptr, tok_groups = W.reverse_index(V, g.row_ptr, g.members)
    ptok = np.empty((B, K), np.int32)
    pgrp = np.empty((B, K), np.int32)
    for i in range(K):
        p = oracle.softmax_row(dft[0, i], tau)
        x = rng.choice(V, size=B, p=p)
        ptok[:, i] = x
        pgrp[:, i] = tok_groups[tok_ptr[x] + (rng.random(B) * g.mult[x]).astype(np.int64)]
    res = oracle.verify(g, tgt, dft, ptok, pgrp, temperature=tau, seed=2024, offset=17, B=B,
                        tgt_batch_stride=0, dft_batch_stride=0, nthreads=8)
    T = oracle.group_probs(g, tgt[0], tau)
    assert chi2_p(np.bincount(res.out_groups[:, 0], minlength=g.G), T[0], B) > 1e-3
    sel = res.accept_len >= 1
    assert sel.sum() > 1e5
    assert chi2_p(np.bincount(res.out_groups[sel, 1], minlength=g.G), T[1], sel.sum()) > 1e-3
    bonus = res.accept_len == K
    assert bonus.sum() > 1e4
    qK = oracle.softmax_row(tgt[0, K], tau)
    assert chi2_p(np.bincount(res.out_tokens[bonus, K], minlength=V), qK, bonus.sum()) > 1e-3
    assert chi2_p(np.bincount(res.out_groups[bonus, K], minlength=g.G), T[K], bonus.sum()) > 1e-3
    # token inside the resampled group at a first-position reject
    rej = res.accept_len == 0
    q0 = oracle.softmax_row(tgt[0, 0], tau)
    gbig = int(np.bincount(res.out_groups[rej, 0]).argmax())
    seg = g.members[g.row_ptr[gbig]:g.row_ptr[gbig + 1]]
    cond = q0[seg] / g.mult[seg]
    cond /= cond.sum()
    toks = res.out_tokens[rej & (res.out_groups[:, 0] == gbig), 0]
    cnt = np.array([(toks == t).sum() for t in seg])
    assert cnt.sum() == len(toks) and len(toks) > 1000
    assert chi2_p(cnt, cond, len(toks)) > 1e-3
    # accept-length law
    D = oracle.group_probs(g, dft[0], tau)
    alpha = [1 - 0.5 * np.abs(T[i] - D[i]).sum() for i in range(K)]
    expect = np.array([1 - alpha[0], alpha[0] * (1 - alpha[1]), alpha[0] * alpha[1]])
    assert chi2_p(np.bincount(res.accept_len, minlength=K + 1), expect, B) > 1e-3
    # accepted positions hand the draft token through unchanged
    assert (res.out_tokens[sel, 0] == ptok[sel, 0]).all() and (res.out_groups[sel, 0] == pgrp[sel, 0]).all()


# --------------------------------------------------------------------------- edge cases and plumbing

def test_zero_draft_mass_and_zero_residual():
    V = 6
    g = oracle.canonicalize(V, [0, 2, 4, 6], [0, 1, 2, 3, 4, 5])
    big = 200.0
    # D[g0] underflows to exactly 0 while T[g0] > 0: accept for any u
    tgt = f32([[[0, 0, 0, 0, 0, 0], [0, 0, 0, 0, 0, 0]]])
    dft = f32([[[-np.inf, -np.inf, 0, 0, 0, 0]]])
    res = run_one(g, tgt, dft, [0], [1 - 2.0 ** -24], [0.5] * 2, [0.5] * 2)
    assert res.accept_len[0] == 1 and res.flags[0] & 2
    # T == D == 0 for the proposed group: reject, then a regular residual
    tgt2 = f32([[[-np.inf, -np.inf, 0, 0, 1, 1], [0] * 6]])
    res = run_one(g, tgt2, dft, [0], [0.0], [0.5] * 2, [0.5] * 2, want_R=True)
    assert res.accept_len[0] == 0 and res.R_norm[0, 0] == 0 and res.out_groups[0, 0] == 2
    # identical rows, proposed group with zero mass on both: residual total is 0 -> fall back to T
    res = run_one(g, f32([[dft[0, 0], [0] * 6]]), dft, [0], [0.0], [0.3, 0.5], [0.5] * 2, want_R=True)
    assert res.accept_len[0] == 0 and res.flags[0] & 1
    np.testing.assert_allclose(res.R_norm[0], [0, 0.5, 0.5])
    assert res.out_groups[0, 0] == 1
    # u = 0 picks the first group that has mass, never a zero-mass one
    res = run_one(g, f32([[dft[0, 0], [0] * 6]]), dft, [0], [0.0], [0.0, 0.0], [0.0, 0.0])
    assert res.out_groups[0, 0] == 1 and res.out_tokens[0, 0] == 2
    del big


def test_near_tie_flags():
    g, tgt, dft = small_case(V=9, G=6, seed=5, K=1)
    base = run_one(g, tgt, dft, [0], [0.5], [0.5] * 2, [0.5] * 2)
    k = next(k for k in range(g.G)
             if (r := run_one(g, tgt, dft, [k], [0.5], [0.5] * 2, [0.5] * 2)).T_prop[0, 0] < r.D_prop[0, 0])
    res = run_one(g, tgt, dft, [k], [0.5], [0.5] * 2, [0.5] * 2)
    r = res.T_prop[0, 0] / res.D_prop[0, 0]
    assert run_one(g, tgt, dft, [k], [r + 5e-7], [0.5] * 2, [0.5] * 2).near_acc[0, 0] == 1
    assert run_one(g, tgt, dft, [k], [r - 5e-7], [0.5] * 2, [0.5] * 2).near_acc[0, 0] == 1
    assert run_one(g, tgt, dft, [k], [r + 3e-6], [0.5] * 2, [0.5] * 2).near_acc[0, 0] == 0
    rej = run_one(g, tgt, dft, [k], [0.999999], [0.5] * 2, [0.5] * 2)
    assert rej.accept_len[0] == 0 and 0 < rej.res_lo[0] < rej.res_hi[0] < 1
    for ug, flag in [(rej.res_lo[0] + 4e-7, 1), (rej.res_hi[0] - 4e-7, 1),
                     (0.5 * (rej.res_lo[0] + rej.res_hi[0]), 0)]:
        rr = run_one(g, tgt, dft, [k], [0.999999], [ug, 0.5], [0.5] * 2)
        assert rr.out_groups[0, 0] == rej.out_groups[0, 0] and rr.near_grp[0] == flag
    assert base.near_grp[0] in (0, 1)


def test_strides_and_philox_wrapper_agree():
    V, G, K, B = 30, 20, 3, 16
    rp, mem = W.random_groups(V, G, 2, 6, seed=81, cover=True)
    g = oracle.canonicalize(V, rp, mem)
    rng = np.random.default_rng(82)
    tgt = f32(2 * rng.standard_normal((B, K + 1, V)))
    dfull = f32(tgt + rng.standard_normal((B, K + 1, V)))      # a [B, K+1, V] draft buffer
    ptok = rng.integers(0, V, (B, K)).astype(np.int32)
    pgrp = rng.integers(0, g.G, (B, K)).astype(np.int32)
    a = oracle.verify(g, tgt, dfull, ptok, pgrp, seed=3, offset=9)
    b = oracle.verify(g, tgt, np.ascontiguousarray(dfull[:, :K]), ptok, pgrp, seed=3, offset=9,
                      nthreads=4)
    ua = np.array([[oracle.uniforms(3, 9, s, i)[0] for i in range(K)] for s in range(B)])
    ug = np.array([[oracle.uniforms(3, 9, s, i)[1] for i in range(K + 1)] for s in range(B)])
    ut = np.array([[oracle.uniforms(3, 9, s, i)[2] for i in range(K + 1)] for s in range(B)])
    c = oracle.verify(g, tgt, dfull, ptok, pgrp, uniforms_explicit=(ua, ug, ut))
    for r in (b, c):
        np.testing.assert_array_equal(a.accept_len, r.accept_len)
        np.testing.assert_array_equal(a.out_tokens, r.out_tokens)
        np.testing.assert_array_equal(a.out_groups, r.out_groups)
    assert len(set(a.accept_len.tolist())) > 1
    # a different offset is a different stream
    d = oracle.verify(g, tgt, dfull, ptok, pgrp, seed=3, offset=10)
    assert (d.out_tokens != a.out_tokens).any()
    # emitted token is always a member of the emitted group; exactly accept_len+1 pairs
    for s in range(B):
        n = a.accept_len[s] + 1
        for i in range(n):
            k, t = a.out_groups[s, i], a.out_tokens[s, i]
            if i < n - 1:
                assert (t, k) == (ptok[s, i], pgrp[s, i])
            else:
                assert t in g.members[g.row_ptr[k]:g.row_ptr[k + 1]]
        assert (a.out_groups[s, n:] == -1).all()
