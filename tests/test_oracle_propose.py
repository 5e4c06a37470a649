"""Pins for the oracle's draft-side proposal coupling (Sec. 2.2 "Proposal coupling and
acceptance", Eq. 6): draw layout against the known-answer-pinned Philox, the token draw against
numpy's searchsorted on a library softmax, the group-label law Pr(K = k) = D[k] by exact
enumeration of the (token bin, membership entry) cells, chi-square at scale, and the whole chain
proposal -> verification emitting the target's group law (Proposition)."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
import workloads as W
from test_oracle_pins import chi2_p, exact_group_probs, exact_probs, f32, small_case


def test_proposal_draw_layout_and_independence_of_the_verifier_blocks():
    seed, offset = 0x0123456789ABCDEF, (5 << 32) | 9
    for b, i in [(0, 0), (9, 3), (70000, 64)]:
        w = oracle.philox4x32_10([offset & 0xFFFFFFFF, offset >> 32, b, i | 0xFFFF0000],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        ux, k24 = oracle.propose_uniforms(seed, offset, b, i)
        assert (ux, k24) == (float(int(w[0]) >> 8) / 2 ** 24, int(w[1]) >> 8)
    # the counter differs from the accept block (trial field 0) and from every thinning trial
    # (trial field 1 .. 65520) of the same position
    ux = oracle.propose_uniforms(1, 2, 3, 4)[0]
    assert ux != oracle.uniforms(1, 2, 3, 4)[0]
    assert all(ux != oracle.trial_uniforms(1, 2, 3, 4, t)[0] for t in (0, 1, 65518, 65519))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_token_and_group_against_searchsorted(dtype):
    V, G, B, K, tau = 500, 300, 40, 3, 0.8
    rp, mem = W.random_groups(V, G, 1, 9, seed=3, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rev = oracle.reverse_index(g)
    rng = np.random.default_rng(4)
    logits = f32(3 * rng.standard_normal((B, K, V)))
    logits[0, 0, 100:200] = -np.inf
    if dtype == "bf16":
        import torch
        t = torch.from_numpy(logits).to(torch.bfloat16)
        arg, vals = oracle.bf16_bits(t), t.float().numpy().astype(np.float64)
    else:
        arg, vals = logits, logits.astype(np.float64)
    u = rng.integers(0, 1 << 24, size=(B, K)) / 2 ** 24
    k24 = rng.integers(0, 1 << 24, size=(B, K)).astype(np.uint32)
    u[1, 0], u[1, 1] = 0.0, (2 ** 24 - 1) / 2 ** 24
    got = oracle.propose(g, rev, arg, temperature=tau, u_x=u, k24=k24)
    tok_ptr, tok_groups = rev
    for b in range(B):
        for i in range(K):
            p = scipy.special.softmax(vals[b, i] / tau)
            cum = np.cumsum(p)
            x = int(np.searchsorted(cum, u[b, i] * cum[-1], side="right"))
            if got.near[b, i]:
                assert abs(int(got.tokens[b, i]) - x) <= 1
                continue
            assert int(got.tokens[b, i]) == x, (b, i)
            n = int(tok_ptr[x + 1] - tok_ptr[x])
            assert int(got.groups[b, i]) == int(tok_groups[tok_ptr[x] + (int(k24[b, i]) * n) // 2 ** 24])
            assert x in g.members[g.row_ptr[got.groups[b, i]]:g.row_ptr[got.groups[b, i] + 1]]
    assert not np.isin(got.tokens[0, 0], np.arange(100, 200))       # masked tokens are never proposed
    assert got.near.sum() <= 2


@pytest.mark.parametrize("seed", range(4))
def test_group_label_law_equals_draft_group_distribution_by_enumeration(seed):
    """Every (token bin, membership entry) cell is sent through the oracle; the mass landing on
    group k is D[k] up to the 2^-24 granularity of the entry pick."""
    g, _, dft = small_case(V=8, G=6, seed=40 + seed, K=1)
    rev = oracle.reverse_index(g)
    tok_ptr, tok_groups = rev
    p = exact_probs(dft[0, 0])
    total = sum(p, Fraction(0))
    D = exact_group_probs(g, p)
    mass = [Fraction(0)] * g.G
    cum = Fraction(0)
    for x in range(g.V):
        n = int(g.mult[x])
        ux = float((cum + p[x] / 2) / total)              # middle of the token's bin
        for j in range(n):
            lo, hi = -(-j * 2 ** 24 // n), -(-(j + 1) * 2 ** 24 // n)      # k24 cells of entry j
            for k24 in (lo, (lo + hi) // 2, hi - 1):
                r = oracle.propose(g, rev, dft, u_x=[[ux]], k24=[[k24]])
                assert int(r.tokens[0, 0]) == x and int(r.groups[0, 0]) == int(tok_groups[tok_ptr[x] + j])
            mass[int(tok_groups[tok_ptr[x] + j])] += p[x] / total * Fraction(hi - lo, 2 ** 24)
        cum += p[x]
    assert sum(mass) == 1
    for k in range(g.G):
        assert abs(mass[k] - D[k] / total) <= Fraction(1, 2 ** 24)
    np.testing.assert_allclose([float(m) for m in mass], oracle.group_probs(g, dft[0])[0], atol=1e-7)


def test_proposal_marginals_chi_square_and_position_offset():
    V, G, Bs, tau = 60, 45, 1 << 20, 0.9
    rp, mem = W.random_groups(V, G, 1, 7, seed=11, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rev = oracle.reverse_index(g)
    rng = np.random.default_rng(12)
    dft = f32(1.5 * rng.standard_normal((1, 2, V)))
    r = oracle.propose(g, rev, dft, temperature=tau, seed=7, offset=3, B=Bs, dft_batch_stride=0, nthreads=8)
    for i in range(2):
        p = oracle.softmax_row(dft[0, i], tau)
        D = oracle.group_probs(g, dft[0], tau)[i]
        assert chi2_p(np.bincount(r.tokens[:, i], minlength=V), p, Bs) > 1e-3
        assert chi2_p(np.bincount(r.groups[:, i], minlength=g.G), D, Bs) > 1e-3
    # positions are independent draws
    assert (r.tokens[:, 0] == r.tokens[:, 1]).mean() < 0.5
    # pos0 names the position of row 0: a one-row call at pos0 = 1 repeats column 1
    one = oracle.propose(g, rev, dft[:, 1:2], temperature=tau, seed=7, offset=3, pos0=1, B=4096,
                         dft_batch_stride=0)
    np.testing.assert_array_equal(one.tokens[:, 0], r.tokens[:4096, 1])
    np.testing.assert_array_equal(one.groups[:, 0], r.groups[:4096, 1])


def test_chain_propose_then_verify_emits_the_target_group_law():
    """Proposals and verification under the same (seed, offset): the first emitted group follows
    T (Proposition), which also needs the proposal draws to be independent of the accept draws."""
    V, G, Bs, K = 40, 30, 1 << 19, 2
    rp, mem = W.random_groups(V, G, 2, 6, seed=21, cover=False)
    g = oracle.canonicalize(V, rp, mem)
    rev = oracle.reverse_index(g)
    rng = np.random.default_rng(22)
    tgt = f32(2 * rng.standard_normal((1, K + 1, V)))
    dft = f32(tgt[:, :K] + 0.8 * rng.standard_normal((1, K, V)))
    pr = oracle.propose(g, rev, dft, seed=5, offset=1, B=Bs, dft_batch_stride=0, nthreads=8)
    res = oracle.verify(g, tgt, dft, pr.tokens, pr.groups, seed=5, offset=1, B=Bs,
                        tgt_batch_stride=0, dft_batch_stride=0, nthreads=8)
    T = oracle.group_probs(g, tgt[0])
    assert chi2_p(np.bincount(res.out_groups[:, 0], minlength=g.G), T[0], Bs) > 1e-3
    sel = res.accept_len >= 1
    assert chi2_p(np.bincount(res.out_groups[sel, 1], minlength=g.G), T[1], int(sel.sum())) > 1e-3
    # acceptance rate at position 0 is 1 - TV(T, D)
    D = oracle.group_probs(g, dft[0])
    alpha = 1.0 - 0.5 * np.abs(T[0] - D[0]).sum()
    rate = (res.accept_len >= 1).mean()
    assert abs(rate - alpha) < 5 * np.sqrt(alpha * (1 - alpha) / Bs)


def test_propose_argument_errors():
    g, _, dft = small_case(V=8, G=6, seed=1, K=2)
    rev = oracle.reverse_index(g)
    with pytest.raises(oracle.OracleError):
        oracle.propose(g, rev, dft, temperature=0.0)
    with pytest.raises(oracle.OracleError):
        oracle.propose(g, rev, dft, pos0=0xFFFF)                       # position field would overflow
    bad = dft.copy()
    bad[0, 0, :] = -np.inf
    with pytest.raises(oracle.OracleError):
        oracle.propose(g, rev, bad)
