"""GPU parity of the thinning sampler (Sec. 2.2 "Residual sampling via thinning", Eq. 9):
pcg_verify_thinning through the C ABI against the oracle's thinning step on the same seeded
inputs and the same Philox draws.  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest
import scipy.stats
import torch

import oracle
import paper_2511_13732_amd as pcg
import workloads as W
from parity import Tally, compare_thinning, oracle_groups, run_both_thinning
from test_gpu_parity import coupled_proposals, logits_pair

pytestmark = pytest.mark.gpu


def both_groups(V, rp, mem, prepare=False):
    og = oracle_groups(V, rp, mem)
    dg = pcg.Groups.from_csr(V, rp, mem, "cuda", prepare=prepare, reverse=True)
    rev = oracle.reverse_index(og)
    np.testing.assert_array_equal(rev[0], dg.tok_ptr.cpu().numpy())
    np.testing.assert_array_equal(rev[1], dg.tok_groups.cpu().numpy()[:og.nnz])
    return og, dg, rev


@pytest.mark.parametrize("V,G,smin,smax,B,K,dtype,tau", [
    (64, 40, 1, 6, 33, 3, "f32", 1.0),
    (1000, 800, 2, 9, 17, 5, "bf16", 0.8),
    (4097, 3000, 4, 20, 9, 8, "bf16", 1.0),      # unaligned rows, a part with one element
    (2048, 2048, 10, 40, 12, 1, "f32", 0.7),     # K = 1, exactly one part
    (3000, 500, 40, 128, 5, 64, "f32", 1.0),     # K = PCG_MAX_K, groups wider than a wave
    (50000, 6000, 10, 30, 6, 4, "f32", 1.0),     # 25 parts, ragged last part
    (5, 4, 1, 3, 200, 2, "f32", 1.0),            # tiny vocabulary
])
def test_thinning_matches_oracle(V, G, smin, smax, B, K, dtype, tau):
    rp, mem = W.random_groups(V, G, smin, smax, seed=V * 3 + K, cover=False)
    og, dg, rev = both_groups(V, rp, mem)
    total = Tally()
    ntrials, lens = [], []
    for step in range(6):
        tgt, dft = logits_pair(B, K, V, dtype, seed=1000 * step + V, sigma_d=0.6)
        ptok, pgrp = coupled_proposals(dft, tau, og, seed=step)
        gpu, trials, ref, diag = run_both_thinning(V, tgt, dft, ptok, pgrp, dg=dg, og=og, rev=rev,
                                                   temperature=tau, seed=42, offset=step)
        total.add(compare_thinning(gpu, trials, ref, og, ptok, pgrp))
        assert diag["sequences"] == B and diag["bad_proposal"] == 0
        assert not (ref.flags & 2).any() and diag["residual_fallback"] == 0
        ntrials += ref.trials.tolist()
        lens += ref.accept_len.tolist()
    total.report(f"thinning small V={V} K={K} {dtype}")
    assert total.tolerated <= max(1, total.sequences // 200)
    assert len(set(lens)) > 1 and max(ntrials) >= 1


def test_thinning_many_rounds():
    """Draft close to the target: a rejection is rare and then takes many trials (1 / TV on
    average), so the kernel goes through several rounds of 16 concurrent trials."""
    V, B, K = 1000, 512, 2
    rp, mem = W.random_groups(V, 700, 2, 9, seed=77, cover=False)
    og, dg, rev = both_groups(V, rp, mem)
    tgt, dft = logits_pair(B, K, V, "f32", seed=5, sigma_d=0.05)
    ptok, pgrp = coupled_proposals(dft, 1.0, og, seed=6)
    gpu, trials, ref, _ = run_both_thinning(V, tgt, dft, ptok, pgrp, dg=dg, og=og, rev=rev, seed=8)
    t = compare_thinning(gpu, trials, ref, og, ptok, pgrp)
    t.report("thinning many rounds")
    assert t.tolerated <= 2
    assert (ref.trials > 16).sum() >= 3, ref.trials.max()


def test_thinning_accept_scan_equals_enumerated_path():
    """The accept scan is shared: both entry points give the same accept lengths and the same
    accepted prefix on the same inputs and stream."""
    V, B, K = 5000, 32, 4
    rp, mem = W.random_groups(V, 4000, 3, 12, seed=3, cover=True)
    og, dg, rev = both_groups(V, rp, mem, prepare=True)
    tgt, dft = logits_pair(B, K, V, "bf16", seed=8)
    ptok, pgrp = coupled_proposals(dft, 1.0, og, seed=1)
    args = (dg, tgt.cuda(), dft.cuda(), torch.from_numpy(ptok).cuda(), torch.from_numpy(pgrp).cuda())
    a = pcg.verify(*args, seed=5, offset=9)
    b, trials = pcg.verify_thinning(*args, seed=5, offset=9)
    c, trials2 = pcg.verify_thinning(*args, seed=5, offset=9)
    assert torch.equal(a.accept_len, b.accept_len)
    al = a.accept_len.cpu().numpy()
    ta, tb = a.out_tokens.cpu().numpy(), b.out_tokens.cpu().numpy()
    for s in range(B):
        assert (ta[s, :al[s]] == tb[s, :al[s]]).all()
    assert torch.equal(b.out_tokens, c.out_tokens) and torch.equal(trials, trials2)   # deterministic


def test_thinning_degenerate_cases():
    V, K = 64, 2
    rp, mem = W.random_groups(V, 30, 2, 6, seed=4, cover=True)
    og, dg, rev = both_groups(V, rp, mem)
    g0 = 0
    seg = og.members[og.row_ptr[g0]:og.row_ptr[g0 + 1]]
    rng = np.random.default_rng(1)
    base = rng.standard_normal((4, K + 1, V)).astype(np.float32)
    tgt = base.copy()
    dft = base[:, :K].copy() + 0.5 * rng.standard_normal((4, K, V)).astype(np.float32)
    # sequence 0: draft == target everywhere: every proposal is accepted, bonus position
    dft[0] = tgt[0, :K]
    # sequence 1: draft row == target row, proposed group without mass on either: rejected, and
    # no trial can ever be accepted (T == D for every group): the trial limit ends the loop
    dft[1, 0] = tgt[1, 0]
    tgt[1, 0, seg] = -np.inf
    dft[1, 0, seg] = -np.inf
    # sequence 2: half the vocabulary masked on the target
    tgt[2, :, ::2] = -np.inf
    # sequence 3: out-of-range proposal on the GPU side only is covered below
    ptok = np.zeros((4, K), np.int32) + seg[0]
    pgrp = np.zeros((4, K), np.int32) + g0
    gpu, trials, ref, diag = run_both_thinning(V, torch.from_numpy(tgt), torch.from_numpy(dft), ptok,
                                               pgrp, dg=dg, og=og, rev=rev, seed=3)
    assert compare_thinning(gpu, trials, ref, og, ptok, pgrp).tolerated == 0
    assert ref.accept_len[0] == K and ref.trials[0] == 0
    assert ref.accept_len[1] == 0 and ref.flags[1] & 2 and ref.trials[1] == pcg.THIN_MAX_TRIALS
    assert int(trials[1]) == pcg.THIN_MAX_TRIALS and diag["residual_fallback"] == 1
    z2 = gpu.out_tokens.cpu().numpy()[2]
    assert z2[int(gpu.accept_len[2])] % 2 == 1          # a masked token is never emitted
    # out-of-range proposals are rejected, not dereferenced
    pg = pgrp.copy()
    pg[3, 0] = dg.G + 7
    out, tr = pcg.verify_thinning(dg, torch.from_numpy(tgt).cuda(), torch.from_numpy(dft).cuda(),
                                  torch.from_numpy(ptok).cuda(), torch.from_numpy(pg).cuda(), seed=3)
    assert int(out.accept_len[3]) == 0 and int(tr[3]) >= 1
    # empty batch
    out, tr = pcg.verify_thinning(dg, torch.zeros((0, 3, V), device="cuda"),
                                  torch.zeros((0, 2, V), device="cuda"),
                                  torch.zeros((0, 2), dtype=torch.int32, device="cuda"),
                                  torch.zeros((0, 2), dtype=torch.int32, device="cuda"))
    assert out.accept_len.numel() == 0 and tr.numel() == 0


def chi2_p(counts, probs):
    n = counts.sum()
    keep = probs * n >= 5
    obs = np.append(counts[keep], counts[~keep].sum())
    exp = np.append(probs[keep], probs[~keep].sum()) * n
    if exp[-1] == 0:
        obs, exp = obs[:-1], exp[:-1]
    return scipy.stats.chisquare(obs, exp * obs.sum() / exp.sum()).pvalue


def test_gpu_thinning_law():
    """On the HIP path itself, 2^17 sequences sharing one set of rows: groups emitted after a
    rejection at position 0 follow the enumerated residual of Eq. (8), the first emitted group
    overall follows the target's group distribution (Proposition), the mean number of trials is
    1 / sum_k [T - D]_+, and the bonus token follows q_K."""
    V, K, Bs, tau = 48, 2, 1 << 17, 0.8
    rp, mem = W.random_groups(V, 36, 2, 6, seed=71, cover=False)
    og, dg, rev = both_groups(V, rp, mem)
    t1, d1 = logits_pair(1, K, V, "f32", seed=72, sigma_t=2.0, sigma_d=0.7)
    ptok, pgrp = coupled_proposals(d1.expand(Bs, K, V), tau, og, seed=5)
    gpu, trials = pcg.verify_thinning(dg, t1.cuda(), d1.cuda(), torch.from_numpy(ptok).cuda(),
                                      torch.from_numpy(pgrp).cuda(), temperature=tau, seed=11,
                                      offset=3, B=Bs)
    grp, tok = gpu.out_groups.cpu().numpy(), gpu.out_tokens.cpu().numpy()
    al, ntr = gpu.accept_len.cpu().numpy(), trials.cpu().numpy()
    T = oracle.group_probs(og, t1[0].numpy(), tau)
    D = oracle.group_probs(og, d1[0].numpy(), tau)
    R = np.maximum(0.0, T[0] - D[0])
    rej = al == 0
    assert rej.sum() > 10000
    assert chi2_p(np.bincount(grp[rej, 0], minlength=og.G), R / R.sum()) > 1e-3
    assert chi2_p(np.bincount(grp[:, 0], minlength=og.G), T[0]) > 1e-3
    mean, want = ntr[rej].mean(), 1.0 / R.sum()
    sd = np.sqrt(1.0 - R.sum()) / R.sum() / np.sqrt(rej.sum())     # geometric law
    assert abs(mean - want) < 5 * sd, (mean, want, sd)
    bonus = al == K
    qK = oracle.softmax_row(t1[0, K].numpy(), tau)
    assert chi2_p(np.bincount(tok[bonus, K], minlength=V), qK) > 1e-3
    # token inside the emitted group, Eq. (10), for the most frequent wide group after a rejection
    wide = [g for g in range(og.G) if og.row_ptr[g + 1] - og.row_ptr[g] >= 3]
    g = max(wide, key=lambda k: (grp[rej, 0] == k).sum())
    seg = og.members[og.row_ptr[g]:og.row_ptr[g + 1]]
    q0 = oracle.softmax_row(t1[0, 0].numpy(), tau)
    w = q0[seg] / og.mult[seg]
    sel = rej & (grp[:, 0] == g)
    counts = np.array([(tok[sel, 0] == t).sum() for t in seg])
    assert chi2_p(counts, w / w.sum()) > 1e-3


@pytest.mark.parametrize("name,steps", [("C1", 200), ("C2", 60), ("C3", 1), ("C4", 1), ("C5", 1), ("C6", 1)])
def test_thinning_recipes(name, steps):
    cfg = W.CONFIGS[name]
    rp, mem = W.groups(cfg)
    og, dg, rev = both_groups(cfg.V, rp, mem)
    total = Tally()
    ntr = []
    for step in range(steps):
        tgt, dft, ptok, pgrp = W.step_inputs(cfg, og.row_ptr, og.members, step)
        gpu, trials, ref, diag = run_both_thinning(cfg.V, tgt, dft, ptok, pgrp, dg=dg, og=og, rev=rev,
                                                   temperature=cfg.temperature, seed=0, offset=step)
        total.add(compare_thinning(gpu, trials, ref, og, ptok, pgrp))
        ntr += ref.trials[ref.trials > 0].tolist()
    total.report(f"thinning recipe {name}")
    print(f"{name}: trials per rejection mean {np.mean(ntr):.2f} max {max(ntr)}", flush=True)
    assert total.tolerated <= max(1, total.sequences // 200)
