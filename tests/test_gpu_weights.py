"""GPU parity with general per-entry weights w_{k,t} (Sec. 2.2, Eq. 2 and Eq. 4): every entry
point through the C ABI against the oracle's weighted form on the same seeded inputs and
Philox draws.  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_13732_amd as pcg
import workloads as W
from parity import (Tally, as_oracle_logits, compare_thinning, compare_verify, group_probs_error,
                    oracle_groups, report_error, run_both, run_both_thinning)
from test_gpu_parity import TOL_F32, coupled_proposals, logits_pair
from test_gpu_propose import compare_proposals
from test_gpu_thinning import chi2_p

pytestmark = pytest.mark.gpu


def weighted_groups(V, rp, mem, seed, prepare=True):
    """The same membership and the same random weights on both sides; on the device with the
    weights inside the prepared layout, or (prepare=False) read from the CSR."""
    og0 = oracle_groups(V, rp, mem)
    w = W.random_weights(og0.V, og0.members, seed)
    og = oracle.with_weights(og0, w)
    dg = pcg.Groups.from_csr(V, rp, mem, "cuda", weights=w, reverse=True, prepare=prepare)
    assert (dg.prepared is not None) == prepare and dg.nnz == og.nnz
    assert not prepare or dg.prepared_info.off_weights > 0
    np.testing.assert_array_equal(dg.tok_weights.cpu().numpy()[:og.nnz], og.tok_weights)
    return og, dg, oracle.reverse_index(og)


SHAPES = [
    (64, 40, 1, 6, 33, 3, "f32", 1.0),
    (1000, 800, 2, 9, 17, 5, "bf16", 0.8),
    (4097, 3000, 4, 20, 9, 8, "bf16", 1.0),      # unaligned rows
    (3000, 500, 40, 128, 5, 16, "f32", 1.0),     # groups wider than a wave
    (50000, 6000, 10, 30, 6, 4, "f32", 1.3),     # two LDS tiles
    (100000, 3000, 5, 40, 3, 2, "bf16", 1.0),    # three LDS tiles
]


@pytest.mark.parametrize("layout", ["prepared", "csr"])
@pytest.mark.parametrize("V,G,smin,smax,B,K,dtype,tau", SHAPES)
def test_weighted_entry_points_match_oracle(V, G, smin, smax, B, K, dtype, tau, layout):
    rp, mem = W.random_groups(V, G, smin, smax, seed=V * 3 + K, cover=False)
    og, dg, rev = weighted_groups(V, rp, mem, seed=V, prepare=layout == "prepared")
    # Eq. (4) for a few rows
    t, _ = logits_pair(4, 1, V, dtype, seed=V, sigma_t=4.0)
    x = t[:, 0].contiguous()
    err = group_probs_error(pcg.group_probs(dg, x.cuda(), tau), oracle.group_probs(og, as_oracle_logits(x), tau))
    report_error(f"weighted group_probs V={V} {dtype} {layout}", err)
    assert err <= TOL_F32
    tv, tt, tp = Tally(), Tally(), Tally()
    for step in range(5):
        tgt, dft = logits_pair(B, K, V, dtype, seed=1000 * step + V, sigma_d=0.6)
        # proposals by the library itself, checked against the oracle's
        tok, grp = pcg.propose(dg, dft.cuda(), temperature=tau, seed=42, offset=step)
        ref = oracle.propose(og, rev, as_oracle_logits(dft), temperature=tau, seed=42, offset=step, nthreads=8)
        tp.add(compare_proposals(tok, grp, ref, og))
        ptok, pgrp = ref.tokens, ref.groups
        gpu, r, _, diag = run_both(V, rp, mem, tgt, dft, ptok, pgrp, temperature=tau, seed=42,
                                   offset=step, dg=dg, og=og)
        tv.add(compare_verify(gpu, r, og, ptok, pgrp))
        assert diag["sequences"] == B
        gpu, trials, r, _ = run_both_thinning(V, tgt, dft, ptok, pgrp, dg=dg, og=og, rev=rev,
                                              temperature=tau, seed=42, offset=step)
        tt.add(compare_thinning(gpu, trials, r, og, ptok, pgrp))
    tv.report(f"weighted verify V={V} K={K} {dtype} {layout}")
    tt.report(f"weighted thinning V={V} K={K} {dtype} {layout}")
    tp.report(f"weighted propose V={V} K={K} {dtype} {layout}")
    for t in (tv, tt, tp):
        assert t.tolerated <= max(1, t.sequences // 200)


def test_equal_split_written_as_weights_gives_the_equal_split_laws():
    """weights = 1 / N(t) through the weighted code path: same group probabilities as the
    unweighted path to fp32 rounding, and on 2^17 shared-row sequences the emitted groups of both
    residual samplers follow T."""
    V, K, Bs, tau = 48, 2, 1 << 17, 0.8
    rp, mem = W.random_groups(V, 36, 2, 6, seed=71, cover=False)
    og0 = oracle_groups(V, rp, mem)
    w = (1.0 / og0.mult[og0.members]).astype(np.float32)
    dgw = pcg.Groups.from_csr(V, rp, mem, "cuda", weights=w, reverse=True)
    dg0 = pcg.Groups.from_csr(V, rp, mem, "cuda", prepare=False, reverse=True)
    t1, d1 = logits_pair(1, K, V, "f32", seed=72, sigma_t=2.0, sigma_d=0.7)
    a = pcg.group_probs(dgw, t1[0].cuda(), tau)
    b = pcg.group_probs(dg0, t1[0].cuda(), tau)
    assert float((a - b).abs().max() / b.max()) < 1e-6
    T = oracle.group_probs(og0, t1[0].numpy(), tau)
    tok, grp = pcg.propose(dgw, d1.cuda(), temperature=tau, seed=11, offset=3, B=Bs)
    D = oracle.group_probs(og0, d1[0].numpy(), tau)
    assert chi2_p(np.bincount(grp.cpu().numpy()[:, 0], minlength=og0.G), D[0]) > 1e-3
    for fn in (pcg.verify, lambda *a_, **k_: pcg.verify_thinning(*a_, **k_)[0]):
        out = fn(dgw, t1.cuda(), d1.cuda(), tok, grp, temperature=tau, seed=11, offset=3, B=Bs)
        assert chi2_p(np.bincount(out.out_groups.cpu().numpy()[:, 0], minlength=og0.G), T[0]) > 1e-3


@pytest.mark.parametrize("name,steps", [("C2", 40), ("C4", 1), ("C5", 1), ("C6", 1)])
def test_weighted_recipes(name, steps):
    cfg = W.CONFIGS[name]
    rp, mem = W.groups(cfg)
    og, dg, rev = weighted_groups(cfg.V, rp, mem, seed=cfg.data_seed)
    tv, tt = Tally(), Tally()
    for step in range(steps):
        tgt, dft, _, _ = W.step_inputs(cfg, og.row_ptr, og.members, step)
        pr = oracle.propose(og, rev, as_oracle_logits(dft), temperature=cfg.temperature, seed=0,
                            offset=step, nthreads=16)
        gpu, r, _, _ = run_both(cfg.V, rp, mem, tgt, dft, pr.tokens, pr.groups,
                                temperature=cfg.temperature, seed=0, offset=step, dg=dg, og=og)
        tv.add(compare_verify(gpu, r, og, pr.tokens, pr.groups))
        gpu, trials, r, _ = run_both_thinning(cfg.V, tgt, dft, pr.tokens, pr.groups, dg=dg, og=og, rev=rev,
                                              temperature=cfg.temperature, seed=0, offset=step)
        tt.add(compare_thinning(gpu, trials, r, og, pr.tokens, pr.groups))
    tv.report(f"weighted verify recipe {name}")
    tt.report(f"weighted thinning recipe {name}")
    assert tv.tolerated <= max(1, tv.sequences // 100) and tt.tolerated <= max(1, tt.sequences // 100)
