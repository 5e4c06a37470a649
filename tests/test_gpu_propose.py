"""GPU parity of the draft-side proposal coupling (Sec. 2.2 "Proposal coupling and acceptance",
Eq. 6): pcg_propose through the C ABI against the oracle's proposals on the same seeded inputs
and Philox draws, and the whole chain propose -> verify on the GPU.  Run with ``-m gpu``."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_13732_amd as pcg
import workloads as W
from parity import Tally, as_oracle_logits, compare_verify
from test_gpu_parity import logits_pair
from test_gpu_thinning import both_groups, chi2_p

pytestmark = pytest.mark.gpu


def compare_proposals(tok, grp, ref, og) -> Tally:
    """Tokens and groups agree exactly unless the oracle flagged the token draw as a near-tie;
    whatever the draw, the token is a member of its group."""
    tok, grp = tok.cpu().numpy(), grp.cpu().numpy()
    t = Tally(sequences=tok.size)
    t.flagged_token = int(ref.near.sum())
    for b, i in np.ndindex(tok.shape):
        x, g = int(tok[b, i]), int(grp[b, i])
        assert 0 <= g < og.G and x in og.members[og.row_ptr[g]:og.row_ptr[g + 1]], (b, i, x, g)
        if (x, g) != (int(ref.tokens[b, i]), int(ref.groups[b, i])):
            assert ref.near[b, i], f"({b},{i}): ({x},{g}) vs oracle ({ref.tokens[b, i]},{ref.groups[b, i]})"
            t.tolerated += 1
            t.detail.append({"b": b, "i": i, "gpu": (x, g), "oracle": (int(ref.tokens[b, i]), int(ref.groups[b, i]))})
    return t


@pytest.mark.parametrize("V,G,smin,smax,B,K,dtype,tau", [
    (64, 40, 1, 6, 33, 3, "f32", 1.0),
    (1000, 800, 2, 9, 17, 5, "bf16", 0.8),
    (4097, 3000, 4, 20, 9, 8, "bf16", 1.0),      # unaligned rows, a part with one element
    (2048, 2048, 10, 40, 12, 1, "f32", 0.7),     # K = 1, exactly one part
    (3000, 500, 40, 128, 5, 64, "f32", 1.0),     # K = PCG_MAX_K
    (50000, 6000, 10, 30, 6, 4, "f32", 1.3),     # 25 parts, ragged last part
    (5, 4, 1, 3, 200, 2, "f32", 1.0),            # tiny vocabulary
])
def test_propose_matches_oracle(V, G, smin, smax, B, K, dtype, tau):
    rp, mem = W.random_groups(V, G, smin, smax, seed=V * 3 + K, cover=False)
    og, dg, rev = both_groups(V, rp, mem)
    total = Tally()
    for step in range(6):
        _, dft = logits_pair(B, K, V, dtype, seed=1000 * step + V, sigma_d=2.0)
        diag = torch.zeros(8, dtype=torch.int32, device="cuda")
        tok, grp = pcg.propose(dg, dft.cuda(), temperature=tau, seed=42, offset=step, diag=diag)
        ref = oracle.propose(og, rev, as_oracle_logits(dft), temperature=tau, seed=42, offset=step, nthreads=8)
        total.add(compare_proposals(tok, grp, ref, og))
        assert int(diag[7]) == B * K
    total.report(f"propose V={V} K={K} {dtype}")
    assert total.tolerated <= max(1, total.sequences // 200)


def test_propose_strides_masks_pos0_and_empty_batch():
    V, B, K = 3000, 10, 3
    rp, mem = W.random_groups(V, 2000, 2, 10, seed=12, cover=True)
    og, dg, rev = both_groups(V, rp, mem)
    rng = np.random.default_rng(13)
    full = torch.from_numpy((3 * rng.standard_normal((B, K + 2, V + 24))).astype(np.float32))
    full[0, 0, 5:2000] = -np.inf                 # masked tokens are never proposed
    full[1, 1, :V] *= 30.0                       # sharply peaked row
    view = full[:, :K, :V]
    tok, grp = pcg.propose(dg, full.cuda()[:, :K, :V], seed=3, offset=8)
    ref = oracle.propose(og, rev, view.contiguous().numpy(), seed=3, offset=8)
    assert compare_proposals(tok, grp, ref, og).tolerated == 0
    assert not (5 <= int(tok[0, 0]) < 2000)
    # one position per call, as an autoregressive draft would: pos0 selects the counter
    for i in range(K):
        t1, g1 = pcg.propose(dg, full.cuda()[:, i:i + 1, :V], seed=3, offset=8, pos0=i)
        assert torch.equal(t1[:, 0], tok[:, i]) and torch.equal(g1[:, 0], grp[:, i])
    t0, g0 = pcg.propose(dg, torch.zeros((0, 2, V), device="cuda"))
    assert t0.numel() == 0 and g0.numel() == 0


def test_gpu_proposal_law_and_chain_with_verify():
    """2^18 sequences sharing one set of rows, everything on the GPU: proposed tokens follow p,
    proposed groups follow D (Eq. 6), and proposals fed to pcg_verify under the same seed and
    offset emit groups that follow T (Proposition)."""
    V, K, Bs, tau = 48, 2, 1 << 18, 0.8
    rp, mem = W.random_groups(V, 36, 2, 6, seed=71, cover=False)
    og, dg, rev = both_groups(V, rp, mem, prepare=True)
    t1, d1 = logits_pair(1, K, V, "f32", seed=72, sigma_t=2.0, sigma_d=0.7)
    tok, grp = pcg.propose(dg, d1.cuda(), temperature=tau, seed=11, offset=3, B=Bs)
    D = oracle.group_probs(og, d1[0].numpy(), tau)
    T = oracle.group_probs(og, t1[0].numpy(), tau)
    tk, gr = tok.cpu().numpy(), grp.cpu().numpy()
    for i in range(K):
        p = oracle.softmax_row(d1[0, i].numpy(), tau)
        assert chi2_p(np.bincount(tk[:, i], minlength=V), p) > 1e-3
        assert chi2_p(np.bincount(gr[:, i], minlength=og.G), D[i]) > 1e-3
    out = pcg.verify(dg, t1.cuda(), d1.cuda(), tok, grp, temperature=tau, seed=11, offset=3, B=Bs)
    og_out, al = out.out_groups.cpu().numpy(), out.accept_len.cpu().numpy()
    assert chi2_p(np.bincount(og_out[:, 0], minlength=og.G), T[0]) > 1e-3
    sel = al >= 1
    assert chi2_p(np.bincount(og_out[sel, 1], minlength=og.G), T[1]) > 1e-3
    alpha = 1.0 - 0.5 * np.abs(T[0] - D[0]).sum()
    assert abs(sel.mean() - alpha) < 5 * np.sqrt(alpha * (1 - alpha) / Bs)
    # and the chain agrees with the oracle's chain sequence by sequence on a sample
    n = 4096
    pr = oracle.propose(og, rev, d1.numpy(), temperature=tau, seed=11, offset=3, B=n, dft_batch_stride=0)
    t = compare_proposals(tok[:n], grp[:n], pr, og)
    ref = oracle.verify(og, t1.numpy(), d1.numpy(), pr.tokens, pr.groups, temperature=tau, seed=11,
                        offset=3, B=n, tgt_batch_stride=0, dft_batch_stride=0, nthreads=8)
    if t.tolerated == 0:
        sub = pcg.VerifyOutput(out.accept_len[:n], out.out_tokens[:n], out.out_groups[:n])
        assert compare_verify(sub, ref, og, pr.tokens, pr.groups).tolerated <= 1


@pytest.mark.parametrize("name,steps", [("C1", 200), ("C2", 60), ("C4", 2), ("C5", 1)])
def test_propose_recipes(name, steps):
    cfg = W.CONFIGS[name]
    rp, mem = W.groups(cfg)
    og, dg, rev = both_groups(cfg.V, rp, mem)
    total = Tally()
    for step in range(steps):
        _, dft, _, _ = W.step_inputs(cfg, og.row_ptr, og.members, step)
        tok, grp = pcg.propose(dg, dft.cuda(), temperature=cfg.temperature, seed=0, offset=step)
        ref = oracle.propose(og, rev, as_oracle_logits(dft), temperature=cfg.temperature, seed=0,
                             offset=step, nthreads=16)
        total.add(compare_proposals(tok, grp, ref, og))
    total.report(f"propose recipe {name}")
    assert total.tolerated <= max(1, total.sequences // 200)
