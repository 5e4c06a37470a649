"""GPU parity of the similarity-group construction (Sec. 2.1, Eq. 1): pcg_asg_normalize,
pcg_asg_build and pcg_asg_build_exact through the C ABI against the oracle.  Unit vectors
bit-exact; membership of the bf16 form exact except for pairs the oracle flags as within 1e-5
of the threshold (fp32 accumulation against fp64), which are counted; membership of the exact
form equal to Eq. (1) on the embeddings in double (a cosine within 1e-12 of the threshold would
be flagged: none occurs).  Run with ``-m gpu`` on an MI355X."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2511_13732_amd as pcg
import workloads as W
from parity import Tally
from test_oracle_asg import bf16_to_f64, embeddings

pytestmark = pytest.mark.gpu


def as_bf16_tensor(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)


def csr_rows(row_ptr, members):
    return [members[row_ptr[k]:row_ptr[k + 1]] for k in range(len(row_ptr) - 1)]


def compare_groups(got: pcg.AsgGroups, ref: oracle.AsgResult, name: str) -> Tally:
    """Exact CSR equality when the oracle flagged no near-tie row; otherwise every kept group of
    either side whose seed and all of whose members are unflagged must appear on the other."""
    t = Tally(sequences=ref.groups.V)
    t.flagged_group = int(ref.near_rows.sum())
    rp, mem = got.row_ptr.cpu().numpy(), got.members.cpu().numpy()
    seed = got.seed_of.cpu().numpy()
    g = ref.groups
    assert rp[0] == 0 and rp[-1] == got.nnz and (np.diff(rp) >= 1).all()
    np.testing.assert_array_equal(got.mult.cpu().numpy(), np.bincount(mem, minlength=g.V))
    for k, row in enumerate(csr_rows(rp, mem)):
        assert (np.diff(row) > 0).all() and seed[k] in row, (name, k)
    if t.flagged_group == 0:
        assert (got.G, got.nnz) == (g.G, g.nnz), name
        np.testing.assert_array_equal(rp, g.row_ptr)
        np.testing.assert_array_equal(mem, g.members)
        np.testing.assert_array_equal(seed, ref.seed_of)
        return t
    mine = {int(s): r for s, r in zip(seed, csr_rows(rp, mem))}
    theirs = {int(s): r for s, r in zip(ref.seed_of, csr_rows(g.row_ptr, g.members))}
    flagged = ref.near_rows.astype(bool)
    for s in sorted(set(mine) | set(theirs)):
        a, b = mine.get(s), theirs.get(s)
        if a is not None and b is not None and np.array_equal(a, b):
            continue
        rows = [r for r in (a, b) if r is not None]
        assert flagged[s] or any(flagged[r].any() for r in rows), f"{name}: group of token {s} differs, no near-tie"
        t.tolerated += 1
    return t


@pytest.mark.parametrize("V,d", [(100, 64), (1000, 256), (4096, 512)])
def test_unit_vectors_are_bit_exact(V, d):
    E = embeddings(V, d, 5)
    E[3] = 0.0
    E[4] *= 1e-20
    E[5] *= 1e15
    E[6, 1], E[6, 2] = -0.0, 0.0                # signed zeros keep their sign
    unit = pcg.asg_normalize(torch.from_numpy(E).cuda())
    torch.cuda.synchronize()
    got = unit.view(torch.int16).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(got, oracle.asg_normalize(E))


@pytest.mark.parametrize("V,d,theta,centres,sigma", [
    (128, 64, 0.3, 0, 0),          # exactly one tile
    (300, 64, 0.25, 0, 0),         # ragged: three tiles, the last with 44 rows
    (1000, 128, 0.2, 0, 0),
    (2000, 256, 0.5, 40, 0.5),     # clustered: groups of tens of tokens
    (4096, 512, 0.12, 0, 0),       # 32 x 32 tiles
    (1500, 192, 0.6, 30, 0.3),
    (777, 64, -2.0, 0, 0),         # everything in one group: a group larger than cap, retried
])
def test_groups_match_oracle(V, d, theta, centres, sigma):
    E = embeddings(V, d, V + d) if centres == 0 else embeddings(V, d, V + d, centres, sigma)[0]
    bits = oracle.asg_normalize(E)
    ref = oracle.asg_build(bits, theta, nthreads=16)
    got = pcg.asg_build(as_bf16_tensor(bits).cuda(), theta, cap=64)
    t = compare_groups(got, ref, f"V={V} d={d} theta={theta}")
    t.report(f"asg V={V} d={d} theta={theta}")
    sizes = np.diff(ref.groups.row_ptr)
    print(f"asg V={V}: G={ref.groups.G} nnz={ref.groups.nnz} sizes {sizes.min()}..{sizes.max()} "
          f"largest G(t) {got.max_size}", flush=True)
    assert got.max_size >= sizes.max()
    assert t.tolerated <= max(2, t.flagged_group)


def test_duplicates_are_merged_and_the_result_feeds_verification():
    """Identical embeddings give identical sets, kept once; the device CSR is accepted by the
    library's own validation and by pcg_verify."""
    V, d = 1024, 128
    E, assign = embeddings(V, d, 21, centres=50, sigma=0.3)
    E[700:720] = E[100:120]
    bits = oracle.asg_normalize(E)
    ref = oracle.asg_build(bits, 0.7, nthreads=16)
    got = pcg.asg_build(as_bf16_tensor(bits).cuda(), 0.7)
    assert compare_groups(got, ref, "duplicates").tolerated == 0 or ref.near_rows.any()
    assert got.G < V
    rp, mem = got.row_ptr.cpu().numpy(), got.members.cpu().numpy()
    assert pcg.groups_validate_host(V, rp, mem, got.mult.cpu().numpy()) == 0
    dg = pcg.Groups.from_csr(V, rp, mem, "cuda")
    assert dg.G == got.G                                  # every token is covered: nothing appended
    x = torch.randn(3, V, device="cuda")
    np.testing.assert_allclose(pcg.group_probs(dg, x).double().sum(dim=1).cpu().numpy(), 1.0, atol=2e-6)


def test_recipe_rows_at_full_size():
    """C4's embeddings (65 536 x 1024) at a threshold that gives groups of tens of tokens.  The
    oracle forms the unit vectors of every row itself; the device's must equal them bit for bit.
    The oracle cannot run all 4.3e9 pairs, so it computes sampled rows of G(t) one by one, from
    its own unit vectors; each must equal the device's set for that token (through seed_of /
    equality of sets).  The same rows by Eq. (1) on the unrounded embeddings (double, strict >)
    may differ from the device's only for pairs inside the bf16 rounding band around theta."""
    from test_oracle_asg import BF16_BAND
    cfg = W.CONFIGS["C4"]
    E = W.embeddings(cfg)
    bits = oracle.asg_normalize(E)                      # every row, by the oracle
    unit = pcg.asg_normalize(torch.from_numpy(E).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(unit.view(torch.int16).cpu().numpy().view(np.uint16), bits)
    theta = 0.105                      # iid N(0,1) in d = 1024: cosines are N(0, 1/1024)
    got = pcg.asg_build(as_bf16_tensor(bits).cuda(), theta, cap=512)      # the oracle's own bits go in
    rp, mem, seed = got.row_ptr.cpu().numpy(), got.members.cpu().numpy(), got.seed_of.cpu().numpy()
    print(f"C4 theta={theta}: G={got.G} nnz={got.nnz} mean size {got.nnz / got.G:.1f} largest {got.max_size}", flush=True)
    assert got.G == cfg.V and 5 < got.nnz / got.G < 500
    where = {int(s): k for k, s in enumerate(seed)}
    tol = n_mem = n_diff = 0
    worst = 0.0
    for t in [0, 1, 127, 128, 4095, 32768, 65535, 12345, 50000]:
        row, near = oracle.asg_row(bits, theta, t)
        mine = mem[rp[where[t]]:rp[where[t] + 1]]
        if not np.array_equal(mine, row):
            assert near > 0, f"token {t}: sets differ without a near-tie"
            tol += 1
        exact, cos = oracle.asg_row_exact(E, float(np.float32(theta)), t)
        odd = np.setxor1d(mine, exact)
        n_mem += len(exact)
        n_diff += len(odd)
        if len(odd):
            worst = max(worst, float(np.abs(cos[odd] - np.float32(theta)).max()))
            assert (np.abs(cos[odd] - np.float32(theta)) <= BF16_BAND).all(), f"token {t}: outside the band"
    print(f"C4 sampled rows against Eq. (1) on the embeddings: {n_diff} of {n_mem} memberships differ, "
          f"farthest from theta {worst:.2e} (band {BF16_BAND:.2e})", flush=True)
    assert tol <= 2


@pytest.mark.parametrize("V,d,theta,centres,sigma", [
    (128, 64, 0.3, 0, 0),          # exactly one tile
    (300, 64, 0.25, 0, 0),         # ragged
    (1000, 128, 0.2, 0, 0),
    (2000, 256, 0.5, 40, 0.5),     # clustered: the threshold lies inside the clusters' cosines
    (4096, 512, 0.12, 0, 0),
    (1500, 192, 0.6, 30, 0.3),
    (1200, 64, 0.42, 0, 0),        # the paper's range of theta
    (777, 64, -2.0, 0, 0),         # everything in one group
])
def test_exact_groups_are_eq1_on_the_embeddings(V, d, theta, centres, sigma):
    """pcg_asg_build_exact against the oracle's Eq. (1) in double on the float32 embeddings:
    the whole CSR must be equal.  Also counted: how many memberships the rounded form
    (pcg_asg_build on the same embeddings) gets differently, i.e. what the exact form repairs."""
    E = embeddings(V, d, V + d) if centres == 0 else embeddings(V, d, V + d, centres, sigma)[0]
    E[V // 2] = 0.0                                              # a zero row: cosine 0 with everything
    E[V // 3] = E[V // 3 + 1]                                    # a duplicate: merged
    th = float(np.float32(theta))
    ref = oracle.asg_build_exact(E, th, nthreads=16)
    dev = torch.from_numpy(E).cuda()
    got = pcg.asg_build_exact(dev, theta, cap=64)
    t = compare_groups(got, ref, f"exact V={V} d={d} theta={theta}")
    t.report(f"asg exact V={V} d={d} theta={theta}")
    assert t.flagged_group == 0 and t.tolerated == 0
    rounded = pcg.asg_build(pcg.asg_normalize(dev), theta, cap=64)
    a = set(zip(np.repeat(got.seed_of.cpu().numpy(), np.diff(got.row_ptr.cpu().numpy())).tolist(),
                got.members.cpu().numpy().tolist()))
    b = set(zip(np.repeat(rounded.seed_of.cpu().numpy(), np.diff(rounded.row_ptr.cpu().numpy())).tolist(),
                rounded.members.cpu().numpy().tolist()))
    print(f"asg exact V={V} d={d} theta={theta}: G={got.G} nnz={got.nnz} largest {got.max_size}; "
          f"the rounded form differs in {len(a ^ b)} (seed, member) entries", flush=True)
    assert got.max_size == int(np.diff(ref.groups.row_ptr).max()) or theta < -1


def test_exact_recipe_rows_at_full_size():
    """C4's embeddings (65 536 x 1024) through pcg_asg_build_exact: sampled rows of G(t) must
    equal Eq. (1) in double on the embeddings, member for member (the oracle computes the rows one
    by one and reports every cosine, so a pair close enough to theta for the order of summation
    to matter would be seen: the closest is printed)."""
    cfg = W.CONFIGS["C4"]
    E = W.embeddings(cfg)
    theta = 0.105
    th = float(np.float32(theta))
    got = pcg.asg_build_exact(torch.from_numpy(E).cuda(), theta, cap=512)
    rp, mem, seed = got.row_ptr.cpu().numpy(), got.members.cpu().numpy(), got.seed_of.cpu().numpy()
    print(f"C4 exact theta={theta}: G={got.G} nnz={got.nnz} mean size {got.nnz / got.G:.1f} largest {got.max_size}", flush=True)
    assert got.G == cfg.V
    np.testing.assert_array_equal(got.mult.cpu().numpy(), np.bincount(mem, minlength=cfg.V))
    where = {int(s): k for k, s in enumerate(seed)}
    closest = 1.0
    n_mem = 0
    for t in [0, 1, 127, 128, 4095, 32768, 65535, 12345, 50000, 256, 65280, 33333]:
        exact, cos = oracle.asg_row_exact(E, th, t)
        closest = min(closest, float(np.abs(np.delete(cos, t) - th).min()))
        mine = mem[rp[where[t]]:rp[where[t] + 1]]
        np.testing.assert_array_equal(mine, exact, err_msg=f"token {t}")
        n_mem += len(exact)
    print(f"C4 exact: {n_mem} memberships of 12 sampled rows equal to Eq. (1) in double; "
          f"closest cosine to theta {closest:.2e} away", flush=True)
    assert closest > 1e-12


def test_exact_rows_of_a_clustered_recipe_at_full_size():
    """C5's embeddings (32 768 x 512, clusters of very different sizes) at a threshold inside the
    clusters' own cosines: groups from one to over a thousand members, a large share of every
    group's candidates inside the rounding band, and a first room per group that is too small
    (the call is repeated with the room the library reports).  Sampled rows, from the largest
    cluster to singletons, must equal Eq. (1) in double on the embeddings."""
    cfg = W.CONFIGS["C5"]
    E = W.embeddings(cfg)
    theta = 0.83
    th = float(np.float32(theta))
    got = pcg.asg_build_exact(torch.from_numpy(E).cuda(), theta, cap=256)
    rp, mem, seed = got.row_ptr.cpu().numpy(), got.members.cpu().numpy(), got.seed_of.cpu().numpy()
    sizes = np.diff(rp)
    print(f"C5 exact theta={theta}: G={got.G} nnz={got.nnz} sizes {sizes.min()}..{sizes.max()} "
          f"largest G(t) {got.max_size}", flush=True)
    assert got.max_size > 256 and sizes.max() == got.max_size
    np.testing.assert_array_equal(got.mult.cpu().numpy(), np.bincount(mem, minlength=cfg.V))
    where = {int(s): k for k, s in enumerate(seed)}
    order = np.argsort(sizes)
    picks = [int(seed[order[-1]]), int(seed[order[len(order) // 2]]), int(seed[order[0]]), 0, 1, cfg.V - 1, 12345, 20000]
    closest, n_mem, n_band = 1.0, 0, 0
    for t in picks:
        exact, cos = oracle.asg_row_exact(E, th, t)
        others = np.delete(cos, t)
        closest = min(closest, float(np.abs(others - th).min()))
        n_band += int((np.abs(others - th) < 4e-3).sum())
        if t in where:
            mine = mem[rp[where[t]]:rp[where[t] + 1]]
        else:           # an exact duplicate of an earlier token's set: find it through a member
            k = next(k for k in (where.get(int(v)) for v in exact) if k is not None and
                     np.array_equal(mem[rp[k]:rp[k + 1]], exact))
            mine = mem[rp[k]:rp[k + 1]]
        np.testing.assert_array_equal(mine, exact, err_msg=f"token {t}")
        n_mem += len(exact)
    print(f"C5 exact: {n_mem} memberships of {len(picks)} sampled rows equal to Eq. (1) in double; "
          f"{n_band} of their pairs lay inside the rounding band; closest cosine to theta {closest:.2e} away",
          flush=True)
    assert closest > 1e-12 and n_band > 0


@pytest.mark.parametrize("case", range(int(os.environ.get("PCG_RANDOM_CASES", "16"))))
def test_random_construction_shapes(case):
    """Seeded random shapes of the construction: vocabulary, embedding width, threshold, iid or
    clustered embeddings are drawn; both forms run against their oracles (whole CSR)."""
    rng = np.random.default_rng([1, 2511, case])
    V = int(np.exp(rng.uniform(np.log(2), np.log(2500))))
    d = 64 * int(rng.integers(1, 7))
    clustered = bool(rng.random() < 0.5) and V >= 8
    centres = int(rng.integers(2, max(3, V // 4))) if clustered else 0
    sigma = float(rng.uniform(0.1, 0.8))
    E = embeddings(V, d, 100 + case, centres, sigma)[0] if clustered else embeddings(V, d, 100 + case)
    # a threshold that cuts through the cosines that occur: a quantile of a sample of them
    X = E[: min(V, 400)].astype(np.float64)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    S = (X @ X.T)[np.triu_indices(len(X), 1)] if len(X) > 1 else np.array([0.0])
    theta = float(np.float32(np.quantile(S, rng.uniform(0.5, 0.999)))) if len(S) else 0.0
    name = f"asg random #{case}: V={V} d={d} theta={theta:.4f} centres={centres} sigma={sigma:.2f}"
    print(name, flush=True)
    dev = torch.from_numpy(E).cuda()
    exact = pcg.asg_build_exact(dev, theta, cap=64)
    t = compare_groups(exact, oracle.asg_build_exact(E, theta, nthreads=16), name + " exact")
    assert t.flagged_group == 0 and t.tolerated == 0
    bits = oracle.asg_normalize(E)
    ref = oracle.asg_build(bits, theta, nthreads=16)
    t = compare_groups(pcg.asg_build(as_bf16_tensor(bits).cuda(), theta, cap=64), ref, name)
    t.report(name)
    assert t.tolerated <= max(2, t.flagged_group)
