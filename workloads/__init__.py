"""Seeded synthetic inputs for PCG verification: embeddings, groups, logits, proposals.

This module only *makes inputs*.  It holds none of the verification arithmetic
(no softmax, no group probabilities, no accept test): the CPU oracle and the
HIP library each do that on their own, and both read what is produced here.

The paper's workload is a speech LM over a 65 536-entry codec vocabulary with
overlapping cosine-neighbour groups of tens of tokens (Sec. 2.1, Sec. 3.1);
neither the model nor its embedding table is available, so the recipes
below stand in for it: same vocabulary sizes, overlapping nearest-neighbour
groups, one (K+1)-row verification per step.

Everything random on the host comes from ``numpy.random.default_rng`` keyed by
(data seed, purpose, step), so it does not depend on the device.  The
neighbour search may run on a GPU through torch; its result is only ever used
as data that both sides read, so neighbour ties cannot affect parity.
"""
from __future__ import annotations

import functools
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    V: int
    emb_dim: int
    emb_kind: str            # "iid" | "mixture" | "zipf_mixture"
    n_centres: int
    sigma_within: float
    group_kind: str          # "knn" | "threshold"
    knn: int                 # group = token + knn nearest cosine neighbours
    threshold: float         # group = all tokens with cosine >= threshold ...
    max_size: int            # ... truncated to the max_size most similar (incl. self)
    B: int
    K: int
    dtype: str               # "f32" | "bf16"
    temperature: float
    logits_kind: str         # "normal" | "zipf" | "peaked"
    target_sigma: float
    draft_scale: float       # draft = draft_scale * target + N(0, draft_sigma^2)
    draft_sigma: float
    data_seed: int
    steps: int               # number of steps the recipe asks for


CONFIGS = {
    "C1": Config("C1", 1024, 256, "iid", 0, 0.0, "knn", 7, 0.0, 0, 1, 4, "f32", 1.0,
                 "normal", 3.0, 1.0, 1.0, 1, 1000),
    "C2": Config("C2", 4096, 512, "iid", 0, 0.0, "knn", 15, 0.0, 0, 8, 8, "bf16", 1.0,
                 "normal", 4.0, 0.8, 1.5, 2, 10000),
    "C3": Config("C3", 16384, 768, "mixture", 256, 0.3, "knn", 31, 0.0, 0, 32, 8, "bf16", 1.0,
                 "zipf", 0.5, 1.0, 1.0, 3, 100),
    "C4": Config("C4", 65536, 1024, "iid", 0, 0.0, "knn", 31, 0.0, 0, 64, 8, "bf16", 1.0,
                 "normal", 4.0, 1.0, 1.0, 4, 100),
    "C5": Config("C5", 32768, 512, "zipf_mixture", 512, 0.5, "threshold", 0, 0.8, 128, 128, 6,
                 "f32", 0.7, "peaked", 4.0, 1.0, 1.0, 5, 100),
    # The largest groups the paper reports trying (Sec. 2.2 "Complexity and memory": mean size
    # about 140 on the 65 536-entry vocabulary, about 9.2 M membership entries): C4 with 139
    # neighbours per token.
    "C6": Config("C6", 65536, 1024, "iid", 0, 0.0, "knn", 139, 0.0, 0, 64, 8, "bf16", 1.0,
                 "normal", 4.0, 1.0, 1.0, 6, 100),
}


def _rng(cfg: Config, purpose: int, step: int = 0) -> np.random.Generator:
    return np.random.default_rng([cfg.data_seed, purpose, step])


# --------------------------------------------------------------------------- embeddings

def embeddings(cfg: Config) -> np.ndarray:
    """float32 [V, emb_dim] token embeddings of the recipe."""
    rng = _rng(cfg, 0)
    V, d = cfg.V, cfg.emb_dim
    if cfg.emb_kind == "iid":
        return rng.standard_normal((V, d), dtype=np.float32)
    if cfg.emb_kind == "mixture":          # equal-size clusters
        centres = rng.standard_normal((cfg.n_centres, d), dtype=np.float32)
        assign = np.repeat(np.arange(cfg.n_centres), V // cfg.n_centres)
        assign = np.concatenate([assign, np.arange(V - len(assign)) % cfg.n_centres])
    elif cfg.emb_kind == "zipf_mixture":   # cluster sizes ~ rank^-1.2, each >= 1, summing to V
        centres = rng.standard_normal((cfg.n_centres, d), dtype=np.float32)
        w = np.arange(1, cfg.n_centres + 1, dtype=np.float64) ** -1.2
        sizes = np.maximum(1, np.floor(w / w.sum() * (V - cfg.n_centres)).astype(np.int64) + 1)
        sizes[0] += V - sizes.sum()
        assert sizes.sum() == V and sizes.min() >= 1
        assign = np.repeat(np.arange(cfg.n_centres), sizes)
    else:
        raise ValueError(cfg.emb_kind)
    assign = rng.permutation(assign)       # token ids carry no cluster order
    noise = rng.standard_normal((V, d), dtype=np.float32)
    return centres[assign] + np.float32(cfg.sigma_within) * noise


# --------------------------------------------------------------------------- groups

def _neighbour_sets(cfg: Config, emb: np.ndarray, device: str) -> list[np.ndarray]:
    """Per seed token, the sorted token ids of its similarity group (self included)."""
    E = torch.from_numpy(emb).to(device)
    E = E / E.norm(dim=1, keepdim=True)
    V = cfg.V
    width = cfg.knn + 1 if cfg.group_kind == "knn" else min(cfg.max_size, V)
    out: list[np.ndarray] = []
    chunk = 2048
    for lo in range(0, V, chunk):
        hi = min(V, lo + chunk)
        sim = E[lo:hi] @ E.T
        sim[torch.arange(hi - lo, device=device), torch.arange(lo, hi, device=device)] = 2.0
        val, idx = torch.topk(sim, width, dim=1)
        val, idx = val.cpu().numpy(), idx.cpu().numpy()
        for r in range(hi - lo):
            ids = idx[r] if cfg.group_kind == "knn" else idx[r][val[r] >= cfg.threshold]
            out.append(np.sort(ids.astype(np.int32)))
    return out


def groups_from_sets(sets: list[np.ndarray]) -> tuple[np.ndarray, np.ndarray]:
    """Distinct sets, in order of first appearance, as CSR (row_ptr, members)."""
    seen: set[bytes] = set()
    kept: list[np.ndarray] = []
    for s in sets:
        key = s.tobytes()
        if key not in seen:
            seen.add(key)
            kept.append(s)
    row_ptr = np.zeros(len(kept) + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum([len(s) for s in kept])
    members = np.concatenate(kept).astype(np.int32) if kept else np.zeros(0, np.int32)
    return row_ptr, members


@functools.lru_cache(maxsize=8)
def _groups_cached(name: str, device: str):
    cfg = CONFIGS[name]
    return groups_from_sets(_neighbour_sets(cfg, embeddings(cfg), device))


def groups(cfg: Config, device: Optional[str] = None) -> tuple[np.ndarray, np.ndarray]:
    """CSR group -> tokens of the recipe (members ascending inside a group,
    duplicate sets dropped).  Every token is in its own neighbour set, so no
    token is left uncovered."""
    if device is None:
        device = "cuda" if torch.cuda.is_available() else "cpu"
    rp, mem = _groups_cached(cfg.name, device)
    return rp.copy(), mem.copy()


# --------------------------------------------------------------------------- logits

def logits(cfg: Config, step: int = 0, B: Optional[int] = None) -> tuple[torch.Tensor, torch.Tensor]:
    """(target [B, K+1, V], draft [B, K, V]) CPU tensors in the recipe's dtype."""
    rng = _rng(cfg, 1, step)
    B = cfg.B if B is None else B
    K, V = cfg.K, cfg.V
    if cfg.logits_kind == "zipf":
        tgt = np.empty((B, K + 1, V), dtype=np.float32)
        base = (-1.1 * np.log(np.arange(1, V + 1, dtype=np.float64))).astype(np.float32)
        for b in range(B):
            for i in range(K + 1):
                tgt[b, i] = base[rng.permutation(V)]
        tgt += np.float32(cfg.target_sigma) * rng.standard_normal((B, K + 1, V), dtype=np.float32)
    else:
        tgt = np.float32(cfg.target_sigma) * rng.standard_normal((B, K + 1, V), dtype=np.float32)
    dft = np.float32(cfg.draft_scale) * tgt[:, :K] \
        + np.float32(cfg.draft_sigma) * rng.standard_normal((B, K, V), dtype=np.float32)
    if cfg.logits_kind == "peaked":        # half of the draft rows sharply peaked
        odd = (np.arange(B)[:, None] + np.arange(K)[None, :]) % 2 == 1
        dft[odd] *= np.float32(4.0)
    t, d = torch.from_numpy(tgt), torch.from_numpy(dft)
    if cfg.dtype == "bf16":                # round to nearest even once; both sides read the bf16
        t, d = t.to(torch.bfloat16), d.to(torch.bfloat16)
    return t, d


# --------------------------------------------------------------------------- proposals

def reverse_index(V: int, row_ptr: np.ndarray, members: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """token -> groups holding it, as CSR (tok_ptr [V+1], tok_groups [nnz])."""
    G = len(row_ptr) - 1
    entry_group = np.repeat(np.arange(G, dtype=np.int32), np.diff(row_ptr))
    order = np.argsort(members, kind="stable")
    tok_ptr = np.zeros(V + 1, dtype=np.int64)
    tok_ptr[1:] = np.cumsum(np.bincount(members, minlength=V))
    return tok_ptr, entry_group[order]


def proposals(draft: torch.Tensor, temperature: float, row_ptr: np.ndarray, members: np.ndarray,
              rng: np.random.Generator) -> tuple[np.ndarray, np.ndarray]:
    """Draft proposals under the coupling of Eq. (6): a token drawn from the
    draft's distribution at each position (by the Gumbel-max trick, so no
    probabilities are formed here), then one of the groups holding it, uniformly.
    Returns int32 (prop_tokens [B, K], prop_groups [B, K]).

    This is an INPUT GENERATOR, a second sampler unrelated to both implementations of
    pcg_propose: it only makes plausible proposals for the verification tests and the
    benchmark.  It is never the checker of anything -- pcg_propose is compared with
    oracle.propose, draw for draw, and neither of them calls or shares code with this."""
    x = draft.to(torch.float32).numpy().astype(np.float64) / temperature
    B, K, V = x.shape
    gumbel = -np.log(-np.log(rng.random((B, K, V))))
    tok = np.argmax(x + gumbel, axis=2).astype(np.int32)
    tok_ptr, tok_groups = reverse_index(V, row_ptr, members)
    n = (tok_ptr[tok + 1] - tok_ptr[tok])
    if (n < 1).any():
        raise ValueError("proposed token is in no group; canonicalise the groups first")
    pick = np.minimum((rng.random((B, K)) * n).astype(np.int64), n - 1)
    grp = tok_groups[tok_ptr[tok] + pick].astype(np.int32)
    return tok, grp


def step_inputs(cfg: Config, row_ptr: np.ndarray, members: np.ndarray, step: int = 0,
                B: Optional[int] = None):
    """(target, draft, prop_tokens, prop_groups) of one decode step of the recipe."""
    tgt, dft = logits(cfg, step, B)
    tok, grp = proposals(dft, cfg.temperature, row_ptr, members, _rng(cfg, 2, step))
    return tgt, dft, tok, grp


# --------------------------------------------------------------------------- small random cases

def random_groups(V: int, G: int, min_size: int, max_size: int, seed: int,
                  cover: bool = True) -> tuple[np.ndarray, np.ndarray]:
    """Random overlapping groups for unit tests: G groups with sizes uniform in
    [min_size, max_size], members distinct inside a group and ascending.  With
    ``cover`` every token is put in at least one group."""
    rng = np.random.default_rng([seed, 77])
    sets = [np.sort(rng.choice(V, size=int(rng.integers(min_size, max_size + 1)), replace=False))
            for _ in range(G)]
    if cover:
        present = np.zeros(V, dtype=bool)
        for s in sets:
            present[s] = True
        for v in np.nonzero(~present)[0]:
            k = int(rng.integers(0, G))
            sets[k] = np.unique(np.append(sets[k], v))
    row_ptr = np.zeros(G + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum([len(s) for s in sets])
    return row_ptr, np.concatenate(sets).astype(np.int32)


def random_weights(V: int, members: np.ndarray, seed: int) -> np.ndarray:
    """General per-entry weights for a membership (Sec. 2.2, Eq. 2): positive Gamma(0.7) draws,
    normalised over the entries of each token, as float32 [nnz]."""
    rng = np.random.default_rng([seed, 77])
    raw = rng.gamma(0.7, size=len(members)) + 1e-12
    tot = np.zeros(V)
    np.add.at(tot, members, raw)
    return (raw / tot[members]).astype(np.float32)
