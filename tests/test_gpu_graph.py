"""The verification entry points only launch kernels on the caller's stream, so a serving loop can
record a step into a HIP graph and replay it.  Each replay, with the program's own eager work and
synchronisations in between, must give what the eager call gives on the same inputs (which the
other GPU tests compare with the oracle).  Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest
import torch

import paper_2511_13732_amd as pcg
import workloads as W
from test_gpu_parity import logits_pair

pytestmark = pytest.mark.gpu


def same(a: pcg.VerifyOutput, b: pcg.VerifyOutput):
    for x, y in ((a.accept_len, b.accept_len), (a.out_tokens, b.out_tokens), (a.out_groups, b.out_groups)):
        np.testing.assert_array_equal(x.cpu().numpy(), y.cpu().numpy())


def test_a_recorded_step_replays_to_the_eager_result():
    V, G, B, K, tau = 6000, 4000, 24, 4, 0.9
    rp, mem = W.random_groups(V, G, 4, 24, seed=5, cover=False)
    dg = pcg.Groups.from_csr(V, rp, mem, "cuda", reverse=True)
    dev = torch.device("cuda")
    tgt = torch.empty((B, K + 1, V), dtype=torch.bfloat16, device=dev)
    dft = torch.empty((B, K, V), dtype=torch.bfloat16, device=dev)
    ptok = torch.empty((B, K), dtype=torch.int32, device=dev)
    pgrp = torch.empty((B, K), dtype=torch.int32, device=dev)
    new_out = lambda: pcg.VerifyOutput(torch.empty(B, dtype=torch.int32, device=dev),
                                       torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                                       torch.empty((B, K + 1), dtype=torch.int32, device=dev))
    out_v, out_t = new_out(), new_out()
    trials = torch.empty(B, dtype=torch.int32, device=dev)
    ws = torch.empty(max(pcg.verify_workspace_bytes(V, dg.G, B, K), pcg.verify_thinning_workspace_bytes(V, B, K),
                         pcg.propose_workspace_bytes(V, B, K)), dtype=torch.uint8, device=dev)

    def step():
        # the draft side proposes, then both residual samplers verify the same proposals
        pcg.propose(dg, dft, temperature=tau, seed=3, offset=11, prop_tokens=ptok, prop_groups=pgrp, workspace=ws)
        pcg.verify(dg, tgt, dft, ptok, pgrp, temperature=tau, seed=3, offset=11, out=out_v, workspace=ws)
        pcg.verify_thinning(dg, tgt, dft, ptok, pgrp, temperature=tau, seed=3, offset=11, out=out_t,
                            trials=trials, workspace=ws)

    def fill(seed):
        t, d = logits_pair(B, K, V, "bf16", seed=seed, sigma_d=0.7)
        tgt.copy_(t.to(dev))
        dft.copy_(d.to(dev))

    side = torch.cuda.Stream()
    fill(0)
    with torch.cuda.stream(side):
        step()                                       # warm-up outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for seed in (1, 2, 3, 4):
        fill(seed)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (out_v.accept_len, out_v.out_tokens, out_v.out_groups,
                                   out_t.accept_len, out_t.out_tokens, out_t.out_groups, trials, ptok, pgrp)]
        for x in (out_v.accept_len, out_v.out_tokens, out_v.out_groups, out_t.accept_len, out_t.out_tokens,
                  out_t.out_groups, trials, ptok, pgrp):
            x.fill_(-7)                              # eager work between the replays
        step()
        torch.cuda.synchronize()
        want = (out_v.accept_len, out_v.out_tokens, out_v.out_groups, out_t.accept_len, out_t.out_tokens,
                out_t.out_groups, trials, ptok, pgrp)
        for g, w in zip(got, want):
            np.testing.assert_array_equal(g.cpu().numpy(), w.cpu().numpy())
        assert (out_v.accept_len >= 0).all() and (out_v.accept_len <= K).all()


def test_calls_on_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    """The library keeps no device state between calls (pcg_verify_static's array aside), so
    calls that run at the same time on two streams, each with a workspace of its own, must give
    what the same calls give one after the other.  Default-priority streams, several rounds."""
    V, B, K, tau = 20000, 24, 6, 0.9
    rp, mem = W.random_groups(V, 9000, 4, 30, seed=77, cover=False)
    dg = pcg.Groups.from_csr(V, rp, mem, "cuda", reverse=True)
    dev = dg.device
    inputs = []
    for seed in (1, 2):
        t, d = logits_pair(B, K, V, "bf16", seed=seed, sigma_d=0.7)
        t, d = t.to(dev), d.to(dev)
        ptok, pgrp = pcg.propose(dg, d, temperature=tau, seed=5, offset=seed)
        inputs.append((t, d, ptok, pgrp))
    torch.cuda.synchronize()
    nbytes = max(pcg.verify_workspace_bytes(V, dg.G, B, K), pcg.verify_thinning_workspace_bytes(V, B, K))
    ws = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(2)]

    def one(k, rounds):
        t, d, ptok, pgrp = inputs[k]
        res = []
        for r in range(rounds):
            v = pcg.verify(dg, t, d, ptok, pgrp, temperature=tau, seed=9, offset=r, workspace=ws[k])
            th, trials = pcg.verify_thinning(dg, t, d, ptok, pgrp, temperature=tau, seed=9, offset=r, workspace=ws[k])
            res.append((v.accept_len, v.out_tokens, v.out_groups, th.accept_len, th.out_tokens, th.out_groups, trials))
        return res

    rounds = 12
    want = [one(0, rounds), one(1, rounds)]             # one after the other on the current stream
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [None, None]
    for k in (0, 1):
        with torch.cuda.stream(streams[k]):
            got[k] = one(k, rounds)
    for s in streams:
        s.synchronize()
    for k in (0, 1):
        for a, b in zip(got[k], want[k]):
            for x, y in zip(a, b):
                np.testing.assert_array_equal(x.cpu().numpy(), y.cpu().numpy())
