"""pcg_verify_static -- the entry point for callers that cannot allocate -- against pcg_verify,
through the C ABI.  Both run the same kernels, so every output must be identical; the second call
is smaller than the first, so it finds the library's array full of the first call's leftovers.
Run with ``-m gpu`` on an MI355X."""
import numpy as np
import pytest
import torch

import paper_2511_13732_amd as pcg
import workloads as W
from test_gpu_parity import logits_pair

pytestmark = pytest.mark.gpu


def new_out(B, K, dev):
    return pcg.VerifyOutput(torch.full((B,), -9, dtype=torch.int32, device=dev),
                            torch.full((B, K + 1), -9, dtype=torch.int32, device=dev),
                            torch.full((B, K + 1), -9, dtype=torch.int32, device=dev))


def one_call(dg, V, B, K, dtype, seed, tau):
    dev = torch.device("cuda")
    tgt, dft = logits_pair(B, K, V, dtype, seed=seed, sigma_d=0.8)
    tgt, dft = tgt.to(dev), dft.to(dev)
    gen = np.random.default_rng(seed)
    pgrp = torch.from_numpy(gen.integers(0, dg.G, size=(B, K), dtype=np.int32)).to(dev)
    ptok = torch.from_numpy(gen.integers(0, V, size=(B, K), dtype=np.int32)).to(dev)
    want, got = new_out(B, K, dev), new_out(B, K, dev)
    dw = torch.zeros(8, dtype=torch.int32, device=dev)
    dgot = torch.zeros(8, dtype=torch.int32, device=dev)
    pcg.verify(dg, tgt, dft, ptok, pgrp, temperature=tau, seed=5, offset=seed, out=want, diag=dw)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    pcg.verify(dg, tgt, dft, ptok, pgrp, temperature=tau, seed=5, offset=seed, out=got, diag=dgot,
               static_scratch=True)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for a, b in ((want.accept_len, got.accept_len), (want.out_tokens, got.out_tokens),
                 (want.out_groups, got.out_groups), (dw, dgot)):
        np.testing.assert_array_equal(a.cpu().numpy(), b.cpu().numpy())
    al = got.accept_len.cpu().numpy()
    assert ((al >= 0) & (al <= K)).all()


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    assert pcg.static_scratch_bytes() == 48 << 20
    V, G = 9000, 7000
    rp, mem = W.random_groups(V, G, 3, 40, seed=11, cover=False)
    big = pcg.Groups.from_csr(V, rp, mem, "cuda")
    one_call(big, V, 48, 6, "bf16", seed=1, tau=0.9)
    # a smaller step (fewer tokens, groups, sequences and positions) on the same array
    V2, G2 = 1500, 900
    rp2, mem2 = W.random_groups(V2, G2, 2, 17, seed=12, cover=False)
    small = pcg.Groups.from_csr(V2, rp2, mem2, "cuda")
    one_call(small, V2, 5, 3, "fp32", seed=2, tau=1.1)
    # and the CSR gather (no prepared layout) once more, which writes every group's sum
    one_call(small.without_prepared(), V2, 7, 2, "bf16", seed=3, tau=1.0)


def test_static_scratch_refuses_a_step_that_does_not_fit():
    V = G = 65536
    B, K = 128, 8                      # twice the headline batch: 74 MB of scratch
    assert pcg.verify_workspace_bytes(V, G, B, K) > pcg.static_scratch_bytes()
    rp, mem = W.random_groups(512, 300, 2, 9, seed=1, cover=False)
    dg = pcg.Groups.from_csr(512, rp, mem, "cuda")
    gs = dg.struct()
    gs.V, gs.G = V, G                  # only the sizes are looked at before the refusal
    import ctypes as C
    rc = pcg.lib().pcg_verify_static(C.byref(gs), 0x1000, 0x1000, 1, B, K, (K + 1) * V, V, K * V, V, 1.0,
                                     0x1000, 0x1000, 0, 0, 0x1000, 0x1000, 0x1000, None, None)
    assert rc == -11 and "scratch" in pcg.strerror(rc)
