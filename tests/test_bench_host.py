"""Host logic of bench.py (no GPU): the algorithmic bytes of a step against the formula worked out
by hand for the headline workload, the HBM traffic figures read back from the profile summary, and
the refusal of more than one GPU."""
import subprocess
import sys

import bench
import workloads as W


def test_algorithmic_bytes_of_the_headline_step():
    cfg = W.CONFIGS["C4"]
    assert (cfg.V, cfg.B, cfg.K, cfg.dtype) == (65536, 64, 8, "bf16")
    logits, csr, small = bench.algorithmic_bytes(cfg, 65536, 2097152)
    # every logit once: (2K + 1) rows of V bf16 per sequence = 278 528 B per verified position
    assert logits == 142606336 == 278528 * cfg.B * cfg.K
    # members, row pointers, multiplicities: 4 (nnz + G + 1 + V)
    assert csr == 4 * (2097152 + 65537 + 65536) == 8912900
    assert small == 4 * 64 * (19 + 18)
    assert logits + csr + small == 151528708


def test_traffic_figures_come_from_the_profile_summary():
    by_kernel, sources = bench.measured_traffic()
    assert {"row_stats@C4", "gather@C4", "accept_delta@C4", "finalize@C4", "step@C4"} <= set(by_kernel)
    assert len(sources) == 16 and int(sources, 16) >= 0
    assert len(bench.kernel_sources_digest()) == 16
    logits, csr, small = bench.algorithmic_bytes(W.CONFIGS["C4"], 65536, 2097152)
    # measured HBM bytes can exceed the algorithmic ones (re-reads), never fall far below them
    assert by_kernel["row_stats@C4"] >= 0.99 * logits
    assert by_kernel["step@C4"] >= by_kernel["row_stats@C4"] + by_kernel["gather@C4"]
    assert by_kernel["step@C4"] < 3 * (logits + csr + small)


def test_more_than_one_gpu_is_refused_with_a_message():
    out = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True)
    assert out.returncode != 0
    assert "--gpus 1" in (out.stdout + out.stderr)
