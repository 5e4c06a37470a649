#!/usr/bin/env python3
"""Benchmark of PCG group-level verification on one MI355X.

A "step" is one pcg_verify call: the whole hot path (row softmax statistics, accept scan,
residual group and token sampling) over one batch of synthetic logits of the headline
recipe C4 (V = 65 536, 32-member cosine-neighbour groups, B = 64, K = 8, bf16).  Inputs are
resident in HBM before the timed region; several input sets are rotated so that the logits
(142.6 MB per step) cannot be served from the 256 MB Infinity Cache.

Prints ONE JSON line: verified draft positions per second, the HBM roofline of the dominant
kernel (durations from HIP events recorded by the library around each of its kernels, in a
second instrumented pass over the same steps) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size).
# Filled in from profiles/; None until measured for that workload.
MEASURED_TRAFFIC_BYTES = {}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="C4", help="workload recipe (C1..C5); C4 is the headline")
    ap.add_argument("--sets", type=int, default=3, help="distinct input sets rotated through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="lower bound on the CPU oracle's timed work")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain device copies of known size (for scaling PMC counters)")
    return ap.parse_args()


def algorithmic_bytes(cfg, G, nnz):
    """Bytes the method must move per step: every logit once, the CSR membership, the
    multiplicities, and the small per-sequence inputs and outputs."""
    s = 2 if cfg.dtype == "bf16" else 4
    logits = s * cfg.V * cfg.B * (2 * cfg.K + 1)
    csr = 4 * (nnz + (G + 1) + cfg.V)
    small = 4 * cfg.B * (2 * cfg.K + 3 + 2 * (cfg.K + 1))
    return logits, csr, small


def calibrate_copy():
    import torch
    n = 256 << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "device copy", "bytes_read": n, "bytes_written": n, "launches": 5}))


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (the path shards over sequences with no "
                 "exchange step; see DESIGN.md); run with --gpus 1")
    import numpy as np
    import torch

    if args.calibrate_copy:
        calibrate_copy()
        return

    import paper_2511_13732_amd as pcg
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS[args.config]
    t0 = time.time()
    rp, mem = W.groups(cfg)
    groups = pcg.Groups.from_csr(cfg.V, rp, mem, dev)
    rp_c, mem_c, _ = pcg.groups_canonicalize_host(cfg.V, rp, mem)
    print(f"[bench] {cfg.name}: V={cfg.V} G={groups.G} nnz={groups.nnz} B={cfg.B} K={cfg.K} "
          f"{cfg.dtype} (groups built in {time.time() - t0:.1f}s)", file=sys.stderr, flush=True)

    sets = []
    for s in range(args.sets):
        tgt, dft, ptok, pgrp = W.step_inputs(cfg, rp_c, mem_c, step=s)
        sets.append((tgt.to(dev), dft.to(dev), torch.from_numpy(ptok).to(dev),
                     torch.from_numpy(pgrp).to(dev)))
    out = pcg.VerifyOutput(torch.empty(cfg.B, dtype=torch.int32, device=dev),
                           torch.empty((cfg.B, cfg.K + 1), dtype=torch.int32, device=dev),
                           torch.empty((cfg.B, cfg.K + 1), dtype=torch.int32, device=dev))
    ws = torch.empty(pcg.verify_workspace_bytes(cfg.V, groups.G, cfg.B, cfg.K), dtype=torch.uint8,
                     device=dev)
    print(f"[bench] {args.sets} input sets resident ({time.time() - t0:.1f}s)", file=sys.stderr,
          flush=True)

    def step(i):
        tgt, dft, ptok, pgrp = sets[i % len(sets)]
        pcg.verify(groups, tgt, dft, ptok, pgrp, temperature=cfg.temperature, seed=0, offset=i,
                   out=out, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin
    ms_per_step = 1e3 * elapsed / args.steps
    positions = cfg.B * cfg.K
    value = positions * args.steps / elapsed
    mean_accept = float(out.accept_len.float().mean())

    # second pass over the same steps with the library's per-kernel HIP events
    pcg.profile_begin(args.steps)
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    stage_ms, ncalls = pcg.profile_end()
    dominant = max(stage_ms, key=stage_ms.get)
    logits_b, csr_b, small_b = algorithmic_bytes(cfg, groups.G, groups.nnz)
    # algorithmic bytes of one launch of each kernel (units it processes x bytes per unit)
    kernel_bytes = {
        "row_stats": logits_b,                                     # every logit once
        "gather": 4 * cfg.B * cfg.V + 4 * (groups.nnz + groups.G + 1) + 4 * cfg.B * groups.G,
    }
    roof_kernel = dominant if dominant in kernel_bytes else "row_stats"
    dur_s = stage_ms[roof_kernel] * 1e-3
    achieved = kernel_bytes[roof_kernel] / dur_s / 1e9 if dur_s > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": roof_kernel, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(f"{roof_kernel}@{cfg.name}"),
                "algorithmic_bytes": kernel_bytes[roof_kernel],
                "kernel_us": round(1e3 * stage_ms[roof_kernel], 2)}

    result = {
        "metric": "verified draft positions/sec at V=65536,B=64,K=8; achieved HBM GB/s vs peak",
        "value": round(value, 1), "unit": "positions/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: V={cfg.V} G={groups.G} nnz={groups.nnz} B={cfg.B} "
                               f"K={cfg.K} {cfg.dtype} logits, tau={cfg.temperature}",
                   "input_sets": args.sets, "mean_accept_len": round(mean_accept, 3)},
        "step_hbm_frac": round((logits_b + csr_b + small_b) / elapsed * args.steps / 1e9
                               / HBM_PEAK_GBS, 4),
        "stages_us": {k: round(1e3 * v, 2) for k, v in stage_ms.items()},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        import oracle
        og = oracle.canonicalize(cfg.V, rp, mem)
        nthreads = min(16, os.cpu_count() or 1)
        host = [(W.step_inputs(cfg, og.row_ptr, og.members, step=s)) for s in range(1)]
        tgt, dft, ptok, pgrp = host[0]
        tl = oracle.bf16_bits(tgt) if cfg.dtype == "bf16" else tgt.numpy()
        dl = oracle.bf16_bits(dft) if cfg.dtype == "bf16" else dft.numpy()
        n, used = 0, 1
        c0 = time.perf_counter()
        while True:
            r = oracle.verify(og, tl, dl, ptok, pgrp, temperature=cfg.temperature, seed=0,
                              offset=n, nthreads=nthreads)
            used = r.threads
            n += 1
            dt = time.perf_counter() - c0
            if dt >= args.cpu_seconds or n >= 200:
                break
        result["cpu_baseline"] = {"value": round(positions * n / dt, 1), "unit": "positions/s",
                                  "cores": used, "kind": "oracle",
                                  "sample": f"{n} step(s) of the same workload "
                                            f"({cfg.B} sequences each), {dt:.1f}s of wall time"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
