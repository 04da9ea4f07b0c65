#!/usr/bin/env python3
"""Benchmark of the Cassandra self-speculative decode hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

A step is one speculative round on synthetic Llama-3-8B-shaped data resident in HBM:
k draft passes that read only the speculation data, one verification pass over k+1 columns
that reads speculation + verification data, greedy acceptance and the commit.  Prints ONE
JSON line; `value` is the HBM rate of the whole round in algorithmic bytes (the bytes the
format obliges a pass to read), `roofline` describes the dominant kernel (the fused
draft decode+GEMV) from HIP-event timings taken in this process, `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload.
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

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--model", choices=["8b", "70b"], default="8b",
                    help="8b: the configuration the metric is quoted on; 70b: the 80-layer shape (k = 8) as context")
    ap.add_argument("--k", type=int, default=None, help="draft length (8B config: k = 6, 70B config: k = 8)")
    ap.add_argument("--keep", type=int, default=600, help="kept fraction in 1/1000 (paper default 40 %% pruned)")
    ap.add_argument("--trunc", type=int, default=4)
    ap.add_argument("--layers", type=int, default=None, help="default: 32 (8b) / 80 (70b)")
    ap.add_argument("--context", type=int, default=8192, help="committed KV positions when a step starts")
    ap.add_argument("--batch", type=int, default=1,
                    help="sequences decoded together (1..4, batch * (k + 1) <= 16); 1 is the configuration of the metric")
    ap.add_argument("--workload", choices=["model", "linear"], default="model")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.k is None:
        args.k = 8 if args.model == "70b" else 6
    if args.layers is None:
        args.layers = 80 if args.model == "70b" else 32
    return args


def cpu_baseline(keep, t, k):
    """The oracle as it stands, on one 4096x4096 linear layer of the workload: one draft GEMV
    and one verify GEMM with k+1 columns from the packed streams."""
    import numpy as np
    import synth
    from oracle import cassandra_oracle as O
    rows = cols = 4096
    W = synth.weight_matrix(rows, cols, seed=1)
    X = synth.activations(cols, k + 1, seed=2)
    p = O.encode_weight(W, keep, t)
    bw, sw, lw, pw = O.stream_words(cols, p.K, t)
    nbytes = rows * 4 * ((bw + sw) * 1 + (bw + sw + lw + pw))
    t0 = time.perf_counter()
    reps = 0
    while True:
        O.gemv_draft(p, X[0])
        O.gemm_verify(p, X)
        reps += 1
        el = time.perf_counter() - t0
        if el > 10.0 or reps >= 8:
            break
    try:
        import threadpoolctl
        cores = max([i.get("num_threads", 1) for i in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": nbytes * reps / el / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{reps} x (draft GEMV + verify GEMM, {k + 1} columns) on one 4096x4096 linear layer, "
                      f"keep {keep}/1000, t={t}; algorithmic stream bytes / wall time"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures the one-GPU path only: run with --gpus 1 "
              "(no multi-GPU figure is produced in this build)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_26558_amd import binding as B
    from paper_2605_26558_amd import workload

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = workload.build(B, args, dev)

    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    ms_per_step = el * 1e3 / args.steps

    roof = wl.roofline_pass()          # HIP events around the dominant kernel's launches
    out = {
        "metric": "draft/verify step HBM GB/s (% of peak) + batch-1 tokens/s, Llama-3-8B shape"
                  if args.model == "8b" else
                  "draft/verify step HBM GB/s (% of peak) + batch-1 tokens/s, Llama-3-70B shape (context figure)",
        "value": wl.bytes_per_step / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": wl.config,
        "roofline": roof,
        "pct_of_hbm_peak": 100.0 * wl.bytes_per_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
    }
    out.update(wl.extra(ms_per_step))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.keep, args.trunc, args.k)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
