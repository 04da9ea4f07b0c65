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
    ap.add_argument("--workload", choices=["model", "linear", "probe-linear", "probe-attn", "tune", "exp-modes", "cpu-units"], default="model",
                    help="model: the metric's workload; linear: the linear layers alone; probe-*: short fixed "
                         "launch sequences for hardware-counter runs (no JSON line, see workload.py); cpu-units: the "
                         "oracle's time for whole units of the workload, host only, minutes; tune: format "
                         "search on measured draft / verification pass times with user-supplied acceptance rates; "
                         "exp-modes: pass times with raw, unary-coded and shared exponents on the same model")
    ap.add_argument("--kv-exp-mode", choices=["raw", "shared"], default="raw",
                    help="exponents of the KV cache: raw (the metric's configuration) or shared per 32 channels "
                         "(Sec. 4.2, the MX approach; context figures)")
    ap.add_argument("--alpha", type=float, default=0.8, help="tune: acceptance rate assumed for every grid point")
    ap.add_argument("--alpha-grid", default=None, help="tune: JSON file with a [n_keep][n_trunc] table of acceptance rates")
    ap.add_argument("--tune-keeps", default="700,600,500,400", help="tune: kept fractions in 1/1000 (Sec. 7.2.2 grid)")
    ap.add_argument("--tune-truncs", default="0,1,2,3,4,5", help="tune: truncation bits")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.k is None:
        args.k = 8 if args.model == "70b" else 6
    if args.layers is None:
        args.layers = 80 if args.model == "70b" else 32
    return args


def _cpu_sample(keep, t, k, ctx_len):
    """Seeded sample of the bench workload for the CPU oracle: 256 output rows of each of the four
    layer matrices of the 8B shape (encoded with the oracle's own encoder, untimed: encoding is
    offline) and the cache of one kv head of one layer over the benchmark's context.  Returns the
    encoded inputs and the algorithmic bytes of one pass over them (draft, verification)."""
    import numpy as np
    import synth
    from oracle import cassandra_oracle as O
    rows = 256
    mats = []
    draft_b = verify_b = 0
    for i, cols in enumerate((4096, 4096, 4096, 14336)):       # wqkv, wo, wgu read 4096 columns, wd 14336
        W = synth.weight_matrix(rows, cols, seed=10 + i)
        p = O.encode_weight(W, keep, t)
        bw, sw, lw, pw = O.stream_words(cols, p.K, t)
        draft_b += rows * 4 * (bw + sw)
        verify_b += rows * 4 * (bw + sw + lw + pw)
        mats.append((p, synth.activations(cols, k + 1, seed=20 + i)))
    rng = np.random.Generator(np.random.Philox(31))
    Kc = rng.standard_normal((ctx_len, 128)).astype(np.float32)
    Kc[:, [3, 40, 77, 100]] *= 10.0
    Vc = rng.standard_normal((ctx_len, 128)).astype(np.float32)
    to16 = lambda a: (a.view(np.uint32) >> 16).astype(np.uint16)
    pk, pv = O.encode_kv(to16(Kc), keep, t), O.encode_kv(to16(Vc), keep, t)
    bw, sw, lw, pw = O.stream_words(128, pk.K, t)
    draft_b += 2 * ctx_len * 4 * (bw + sw)
    verify_b += 2 * ctx_len * 4 * (bw + sw + lw + pw)
    q = to16(rng.standard_normal((k + 1, 4, 128)).astype(np.float32))     # 4 query heads share the kv head
    return {"mats": mats, "pk": pk, "pv": pv, "q": q, "draft_bytes": draft_b, "verify_bytes": verify_b, "k": k}


def _cpu_sample_pass(S):
    """One draft pass and one verification pass of the oracle over the sample."""
    from oracle import cassandra_oracle as O
    for p, X in S["mats"]:
        O.gemv_draft(p, X[0])
        O.gemm_verify(p, X)
    for full, ncols in ((False, 1), (True, S["k"] + 1)):
        dec = O.decode_full if full else O.decode_draft
        Kd, Vd = O.bf16_to_f64(dec(S["pk"])), O.bf16_to_f64(dec(S["pv"]))
        for c in range(ncols):
            for h in range(4):
                O.attention_one(O.bf16_to_f64(S["q"][c, h]), Kd, Vd)


def _cpu_worker(args):
    """Runs in a process of its own (one BLAS thread): passes over the sample for `seconds`."""
    keep, t, k, ctx_len, seconds = args
    import threadpoolctl
    with threadpoolctl.threadpool_limits(1):
        S = _cpu_sample(keep, t, k, ctx_len)
        _cpu_sample_pass(S)                      # warm
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < seconds:
            _cpu_sample_pass(S)
            reps += 1
        return reps, time.perf_counter() - t0, S["draft_bytes"] + S["verify_bytes"]


def cpu_baseline(keep, t, k, ctx_len):
    """The oracle as it stands, timed on the host cores BEFORE the GPU is touched (worker
    processes are spawned): a bounded sample of the benchmark workload (see _cpu_sample), one
    draft pass + one verification pass per repetition, (a) in one process with one thread and
    (b) in one single-threaded process per available core, each on its own copy of the sample
    (output rows and kv heads are independent, so this is the oracle run row-parallel).  The
    rate is algorithmic stream bytes per second, the unit of the GPU figure; the time of the
    benchmark's whole step at that rate is an extrapolation and labelled so.  Also timed in
    full: the single 4096x4096 linear layer at 25 % kept with 4 extra columns."""
    import multiprocessing as mp
    import numpy as np
    import synth
    from oracle import cassandra_oracle as O
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    nproc = min(nproc, int(os.environ.get("OMP_NUM_THREADS", nproc)) or nproc)
    r1, el1, nbytes = _cpu_worker((keep, t, k, ctx_len, 4.0))
    single = nbytes * r1 / el1 / 1e9
    ctxm = mp.get_context("spawn")
    with ctxm.Pool(nproc) as pool:
        res = pool.map(_cpu_worker, [(keep, t, k, ctx_len, 6.0)] * nproc)
    allc = sum(nb * r / el for r, el, nb in res) / 1e9
    # the single-linear-layer workload in full, one thread
    import threadpoolctl
    with threadpoolctl.threadpool_limits(1):
        W = synth.weight_matrix(4096, 4096, seed=1)
        X = synth.activations(4096, 5, seed=2)
        p = O.encode_weight(W, 250, 4)
        t0 = time.perf_counter(); O.gemv_draft(p, X[0]); td = time.perf_counter() - t0
        t0 = time.perf_counter(); O.gemm_verify(p, X); tv = time.perf_counter() - t0
    return {"value": allc, "unit": "GB/s", "cores": int(nproc), "kind": "oracle",
            "nproc": int(nproc), "single_thread_value": single,
            "sample": f"per repetition one draft pass + one verification pass ({k + 1} columns) over 256 output rows "
                      f"of each 8B-shaped layer matrix (3 x 256x4096, 256x14336) and the cache of one kv head over "
                      f"{ctx_len} positions (4 query heads), keep {keep}/1000, t={t}; `value`: {nproc} single-threaded "
                      f"processes, each on its own copy, {sum(r for r, _, _ in res)} repetitions in "
                      f"{max(el for _, el, _ in res):.1f} s; `single_thread_value`: one process, {r1} repetitions "
                      f"in {el1:.1f} s; algorithmic stream bytes / wall time",
            "single_linear_layer_4096x4096_keep250_k4_one_thread": {"draft_gemv_s": td, "verify_gemm_5col_s": tv}}


def cpu_units(keep, t):
    """`bench.py --workload cpu-units` (host only, minutes): the oracle's time for the units the
    default run only samples.  (1) the single 4096 x 4096 linear layer at 25 % kept, one draft GEMV
    and one verify GEMM with 4 extra columns; (2) one Llama-3-8B-shaped decoder layer (512-row
    output head) over 4096 cached positions, draft length 4: one draft step and one verification
    step of 5 columns, each from the packed streams (decoding them is part of the step; encoding
    is offline and not timed); (3) the 32-layer model per generated token, EXTRAPOLATED from (2).
    Each with one thread and with the BLAS threads the host offers."""
    import numpy as np
    import threadpoolctl
    import synth
    from oracle import cassandra_oracle as O
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    out = {"nproc": int(nproc), "kind": "oracle", "units": {}}
    W = synth.weight_matrix(4096, 4096, seed=1)
    X = synth.activations(4096, 5, seed=2)
    p1 = O.encode_weight(W, 250, 4)
    k, L = 4, 4096
    shape = synth.LlamaShape("llama3-8b-1l", 4096, 1, 32, 8, 128, 14336, 512)
    weights = synth.model_weights(shape, seed=3)
    tab = synth.rope_table(L + 64, shape.head_dim, shape.rope_theta)
    K = synth.kv_tensor(L, shape.n_kv_heads, 128, seed=21, outlier_channels=4)
    V = synth.kv_tensor(L, shape.n_kv_heads, 128, seed=22, outlier_channels=0)
    pk, pv = O.encode_kv(K.reshape(-1, 128), keep, t), O.encode_kv(V.reshape(-1, 128), keep, t)
    om0 = O.OracleModel(shape, weights, tab, w_keep=keep, w_t=t, kv_keep=keep, kv_t=t)
    print("encoded (untimed)", file=sys.stderr, flush=True)
    tokens = synth.token_ids(k + 1, shape.vocab, seed=9)
    empty = [(np.zeros((0, shape.n_kv_heads, 128), np.uint16),) * 2]
    for label, limit in (("one_thread", 1), ("all_threads", None)):
        ctxm = threadpoolctl.threadpool_limits(limit) if limit else threadpoolctl.threadpool_limits(nproc)
        with ctxm:
            t0 = time.perf_counter(); O.gemv_draft(p1, X[0]); t1 = time.perf_counter(); O.gemm_verify(p1, X)
            t2 = time.perf_counter()
            res = {"single_linear_layer_4096x4096_keep250": {"draft_gemv_s": t1 - t0, "verify_gemm_5col_s": t2 - t1}}
            step = {}
            for draft in (True, False):
                om0._dec = {}                       # every step decodes the packed streams itself
                t0 = time.perf_counter()
                dec = O.decode_draft if draft else O.decode_full
                view = (dec(pk).reshape(K.shape), dec(pv).reshape(V.shape))
                om0._cache_kv = lambda layer_index, d, view=view: view
                om0.cache_len = lambda: L
                if draft:
                    om0.forward(tokens[:1], draft=True, extra_kv=empty)
                else:
                    om0.forward(tokens, draft=False)
                step["draft_step_s" if draft else "verify_step_5col_s"] = time.perf_counter() - t0
            res["one_8b_layer_ctx4096_k4"] = step
            res["model_32_layers_per_round_k4_EXTRAPOLATED_s"] = 32 * (4 * step["draft_step_s"] + step["verify_step_5col_s"])
            out["units"][label] = res
        print(label, "done", file=sys.stderr, flush=True)
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures the one-GPU path only: run with --gpus 1 "
              "(no multi-GPU figure is produced in this build)", file=sys.stderr)
        sys.exit(2)
    if args.workload == "cpu-units":
        cpu_units(args.keep, args.trunc)
        return
    # the CPU oracle first: its worker processes are spawned before this process touches the GPU
    cpu = None if args.no_cpu_baseline or args.workload.startswith("probe") or args.workload in ("tune", "exp-modes") else \
        cpu_baseline(args.keep, args.trunc, args.k, args.context)
    import torch
    from paper_2605_26558_amd import binding as B
    from paper_2605_26558_amd import workload

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload.startswith("probe"):
        workload.run_probe(B, args)
        return
    if args.workload == "exp-modes":
        workload.run_exp_modes(B, args, dev)
        return
    if args.workload == "tune":
        workload.run_tune(B, args, dev)
        return
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
    if cpu is not None:
        # time of this benchmark's whole step at the oracle's sampled rate (an extrapolation)
        cpu["extrapolated_s_per_step_all_cores"] = wl.bytes_per_step / (cpu["value"] * 1e9)
        cpu["extrapolated_s_per_step_single_thread"] = wl.bytes_per_step / (cpu["single_thread_value"] * 1e9)
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
