#!/usr/bin/env python3
"""Benchmark of the batched multi-adapter LoRA linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--layers L]

A step is one pass of the whole hot path (route + shrink + base + expand +
combine, i.e. one elora_batched_lora_linear call) over one synthetic batch.
The default workload is the Llama3.1-8B q_proj decode configuration (bf16,
32 tokens, 64 rank-16 adapters, power-law(1.1) adapter popularity).  Inputs
are resident in HBM before the timed region.  To keep the 256 MB last-level
cache from serving the weights, consecutive steps rotate through `--layers`
distinct copies of (W, adapter pool, x), like the layers of a model do.

Prints ONE JSON line: throughput of the whole job plus
  roofline     the dominant kernel's algorithmic bytes / its duration measured
               with HIP events around each of its launches, against 8 TB/s
  cpu_baseline the fp64 oracle timed on this machine's host cores
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=2, choices=[2])
    ap.add_argument("--layers", type=int, default=32, help="distinct (W, pool, x) copies the steps rotate through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2507_01438_amd import build as elora_build
    if elora_build.is_stale() and not os.path.exists(elora_build.LIB):
        elora_build.build()
    from paper_2507_01438_amd import binding as B
    from paper_2507_01438_amd import inputs as I
    from gpu_harness import DeviceCase, rel_err, to_dev, y_to_f64

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = I.CONFIGS[args.config]()
    proj = w.projections[0]
    L = max(1, args.layers)

    # layer 0 from the seeded generators; the other layers are device copies of the same bytes at
    # different addresses (what matters to the caches), so every layer's output can be checked
    case = DeviceCase(w, proj)
    Ws = [case.W] + [case.W.clone() for _ in range(L - 1)]
    xs = [case.x] + [case.x.clone() for _ in range(L - 1)]
    dev_adapters = {i: (to_dev(A), to_dev(Bm), sc) for i, (A, Bm, sc) in case.adapters.items()}
    pools = [case.pool]
    for _ in range(L - 1):
        p = B.AdapterPool(proj.K, proj.N, w.max_rank, w.pool, w.dtype, dev)
        for i, (A_d, B_d, sc) in dev_adapters.items():
            p.load(i, A_d, B_d, sc)
        pools.append(p)
    ys = [torch.zeros_like(case.y) for _ in range(L)]
    lins = [B.LoraLinear(proj.K, proj.N, w.dtype, pools[l], w.T, dev) for l in range(L)]
    idx = case.adapter_idx
    descs = [lins[l].desc(xs[l], Ws[l], ys[l], adapter_idx=idx) for l in range(L)]
    torch.cuda.synchronize()
    plan = B.elora_linear_plan(descs[0])
    stream = torch.cuda.current_stream().cuda_stream

    def step(i):
        B.lib.elora_batched_lora_linear(descs[i % L], stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.T * args.steps / (t1 - t0)

    # second pass over the same steps with HIP events around every launch of the dominant kernel
    n_prof = min(args.steps, 2000)
    B.elora_profile_arm(n_prof)
    for i in range(n_prof):
        step(i)
    torch.cuda.synchronize()
    kern_ms = np.array(B.elora_profile_read(n_prof))
    B.elora_profile_arm(0)
    kern_us = float(np.mean(kern_ms) * 1e3)
    kern_us_med = float(np.median(kern_ms) * 1e3)

    # hot-cache variant (one buffer set), reported separately
    for i in range(50):
        B.lib.elora_batched_lora_linear(descs[0], stream)
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    for i in range(args.steps):
        B.lib.elora_batched_lora_linear(descs[0], stream)
    torch.cuda.synchronize()
    hot_ms = (time.perf_counter() - h0) * 1e3 / args.steps

    # algorithmic bytes: W once, x once, y once, used rows (r_i, not max_rank) of each distinct adapter once.
    # The decode path is a single kernel, so the dominant kernel carries all of them.
    distinct = w.distinct_adapters()
    bytes_call = w.algorithmic_bytes(proj)
    bytes_dom = bytes_call
    achieved = bytes_dom / (kern_us * 1e-6) / 1e9
    flops = w.algorithmic_flops(proj)

    check = None
    if not args.no_check:
        ref = case.reference()
        errs = [rel_err(y_to_f64(ys[l][: w.T], w.dtype), ref) for l in (0, L // 2, L - 1)]
        check = max(errs)
        assert check <= 1e-2, f"parity lost in the benchmark configuration: {errs}"
        assert all(p.poll_error() == (0, -1) for p in (pools[0], pools[-1]))

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ads = case.oracle_adapters()
        ra = w.row_adapter()
        oracle.linear(w.dtype, case.x_h, case.W_h, ads, ra)  # warm (also compiles the C file if needed)
        c0 = time.perf_counter()
        reps, used = 0, 1
        while time.perf_counter() - c0 < 12.0:
            _, used = oracle.linear(w.dtype, case.x_h, case.W_h, ads, ra, return_threads=True)
            reps += 1
        cdt = time.perf_counter() - c0
        cpu = {"value": w.T * reps / cdt, "unit": "tokens/s", "cores": int(used), "kind": "oracle",
               "sample": f"{reps} full batches of {w.T} tokens of the same workload, {cdt:.1f} s"}

    out = {
        "metric": "batched_lora_linear_tokens_per_s",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "Llama3.1-8B q_proj decode: W 4096x4096 bf16, 32 tokens, pool 64 adapters rank 16, "
                        "adapter_idx power-law(1.1), scale 2.0",
            "n_tokens": w.T, "d_in": proj.K, "d_out": proj.N, "distinct_adapters": int(len(distinct)),
            "rotating_layers": L, "path": int(plan.path), "split_k": int(plan.split_k), "grid": int(plan.grid),
            "launches_per_step": int(plan.n_launches),
        },
        "tflops": flops / (ms_per_step * 1e-3) / 1e12,
        "step_gbs": bytes_call / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": bytes_call / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "hot_cache_ms_per_step": hot_ms,
        "max_rel_err_vs_oracle": check,
        "roofline": {
            "bound": "hbm", "kernel": "decode_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": None,
            "bytes_per_launch": int(bytes_dom), "avg_us": kern_us, "median_us": kern_us_med,
            "launches_timed": int(len(kern_ms)), "bytes_per_step_all_kernels": int(bytes_call),
        },
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
