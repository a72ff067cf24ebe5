#!/usr/bin/env python3
"""Benchmark of the batched multi-adapter LoRA linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {2,3,4,5}]

A step is one pass of the whole hot path (route + shrink + base + expand +
combine, i.e. elora_batched_lora_linear) over one synthetic batch, for every
projection the configuration names:

  config 3 (the headline: top-level value, roofline, cpu_baseline; --steps and --warmup apply to it):
           the seven projections of a Llama3.1-8B layer, 64 decode tokens, 256 adapters of mixed rank
  config 2 Llama3.1-8B q_proj decode, bf16, 32 tokens, 64 rank-16 adapters, power-law(1.1) popularity
  config 4 prefill segments (16 prompts, ~8k rows), gate / up / down projections
  config 5 mixed prefill + decode batch on a 4-bit base, gate projection

Without --config the line also carries per_config records for 2, 4 and 5 (the metric has two halves: achieved
HBM GB/s for the decode configurations, MFMA % of peak for the prefill ones), each with its own roofline,
ms_per_step, parity figure and cpu_baseline.  --config N runs configuration N alone as the line's top level.

Inputs are resident in HBM before the timed region.  For the decode configs
consecutive steps rotate through several distinct copies of the weights and
pools (like the layers of a model do) so that the 256 MB last-level cache
cannot serve them.  Set-up runs the step on every copy once and keeps the
device busy for 30 ms, so that short runs (--steps 20 --warmup 5 is under
5 ms of device time) measure the device at its working clocks rather than on
its way out of idle; then come the W warm-up steps and the K timed steps.

Prints ONE JSON line: throughput of the whole job plus
  roofline     the dominant kernel's algorithmic bytes (decode) or flops
               (prefill) per launch / its launch duration from HIP events on the
               launch stream, against 8 TB/s or 2.5 PFLOP/s
  cpu_baseline the fp64 oracle timed on this machine's host cores on a bounded sample
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
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled by what
# the same counter reads for a 1 GiB device copy on the same box (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).  Figures
# and commands: the files named here.  None = not measured for that configuration.
TRAFFIC = {
    2: (46.0e6, "profiles/decode_kernel_config2.md"),
    3: (209.9e6, "profiles/decode_kernels_config3.md"),
    4: (1.86e9, "profiles/lora_gemm_kernel_config4.md"),
    5: (0.69e9, "profiles/lora_gemm_kernel_config5.md"),
}
WORKLOAD = {
    2: "Llama3.1-8B q_proj decode: W 4096x4096 bf16, 32 tokens, pool 64 adapters rank 16, adapter_idx power-law(1.1), scale 2.0",
    3: "Llama3.1-8B layer decode: q,k,v,o,gate,up,down bf16, 64 tokens, pool 256 adapters ranks {8,16,32,64}, uniform adapter_idx",
    4: "Llama3.1-8B prefill segments: 16 prompts U{64..1024} rows, rank-32 adapters from a pool of 128, gate/up/down bf16",
    5: "mixed batch 4x512 prefill + 120 decode rows, W 4096x14336 4-bit g32 fp16 scales, pool 1024 adapters rank 16, power-law(1.0)",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=None, choices=[2, 3, 4, 5],
                    help="only this configuration (default: config 3 as the headline, then 2, 4 and 5 as per_config records)")
    ap.add_argument("--headline-only", action="store_true", help="config 3 alone, without the per_config records")
    ap.add_argument("--layers", type=int, default=None, help="distinct (W, pool, x) copies the decode steps rotate through")
    ap.add_argument("--no-groups", action="store_true",
                    help="config 3: one launch per projection instead of one for q/k/v and one for gate/up")
    ap.add_argument("--w8-base", action="store_true",
                    help="keep the base weight in 8-bit groups of 32 (int8 codes, fp16 scales) instead of bf16 (configs 2, 3, 4)")
    ap.add_argument("--q8-adapters", action="store_true",
                    help="every adapter kept in 8-bit blocks in the pool (the paper's adapter "
                         "storage): a line of its own, not the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--cache-trace", action="store_true",
                    help="instead of the headline metric: config 2's decode call behind the adapter cache, with misses "
                         "loaded from pinned host memory (one JSON line of its own)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that profiler byte counters can be scaled")
    return ap.parse_args()


def cache_trace(args, B, I, dev):
    """Config 2's call (q_proj, 32 rows, rank 16) with the adapter memory manager in front of it (Sec. 3.3 / 4.2):
    requests follow a power law over a universe of adapters held in pinned host memory, the pool has config 2's 64
    blocks, every row's adapter goes through the LRU cache, misses are loaded into their blocks.  Three legs over the
    same request trace: everything resident (a pool as large as the universe), misses loaded on a second stream
    (overlapping the linear calls of earlier batches), misses loaded on the compute stream."""
    import ctypes
    import numpy as np
    import torch
    from gpu_harness import to_dev

    universe, capacity, alpha, rows, K, N, rank = 512, 64, 1.1, 32, 4096, 4096, 16
    steps = args.steps if args.steps is not None else 2000
    warmup = args.warmup if args.warmup is not None else 200
    w = I.small_workload(7, I.BF16, K, N, rows, universe, (rank,), alpha=alpha)
    proj = w.projections[0]
    x, W = to_dev(w.x(proj)), to_dev(w.W(proj)[0])
    host, host_q8 = [], []
    for a in range(universe):
        A, Bm, sc = w.adapter(proj, a)
        host.append((torch.from_numpy(A.view(np.int16)).pin_memory(), torch.from_numpy(Bm.view(np.int16)).pin_memory(), sc))
        Ac, As = I.quantize_q8_blocks(I.bf16_bits_to_f32(A))
        Bc, Bs = I.quantize_q8_blocks(I.bf16_bits_to_f32(Bm))
        host_q8.append(tuple(torch.from_numpy(t.view(np.int8 if t.dtype == np.int8 else np.int16)).pin_memory()
                             for t in (Ac, As, Bc, Bs)))
    trace = I.request_trace(8, universe, alpha, (warmup + steps) * rows).reshape(warmup + steps, rows).astype(np.int32)
    comp = torch.cuda.Stream()
    copy = torch.cuda.Stream()

    def leg(n_blocks, copy_stream, q8=False):
        pool = B.AdapterPool(K, N, rank, n_blocks, I.BF16, dev)
        lin = B.LoraLinear(K, N, I.BF16, pool, rows, dev)
        y = torch.zeros((rows, N), dtype=torch.int16, device=dev)
        n_all = warmup + steps
        idx_dev = torch.zeros((n_all, rows), dtype=torch.int32, device=dev)
        idx_pin = torch.zeros((n_all, rows), dtype=torch.int32).pin_memory()
        idx_np = idx_pin.numpy()
        descs = [lin.desc(x, W, y, adapter_idx=idx_dev[i]) for i in range(n_all)]
        cache = B.elora_cache_create(n_blocks)
        miss_ids, miss_slots = np.zeros(rows, np.int32), np.zeros(rows, np.int32)
        n_miss = ctypes.c_int()
        miss_slots_p = miss_slots.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
        pa, pb = (ctypes.c_void_p * rows)(), (ctypes.c_void_p * rows)()
        ranks_c, scales_c = (ctypes.c_int * rows)(*[rank] * rows), (ctypes.c_float * rows)(*[host[0][2]] * rows)
        a_ptr, b_ptr = [h[0].data_ptr() for h in host], [h[1].data_ptr() for h in host]
        q_ptr = [[h[k].data_ptr() for h in host_q8] for k in range(4)]
        pq = [(ctypes.c_void_p * rows)() for _ in range(4)]
        cs, ps = copy_stream.cuda_stream, comp.cuda_stream
        torch.cuda.synchronize()
        loads = 0
        t0 = None
        with torch.cuda.stream(comp):
            for i in range(n_all):
                if i == warmup:
                    torch.cuda.synchronize()
                    B.elora_cache_reset_stats(cache)
                    loads = 0
                    t0 = time.perf_counter()
                ids, slots = trace[i], idx_np[i]
                rc = B.lib.elora_cache_acquire_batch(cache, ids.ctypes.data, rows, slots.ctypes.data, miss_ids.ctypes.data,
                                                     miss_slots.ctypes.data, ctypes.byref(n_miss))
                assert rc == 0, rc
                nm = n_miss.value
                if nm:
                    B.lib.elora_cache_load_begin(cache, miss_slots_p, nm, cs)
                    if q8:
                        for m in range(nm):
                            for k in range(4):
                                pq[k][m] = q_ptr[k][miss_ids[m]]
                        rc = B.lib.elora_pool_load_adapters_q8(pool.handle, nm, miss_slots.ctypes.data, ranks_c, scales_c, *pq, cs)
                    else:
                        for m in range(nm):
                            pa[m], pb[m] = a_ptr[miss_ids[m]], b_ptr[miss_ids[m]]
                        rc = B.lib.elora_pool_load_adapters(pool.handle, nm, miss_slots.ctypes.data, ranks_c, scales_c, pa, pb, cs)
                    assert rc == 0, rc
                    B.lib.elora_cache_load_end(cache, miss_slots_p, nm, cs)
                loads += nm
                B.lib.elora_cache_batch_begin(cache, slots.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), rows, ps)
                idx_dev[i].copy_(idx_pin[i], non_blocking=True)
                rc = B.lib.elora_batched_lora_linear(descs[i], ps)
                assert rc == 0, rc
                B.lib.elora_cache_batch_end(cache, slots.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), rows, ps)
                B.lib.elora_cache_release_batch(cache, ids.ctypes.data, rows)
            torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        hits, requests, evictions = B.elora_cache_stats(cache)
        bad = pool.poll_error()
        B.elora_cache_destroy(cache)
        pool.close()
        return {"tokens_per_s": rows * steps / dt, "us_per_step": dt / steps * 1e6, "hit_rate": hits / requests,
                "loads_per_step": loads / steps, "evictions": evictions, "bad_rows": bad[0]}

    resident = leg(universe, copy)
    overlapped = leg(capacity, copy)
    serial = leg(capacity, comp)
    overlapped_q8 = leg(capacity, copy, q8=True)
    adapter_bytes = 2 * rank * (K + N)
    out = {"metric": "cached_decode_tokens_per_s", "value": overlapped["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": overlapped["us_per_step"] / 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"config 2's call behind the adapter cache: {universe} rank-{rank} adapters in pinned host "
                                  f"memory ({adapter_bytes} bytes each), {capacity} blocks, requests power-law({alpha}), "
                                  f"{rows} rows per step; host loop in Python"},
           "all_resident": resident, "loads_on_copy_stream": overlapped, "loads_on_compute_stream": serial,
           "loads_of_8bit_blocks_on_copy_stream": overlapped_q8}
    print(json.dumps(out))


def run_config(cfg, steps, warmup, args, B, I, dev, cpu_seconds):
    """One configuration: set-up, `warmup` untimed steps, exactly `steps` timed steps, parity check in the timed
    launch configuration, the oracle on the host cores.  Returns the record (a dict)."""
    import numpy as np
    import torch
    from gpu_harness import DeviceCase, rel_err, to_dev, y_to_f64

    decode = cfg in (2, 3)
    q8 = bool(args.q8_adapters)
    w = I.CONFIGS[cfg]()
    if args.w8_base:
        assert w.wfmt == I.W_SAME and w.dtype == I.BF16, "--w8-base: configurations with a bf16 base (2, 3, 4)"
        w.wfmt = I.W_INT8_G32
    projs = w.projections
    distinct = w.distinct_adapters()

    # One DeviceCase per projection from the seeded generators (only the adapters the batch uses are
    # generated for the big pools).  Decode: further "layers" are device copies of the same bytes at other
    # addresses (what matters to the caches), so every layer's output can be checked against the oracle.
    # Projections with the same d_in read the same activations: their cases share one device copy of x and of the routing
    # tables (what lets a group of them share work).
    cases = []
    for p in projs:
        first = next((c for c in cases if c.proj.K == p.K), None)
        cases.append(DeviceCase(w, p, load_slots=None if cfg == 2 else distinct, share=first, q8=q8))
    layer_bytes = sum(p.N * p.K * 2 for p in projs)
    L = args.layers if args.layers is not None else (max(2, min(32, int(1.6e9 // layer_bytes))) if decode else 1)
    layers = []  # layers[l][pi] = descriptor
    keep = []
    dev_adapters = [{i: tuple(to_dev(t) if isinstance(t, np.ndarray) else t for t in ad) for i, ad in case.adapters.items()}
                    if L > 1 else {} for case in cases]
    for l in range(L):
        descs = []
        x_of = {}  # this layer's copy of x per d_in
        for pi, (p, case) in enumerate(zip(projs, cases)):
            if l == 0:
                descs.append(case.desc())
                continue
            if p.K not in x_of:
                x_of[p.K] = case.x.clone()
            Wc, xc, yc = case.W.clone(), x_of[p.K], torch.zeros_like(case.y)
            pool = B.AdapterPool(p.K, p.N, w.max_rank, w.pool, w.dtype, dev, q8=q8)
            for i, ad in dev_adapters[pi].items():
                if q8:
                    Ac, Bc, sc, As, Bs = ad
                    B.elora_pool_load_adapters_q8(pool.handle, [i], [Ac.shape[0]], [sc], [Ac], [As], [Bc], [Bs])
                else:
                    pool.load(i, ad[0], ad[1], ad[2])
            lin = B.LoraLinear(p.K, p.N, w.dtype, pool, w.T, dev, wfmt=w.wfmt)
            keep += [Wc, xc, yc, pool, lin]
            descs.append(lin.desc(xc, Wc, yc, adapter_idx=case.adapter_idx, seg_offsets=case.seg_offsets,
                                  seg_adapter=case.seg_adapter, wfmt=w.wfmt, w_scales=case.w_scales))
        layers.append(descs)
    torch.cuda.synchronize()
    plans = [B.elora_linear_plan(d) for d in layers[0]]
    stream = torch.cuda.current_stream().cuda_stream
    n_proj = len(projs)
    # Projections that are due at the same time go out as one launch (config 3: q/k/v and gate/up).
    names = [p.name for p in projs]
    group_names = [g for g in (("q", "k", "v"), ("gate", "up")) if all(n in names for n in g)] if not args.no_groups else []
    units = []  # per launch of a step: the projection indices it covers
    for pi, n in enumerate(names):
        g = next((g for g in group_names if n in g), None)
        if g is None:
            units.append([pi])
        elif n == g[0]:
            units.append([names.index(m) for m in g])
    layer_calls = []  # layer_calls[l] = [(descriptor array, n)] per launch
    for descs in layers:
        layer_calls.append([(B.desc_array([descs[pi] for pi in u]), len(u)) for u in units])
    for arr, n in layer_calls[0]:
        if n > 1 and decode:
            assert B.elora_linear_group_launches(arr) == 1, "these projections were expected to share a launch"
        elif n > 1:
            assert B.elora_linear_group_launches(arr) == 2 + n, "these projections were expected to share route and shrink"
    n_launch = len(units)

    def step(i):
        for arr, n in layer_calls[i % L]:
            if n == 1:
                B.lib.elora_batched_lora_linear(arr, stream)
            else:
                B.lib.elora_batched_lora_linear_group(arr, n, stream)

    # set-up: every rotating copy is touched once (first use of its pages), whatever the number of warm-up steps, and the
    # device is kept busy for 30 ms, so that it has left its idle clocks before the warm-up steps start (five warm-up
    # steps of the layer are under a millisecond)
    t_setup = time.perf_counter()
    i = 0
    while i < L or time.perf_counter() - t_setup < 0.03:
        step(i)
        i += 1
        if i % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()  # on torch's current stream, the stream the kernels are launched on
    for i in range(steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    tokens_per_s = w.T * steps / (t1 - t0)
    region_us_per_launch = ev0.elapsed_time(ev1) * 1e3 / (steps * n_launch)

    flops_step = sum(w.algorithmic_flops(p) for p in projs)
    bytes_step = sum(w.algorithmic_bytes(p, q8_adapters=q8) for p in projs)
    if decode:
        # The decode path is one kernel per call and the launches run back to back, so the device time of the
        # timed region (HIP events on the launch stream) divided by the number of launches is the kernel's average
        # launch duration.
        assert all(pl.n_launches == 1 for pl in plans)
        kern_us = region_us_per_launch
        achieved = bytes_step / n_launch / (kern_us * 1e-6) / 1e9
        roofline = {"bound": "hbm", "kernel": "decode_kernel / decode_group_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "bytes_per_launch": int(bytes_step / n_launch), "avg_us": kern_us,
                    "launches_timed": int(steps * n_launch)}
    else:
        # one pair of HIP events around every launch of each call's dominant kernel (second pass over the same steps;
        # an event pair costs a few microseconds against launches of hundreds)
        # (every projection has one GEMM launch, also where projections share their route and shrink launches)
        n_prof = min(steps, 1000)
        B.elora_profile_arm(n_prof * n_proj)
        for i in range(n_prof):
            step(i)
        torch.cuda.synchronize()
        per_launch_us = np.array(B.elora_profile_read(n_prof * n_proj)).reshape(n_prof, n_proj) * 1e3
        B.elora_profile_arm(0)
        kern_us = float(per_launch_us.mean())
        achieved = flops_step / n_proj / (kern_us * 1e-6) / 1e12
        roofline = {"bound": "mfma", "kernel": "lora_gemm_kernel", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                    "flops_per_launch": int(flops_step / n_proj), "avg_us": kern_us,
                    "launches_timed": int(per_launch_us.size)}
    traffic, traffic_src = TRAFFIC.get(cfg, (None, None))
    roofline["traffic"] = traffic
    roofline["traffic_source"] = traffic_src

    # parity in the launch configuration that was timed (sampled outputs for the big shapes)
    check = None
    rng = np.random.default_rng(1)
    if not args.no_check:
        errs = []
        for pi, (p, case) in enumerate(zip(projs, cases)):
            y = y_to_f64(case.y[: w.T], w.dtype)
            if cfg == 2:
                errs.append(rel_err(y, case.reference()))
            else:
                cols = np.sort(rng.choice(p.N, 32, replace=False))
                rows = None if decode else np.sort(rng.choice(w.T, 128, replace=False))
                ysub = y[:, cols] if rows is None else y[np.ix_(rows, cols)]
                errs.append(rel_err(ysub, case.reference(rows=rows, cols=cols)))
            assert case.pool.poll_error() == (0, -1)
        check = max(errs)
        assert check <= 1e-2, f"parity lost in the benchmark configuration: {errs}"

    cpu = None
    if cpu_seconds > 0:
        import oracle
        case, p = cases[0], projs[0]
        ads = case.oracle_adapters()
        ra = w.adapter_idx if w.adapter_idx is not None else oracle.rows_from_segments(w.T, w.seg_offsets, w.seg_adapter)
        # bounded sample: whole rows of the first projection (all of them for config 2), repeated
        n_rows = w.T if cfg == 2 else min(w.T, 16)
        rows = None if cfg == 2 else np.arange(n_rows, dtype=np.int32)
        kw = dict(wfmt=w.wfmt, w_scales=case.ws_h, rows=rows)
        oracle.linear(w.dtype, case.x_h, case.W_h, ads, ra, **kw)  # warm (also compiles the C file if needed)
        c0 = time.perf_counter()
        reps, used = 0, 1
        while time.perf_counter() - c0 < cpu_seconds:
            _, used = oracle.linear(w.dtype, case.x_h, case.W_h, ads, ra, return_threads=True, **kw)
            reps += 1
        cdt = time.perf_counter() - c0
        # one projection was timed; a step runs n_proj of them with flops in proportion
        scale = w.algorithmic_flops(p) / flops_step
        cpu = {"value": n_rows * reps / cdt * scale, "unit": "tokens/s", "cores": int(used), "kind": "oracle",
               "sample": f"{reps} x {n_rows} full rows of projection '{p.name}' in {cdt:.1f} s"
                         + ("" if n_proj == 1 else f", scaled by its share of the step's flops ({scale:.3f})")}

    rec = {
        "value": tokens_per_s,
        "unit": "tokens/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "config": {
            "workload": WORKLOAD[cfg] + (" -- adapters kept in 8-bit blocks (int8 codes, fp16 scale per 32 values)" if q8 else "")
                        + (" -- base weight kept in 8-bit groups of 32 (int8 codes, fp16 scales)" if args.w8_base else ""),
            "config_number": cfg, "n_tokens": w.T, "projections": [p.name for p in projs],
            "distinct_adapters": int(len(distinct)), "rotating_layers": L,
            "path": [int(pl.path) for pl in plans], "split_k": [int(pl.split_k) for pl in plans],
            "tile_rows": [int(pl.tile_rows) for pl in plans],
            "grid": [int(pl.grid) for pl in plans], "launches_per_call": [int(pl.n_launches) for pl in plans],
            "launches_per_step": [[names[pi] for pi in u] for u in units],
        },
        "tflops": flops_step / (ms_per_step * 1e-3) / 1e12,
        "step_gbs": bytes_step / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "step_frac_of_mfma_peak": flops_step / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "max_rel_err_vs_oracle": check,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    for c in cases:
        c.close()
    del cases, layers, layer_calls, keep, dev_adapters
    torch.cuda.empty_cache()
    return rec


DEFAULT_STEPS = {2: 4000, 3: 300, 4: 20, 5: 40}
DEFAULT_WARMUP = {2: 200, 3: 30, 4: 3, 5: 5}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_01438_amd import build as elora_build
    if not os.path.exists(elora_build.LIB):
        elora_build.build()
    from paper_2507_01438_amd import binding as B
    from paper_2507_01438_amd import inputs as I

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.cache_trace:
        cache_trace(args, B, I, dev)
        return
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    # The headline is the layer decode configuration (config 3: the largest HBM-bound one, all seven projections);
    # --steps / --warmup apply to it.  Without --config the other configurations follow as records of their own
    # (config 2: the other half of the HBM figure; configs 4 and 5: the MFMA figure), each with its own step counts.
    head = args.config if args.config is not None else 3
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[head]
    warmup = args.warmup if args.warmup is not None else DEFAULT_WARMUP[head]
    def with_in_kernel_variant(cfg, r):
        """Config 5 names W "dequantized in-kernel": its record also carries the same call with W converted tile by tile
        inside the GEMM kernel (what the library does below 768 rows) instead of once per call into the workspace."""
        if cfg != 5 or args.w8_base:
            return r
        B.elora_debug_w4_copy_rows(1 << 30)
        try:
            v = run_config(5, max(10, DEFAULT_STEPS[5] // 4), 3, args, B, I, dev, 0)
        finally:
            B.elora_debug_w4_copy_rows(768)
        r["w_converted_tile_by_tile_in_the_gemm_kernel"] = {k: v[k] for k in ("ms_per_step", "value", "unit", "roofline", "max_rel_err_vs_oracle") if k in v}
        return r

    rec = with_in_kernel_variant(head, run_config(head, steps, warmup, args, B, I, dev, 0 if args.no_cpu_baseline else 12.0))
    out = {"metric": "batched_lora_linear_tokens_per_s", "value": rec["value"], "unit": rec["unit"], "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": rec["ms_per_step"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    out.update({k: v for k, v in rec.items() if k not in out})
    if args.config is None and not args.headline_only:
        out["per_config"] = {}
        for cfg in (2, 4, 5):
            r = with_in_kernel_variant(cfg, run_config(cfg, DEFAULT_STEPS[cfg], DEFAULT_WARMUP[cfg], args, B, I, dev, 0 if args.no_cpu_baseline else 4.0))
            r.update({"metric": "batched_lora_linear_tokens_per_s", "dtype": "bf16", "data": "synthetic"})
            out["per_config"][str(cfg)] = r
    print(json.dumps(out))


if __name__ == "__main__":
    main()
