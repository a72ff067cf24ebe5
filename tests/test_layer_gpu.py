"""The steps around one linear call, on the GPU and through the C-ABI:

* all seven projections of a Llama3.1-8B layer at 64 decode rows (the benchmark's layer configuration), in the four
  launches the benchmark uses (q/k/v as one group, o, gate/up as one group, down), captured in ONE HIP graph and
  replayed (Sec. 4.3 of the paper computes base model and adapters of a batch in one graph; Sec. 5.3 lists the
  projections the adapters target);
* adaptive adapter selection feeding the memory cache, the pool and the linear call (Algorithm 1 of the paper after
  the router, with synthetic confidence scores; Sec. 3.3 / 4.2 for cache and pool): select -> acquire -> load -> linear,
  every batch's y against the oracle with the adapters the oracle's own selection names.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_harness import DEV, DeviceCase, assert_close, rel_err, to_dev, y_to_f64
from oracle.cache_oracle import LruCacheOracle, select_adapter
from paper_2507_01438_amd import inputs as I

pytestmark = pytest.mark.gpu

LAUNCHES = [("q", "k", "v"), ("o",), ("gate", "up"), ("down",)]


def test_config3_layer_in_one_hip_graph():
    from paper_2507_01438_amd import binding as B
    w = I.config3()
    used = w.distinct_adapters()
    cases = {n: DeviceCase(w, I.LLAMA8B[n], load_slots=used) for g in LAUNCHES for n in g}
    arrays = [B.desc_array([cases[n].desc() for n in g]) for g in LAUNCHES]
    for arr, g in zip(arrays, LAUNCHES):
        if len(g) > 1:
            assert B.elora_linear_group_launches(arr) == 1, g

    def enqueue(stream):
        for arr, g in zip(arrays, LAUNCHES):
            if len(g) == 1:
                B.elora_batched_lora_linear(arr[0], stream=stream)
            else:
                B.elora_batched_lora_linear_group(arr, stream=stream)

    enqueue(None)  # outside the capture: one-time set-up of every kernel instance happens here
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        enqueue(side)
    rng = np.random.default_rng(17)
    cols = {n: np.unique(np.concatenate([rng.choice(c.proj.N, 96, replace=False), np.arange(8), np.arange(c.proj.N - 8, c.proj.N)]))
            for n, c in cases.items()}
    eager = {}
    for rep in range(3):
        if rep > 0:
            # new activations in place (the captured descriptors keep pointing at the same buffers)
            for n, c in cases.items():
                xn = I.f32_to_bf16_bits((rng.standard_normal(c.x_h.shape) * (0.5 + rep)).astype(np.float32))
                c.x_h = xn
                c.x.copy_(to_dev(xn))
        for c in cases.values():
            c.y.fill_(7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = {n: y_to_f64(c.y[: w.T], w.dtype) for n, c in cases.items()}
        for n, c in cases.items():
            e = assert_close(got[n][:, cols[n]], c.reference(cols=cols[n]), c.base_reference(cols=cols[n]), f"replay {rep}, {n}")
            if rep == 0:
                print(f"layer graph: {n:4s} rel err {e:.2e}")
        # eager work on the same workspaces between the replays: the same bits (fixed summation order)
        for c in cases.values():
            c.y.fill_(7)
        enqueue(None)
        torch.cuda.synchronize()
        for n, c in cases.items():
            np.testing.assert_array_equal(got[n], y_to_f64(c.y[: w.T], w.dtype))
    for c in cases.values():
        assert c.pool.poll_error() == (0, -1)
        c.close()


@pytest.mark.parametrize("k", [1, 3])
def test_selection_cache_pool_and_linear_call_in_a_row(k):
    from paper_2507_01438_amd import binding as B
    n_adapters, capacity, rows, n_batches, K, N = 40, 6, 6, 40, 512, 384
    w = I.small_workload(95, I.BF16, K, N, rows, n_adapters, (16, 8, 32))
    proj = w.projections[0]
    x_h, (W_h, _) = w.x(proj), w.W(proj)
    host = [w.adapter(proj, a) for a in range(n_adapters)]
    dev = [(to_dev(A), to_dev(Bm)) for A, Bm, _ in host]
    ref_adapters = [oracle.Adapter(A, Bm, s) for A, Bm, s in host]
    x, W = to_dev(x_h), to_dev(W_h)
    pool = B.AdapterPool(K, N, w.max_rank, capacity, I.BF16, DEV)
    lin = B.LoraLinear(K, N, I.BF16, pool, rows, DEV)
    cache, model = B.elora_cache_create(capacity), LruCacheOracle(capacity)
    # synthetic router: every prompt has three suitable adapters out of a popular few, scored high, the rest low
    rng = np.random.default_rng(96)
    popular = I.request_trace(97, n_adapters, 1.0, n_batches * rows * 3).reshape(n_batches, rows, 3)
    y = torch.zeros((rows, N), dtype=torch.int16, device=DEV)
    slots_h, miss_ids, miss_slots = (np.zeros(rows, np.int32) for _ in range(3))
    worst, resident_picks, loads = 0.0, 0, 0
    for b in range(n_batches):
        chosen = np.zeros(rows, np.int32)
        for t in range(rows):
            scores = (rng.random(n_adapters) * 0.3).astype(np.float32)
            scores[popular[b, t]] = 0.7 + 0.3 * rng.random(3).astype(np.float32)
            explicit = int(popular[b, t, 0]) if (b + t) % 9 == 0 else -1       # some requests name their adapter
            got, resident = B.elora_cache_select(cache, explicit, scores, k)
            want = select_adapter(model.block, explicit, scores, k)
            assert got == want and resident == (want in model.block)
            chosen[t] = got
            resident_picks += int(resident)
        # more distinct adapters than blocks cannot happen here (rows == capacity)
        n_miss = B.elora_cache_acquire_batch(cache, chosen, slots_h, miss_ids, miss_slots)
        want_slots, want_miss = model.acquire_batch(chosen)
        assert slots_h.tolist() == want_slots
        assert list(zip(miss_ids[:n_miss].tolist(), miss_slots[:n_miss].tolist())) == want_miss
        if n_miss:
            m = miss_ids[:n_miss].tolist()
            B.elora_pool_load_adapters(pool.handle, miss_slots[:n_miss].tolist(), [host[a][0].shape[0] for a in m],
                                       [host[a][2] for a in m], [dev[a][0] for a in m], [dev[a][1] for a in m])
            loads += n_miss
        lin(x, W, y, adapter_idx=to_dev(slots_h))
        torch.cuda.synchronize()
        ref = oracle.linear(I.BF16, x_h, W_h, ref_adapters, chosen)
        worst = max(worst, rel_err(y_to_f64(y, I.BF16), ref))
        B.elora_cache_release_batch(cache, chosen)
        for a in chosen:
            assert model.release(int(a))
    hits, requests, evictions = B.elora_cache_stats(cache)
    assert (hits, requests, evictions) == (model.hits, model.requests, model.evictions)
    assert loads == requests - hits and evictions > 0
    assert pool.poll_error() == (0, -1)
    print(f"selection chain k={k}: hit rate {hits / requests:.2f}, {resident_picks} of {n_batches * rows} picks resident, "
          f"{loads} loads, worst rel err {worst:.2e}")
    assert worst <= 1e-2
    B.elora_cache_destroy(cache)
    pool.close()
