"""The C++ adapter cache (host logic of libelora) against the oracle: bit-exact on seeded request traces.  No GPU."""
import numpy as np
import pytest

from oracle.cache_oracle import BUSY, LruCacheOracle
from paper_2507_01438_amd import inputs as I


@pytest.fixture(scope="module")
def B():
    from paper_2507_01438_amd import build
    if build.is_stale():
        build.build()
    from paper_2507_01438_amd import binding
    return binding


@pytest.mark.parametrize("seed,n_adapters,alpha,capacity", [(1, 50, 1.0, 8), (2, 200, 0.5, 16), (3, 30, None, 30),
                                                           (4, 30, 1.5, 1), (5, 1000, 1.0, 64)])
def test_traces_match_the_oracle_request_by_request(B, seed, n_adapters, alpha, capacity):
    trace = I.request_trace(seed, n_adapters, alpha, 4000)
    ref = LruCacheOracle(capacity)
    c = B.elora_cache_create(capacity)
    for a in trace:
        a = int(a)
        want = ref.acquire(a)
        ref.release(a)
        got = B.elora_cache_acquire(c, a)
        B.elora_cache_release(c, a)
        assert got == want, (a, got, want)
    assert B.elora_cache_stats(c) == (ref.hits, ref.requests, ref.evictions)
    for a in range(n_adapters):
        assert B.elora_cache_lookup(c, a) == ref.lookup(a)
    B.elora_cache_reset_stats(c)
    assert B.elora_cache_stats(c) == (0, 0, 0)
    B.elora_cache_destroy(c)


@pytest.mark.parametrize("seed", [7, 8, 9])
def test_random_mix_of_requests_releases_and_drops(B, seed):
    rng = np.random.default_rng(seed)
    capacity, n_adapters = 6, 14
    ref = LruCacheOracle(capacity)
    c = B.elora_cache_create(capacity)
    held = []   # outstanding requests
    for step in range(5000):
        op = rng.integers(0, 10)
        a = int(rng.integers(0, n_adapters))
        if op < 5:
            want = ref.acquire(a)
            if want[0] is None:
                with pytest.raises(B.EloraError) as e:
                    B.elora_cache_acquire(c, a)
                assert e.value.status == B.ELORA_E_BUSY
            else:
                assert B.elora_cache_acquire(c, a) == want
                held.append(a)
        elif op < 8 and held:
            a = held.pop(int(rng.integers(0, len(held))))
            assert ref.release(a)
            B.elora_cache_release(c, a)
        elif op == 8:
            want = ref.drop(a)
            if want is True:
                B.elora_cache_drop(c, a)
            else:
                with pytest.raises(B.EloraError) as e:
                    B.elora_cache_drop(c, a)
                assert e.value.status == (B.ELORA_E_BUSY if want == BUSY else B.ELORA_E_NOT_LOADED)
        else:
            assert B.elora_cache_lookup(c, a) == ref.lookup(a)
    assert B.elora_cache_stats(c) == (ref.hits, ref.requests, ref.evictions)
    B.elora_cache_destroy(c)


def test_argument_errors(B):
    with pytest.raises(B.EloraError):
        B.elora_cache_create(0)
    c = B.elora_cache_create(2)
    with pytest.raises(B.EloraError):
        B.elora_cache_acquire(c, -1)
    with pytest.raises(B.EloraError) as e:
        B.elora_cache_release(c, 5)
    assert e.value.status == B.ELORA_E_NOT_LOADED
    B.elora_cache_acquire(c, 5)
    B.elora_cache_release(c, 5)
    with pytest.raises(B.EloraError):
        B.elora_cache_release(c, 5)   # not pinned any more
    assert B.lib.elora_cache_acquire(None, 1, None, None, None) == 1
    assert "in use" in B.elora_status_string(B.ELORA_E_BUSY)
    B.elora_cache_destroy(c)


def test_hit_rate_under_the_paper_like_power_law(B):
    # Sec. 5.1: requests follow a power law over the adapters; a cache of a tenth of them serves most requests
    n_adapters, capacity = 1000, 100
    trace = I.request_trace(21, n_adapters, 1.2, 20000)
    c = B.elora_cache_create(capacity)
    for a in trace:
        B.elora_cache_acquire(c, int(a))
        B.elora_cache_release(c, int(a))
    hits, requests, _ = B.elora_cache_stats(c)
    B.elora_cache_destroy(c)
    ref = LruCacheOracle(capacity)
    for a in trace:
        ref.acquire(int(a)); ref.release(int(a))
    assert (hits, requests) == (ref.hits, ref.requests)
    assert 0.5 < hits / requests < 0.95


def test_batches_of_rows_match_the_oracle(B):
    # every row is a request; a batch's adapters stay pinned until the batch is released
    capacity, rows = 8, 6
    trace = I.request_trace(31, 40, 1.0, 600 * rows).reshape(600, rows).astype(np.int32)
    trace[5, 2] = -1                                   # a row without adapter is no request
    ref = LruCacheOracle(capacity)
    c = B.elora_cache_create(capacity)
    slots, miss_ids, miss_slots = (np.zeros(rows, np.int32) for _ in range(3))
    for ids in trace:
        want_slots, want_miss = [], []
        for a in ids:
            if a < 0:
                want_slots.append(-1)
                continue
            blk, hit, _ = ref.acquire(int(a))
            want_slots.append(blk)
            if not hit:
                want_miss.append((int(a), blk))
        n_miss = B.elora_cache_acquire_batch(c, ids, slots, miss_ids, miss_slots)
        assert slots.tolist() == want_slots
        assert list(zip(miss_ids[:n_miss].tolist(), miss_slots[:n_miss].tolist())) == want_miss
        B.elora_cache_release_batch(c, ids)
        for a in ids:
            if a >= 0:
                assert ref.release(int(a))
    assert B.elora_cache_stats(c) == (ref.hits, ref.requests, ref.evictions)
    # more distinct adapters in one batch than blocks: refused, and nothing stays pinned
    too_many = np.arange(100, 100 + capacity + 1, dtype=np.int32)
    big = [np.zeros(capacity + 1, np.int32) for _ in range(3)]
    with pytest.raises(B.EloraError) as e:
        B.elora_cache_acquire_batch(c, too_many, *big)
    assert e.value.status == B.ELORA_E_BUSY
    assert ref.acquire_batch(too_many) == BUSY
    # the refused call is undone: none of its adapters is cached (nothing was loaded into the blocks it had assigned),
    # a later request for one of them is a miss, and its requests were not counted
    for a in too_many:
        assert B.elora_cache_lookup(c, int(a)) == -1 == ref.lookup(int(a))
    assert B.elora_cache_stats(c) == (ref.hits, ref.requests, ref.evictions)
    slot, hit, _ = B.elora_cache_acquire(c, int(too_many[0]))
    want_slot, want_hit, _ = ref.acquire(int(too_many[0]))
    assert (slot, hit) == (want_slot, want_hit) == (want_slot, False)
    B.elora_cache_release(c, int(too_many[0]))
    B.elora_cache_destroy(c)


def test_a_refused_batch_leaves_no_adapter_behind(B):
    # capacity 2, three distinct adapters in one batch: the third finds both blocks pinned
    c = B.elora_cache_create(2)
    ids = np.array([7, 8, 9], dtype=np.int32)
    out = [np.zeros(3, np.int32) for _ in range(3)]
    with pytest.raises(B.EloraError) as e:
        B.elora_cache_acquire_batch(c, ids, *out)
    assert e.value.status == B.ELORA_E_BUSY
    assert [B.elora_cache_lookup(c, a) for a in (7, 8, 9)] == [-1, -1, -1]
    assert B.elora_cache_stats(c) == (0, 0, 0)
    assert B.elora_cache_acquire(c, 7) == (0, False, -1)      # block 0 comes off the stack first again, and it is a miss
    assert B.elora_cache_acquire(c, 8) == (1, False, -1)
    assert B.elora_cache_stats(c) == (0, 2, 0)
    # with adapters cached before: they stay, a miss of the refused batch that evicted one of them does not
    B.elora_cache_release(c, 7)
    B.elora_cache_release(c, 8)
    with pytest.raises(B.EloraError):
        B.elora_cache_acquire_batch(c, np.array([7, 20, 21], dtype=np.int32), *out)   # 20 evicts 8, 21 finds none
    assert B.elora_cache_lookup(c, 7) == 0 and B.elora_cache_lookup(c, 8) == -1
    assert B.elora_cache_lookup(c, 20) == -1 and B.elora_cache_lookup(c, 21) == -1
    assert B.elora_cache_stats(c) == (0, 2, 1)
    assert B.elora_cache_acquire(c, 20) == (1, False, -1)     # the freed block, as a miss
    B.elora_cache_destroy(c)


def test_selection_matches_the_oracle_and_raises_the_hit_rate(B):
    from oracle.cache_oracle import select_adapter
    rng = np.random.default_rng(41)
    n, capacity = 60, 8
    c = B.elora_cache_create(capacity)
    ref = LruCacheOracle(capacity)
    for step in range(3000):
        scores = rng.random(n).astype(np.float32)
        if step % 7 == 0:
            scores[rng.integers(0, n, size=5)] = scores[0]            # ties
        if step % 11 == 0:
            scores[int(rng.integers(0, n))] = np.nan
        k = int(rng.integers(1, 6))
        explicit = int(rng.integers(0, n)) if step % 5 == 0 else -1
        want = select_adapter(ref.block, explicit, scores, k)
        got, resident = B.elora_cache_select(c, explicit, None if explicit >= 0 and step % 2 else scores, k)
        assert got == want and resident == (want in ref.block)
        assert B.elora_cache_acquire(c, got) == ref.acquire(want)     # the request itself
        B.elora_cache_release(c, got); ref.release(want)
    B.elora_cache_destroy(c)

    # every prompt has three suitable adapters (drawn from a power-law popularity) that the router scores well above
    # the rest: looking at all three serves more requests from the cache than insisting on the most confident one
    def hit_rate(k):
        rng = np.random.default_rng(42)
        pop = I.power_law_probs(200, 1.0)
        c = B.elora_cache_create(20)
        for _ in range(4000):
            scores = (0.1 * rng.random(200)).astype(np.float32)
            scores[rng.choice(200, size=3, replace=False, p=pop)] = (0.5 + 0.5 * rng.random(3)).astype(np.float32)
            a, _ = B.elora_cache_select(c, -1, scores, k)
            B.elora_cache_acquire(c, a); B.elora_cache_release(c, a)
        h, r, _ = B.elora_cache_stats(c)
        B.elora_cache_destroy(c)
        return h / r
    h1, h3 = hit_rate(1), hit_rate(3)
    print(f"hit rate with the most confident adapter only {h1:.3f}, with the first cached of the top three {h3:.3f}")
    assert h3 > h1 + 0.05
