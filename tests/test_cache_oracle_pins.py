"""The cache oracle against what the mathematics of LRU fixes (no GPU, no product code)."""
import numpy as np
import pytest

from oracle.cache_oracle import BUSY, LruCacheOracle, run_trace
from paper_2507_01438_amd import inputs as I


def _reuse_distance_hits(capacity, trace):
    """Independent characterisation of LRU: a request hits iff fewer than `capacity` distinct OTHER adapters were
    requested since the previous request for the same adapter."""
    out = []
    for i, a in enumerate(trace):
        prev = max((j for j in range(i) if trace[j] == a), default=None)
        out.append(prev is not None and len(set(trace[prev + 1:i])) < capacity)
    return out


def _optimal_misses(capacity, trace):
    """Belady's policy by brute force: evict the adapter whose next request lies farthest ahead."""
    cached, misses = set(), 0
    for i, a in enumerate(trace):
        if a in cached:
            continue
        misses += 1
        if len(cached) == capacity:
            def next_use(b):
                return next((j for j in range(i + 1, len(trace)) if trace[j] == b), len(trace) + 1)
            cached.remove(max(cached, key=next_use))
        cached.add(a)
    return misses


def _fifo_misses(capacity, trace):
    queue, misses = [], 0
    for a in trace:
        if a not in queue:
            misses += 1
            if len(queue) == capacity:
                queue.pop(0)
            queue.append(a)
    return misses


# The 20-request example used in operating-systems textbooks for page replacement with three frames: 12 misses under
# LRU, 15 under first-in-first-out, 9 under the optimal policy.
CLASSIC = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]


def test_classic_three_block_example():
    hits, _, _ = run_trace(3, CLASSIC)
    assert hits.count(False) == 12
    assert _fifo_misses(3, CLASSIC) == 15 and _optimal_misses(3, CLASSIC) == 9   # the helpers used below agree with it too


def test_cyclic_trace_never_hits_and_single_adapter_always_does():
    l = 5
    hits, _, evicted = run_trace(l, [i % (l + 1) for i in range(60)])
    assert not any(hits)
    assert evicted[:l] == [-1] * l and evicted[l:] == [(i - l) % (l + 1) for i in range(l, 60)]  # always the oldest
    hits, blocks, _ = run_trace(l, [42] * 30)
    assert hits == [False] + [True] * 29 and set(blocks) == {0}


@pytest.mark.parametrize("seed,capacity,alpha", [(1, 1, None), (2, 3, None), (3, 4, 1.0), (4, 8, 0.5), (5, 6, 1.5)])
def test_hits_are_exactly_the_short_reuse_distances(seed, capacity, alpha):
    trace = list(I.request_trace(seed, 20, alpha, 300))
    assert run_trace(capacity, trace)[0] == _reuse_distance_hits(capacity, trace)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_inclusion_property_and_optimal_bound(seed):
    trace = list(I.request_trace(seed, 12, 1.0, 200))
    prev_sets = None
    for capacity in (1, 2, 3, 5, 8):
        c = LruCacheOracle(capacity)
        sets = []
        for a in trace:
            c.acquire(a)
            c.release(a)
            sets.append(set(c.block))
            assert len(c.block) <= capacity and sorted(c.order) == sorted(c.block)
            assert sorted(list(c.block.values()) + c.free) == list(range(capacity))   # every block is somewhere, once
        if prev_sets is not None:   # what a smaller LRU cache holds, a larger one holds too
            assert all(s <= t for s, t in zip(prev_sets, sets))
        prev_sets = sets
        assert c.requests - c.hits >= _optimal_misses(capacity, trace)
        assert c.hit_rate() == c.hits / len(trace)


def test_blocks_come_off_a_stack():
    c = LruCacheOracle(4)
    assert [c.acquire(a)[0] for a in (10, 11, 12)] == [0, 1, 2]
    for a in (10, 11, 12):
        c.release(a)
    assert c.drop(11) is True and c.drop(10) is True and c.drop(99) is False
    assert c.acquire(20)[0] == 0 and c.acquire(21)[0] == 1 and c.acquire(22)[0] == 3   # last returned first, then the untouched one
    assert c.lookup(12) == 2 and c.lookup(11) == -1


def test_pinned_adapters_are_never_the_victim():
    c = LruCacheOracle(2)
    c.acquire(1)
    c.acquire(2)                         # both pinned
    assert c.acquire(3) == (None, False, -1) and c.requests == 2
    assert c.drop(1) == BUSY
    c.release(2)
    assert c.acquire(3) == (1, False, 2)  # 1 is older but pinned: 2 goes
    c.release(1)
    c.release(3)
    assert c.acquire(4) == (0, False, 1)
    assert not c.release(2)               # not cached any more


# ---- adaptive adapter selection after the router (Algorithm 1) -------------------------------------------------------

def test_selection_worked_examples():
    from oracle.cache_oracle import select_adapter
    scores = [0.10, 0.90, 0.30, 0.80, 0.85]            # confidence order: 1, 4, 3, 2, 0
    assert select_adapter({3, 0}, -1, scores, 3) == 3  # 1 and 4 are not cached, 3 is
    assert select_adapter({3, 4}, -1, scores, 3) == 4  # the more confident of the cached ones
    assert select_adapter({0, 2}, -1, scores, 3) == 1  # none of the top three cached: the most confident, to be loaded
    assert select_adapter({2}, -1, scores, 4) == 2 and select_adapter({2}, -1, scores, 3) == 1
    assert select_adapter({3}, 0, scores, 3) == 0      # explicitly named: taken as it is
    assert select_adapter({2, 3}, -1, [0.5, 0.5, 0.5, 0.5], 2) == 0      # ties: lower id first, top two are 0 and 1
    assert select_adapter({1}, -1, [float("nan"), 0.1, 0.2], 2) == 1     # NaN ranks last: top two are 2 and 1


@pytest.mark.parametrize("seed", range(5))
def test_selection_against_an_independent_formulation(seed):
    from oracle.cache_oracle import select_adapter
    rng = np.random.default_rng(seed)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        k = int(rng.integers(1, n + 1))
        scores = rng.permutation(n).astype(np.float32) / n       # distinct
        cached = set(rng.choice(n, size=int(rng.integers(0, n + 1)), replace=False).tolist())
        rank = {j: int((scores > scores[j]).sum()) for j in range(n)}   # adapters with a higher score
        eligible = [j for j in cached if rank[j] < k]
        want = max(eligible, key=lambda j: scores[j]) if eligible else int(np.argmax(scores))
        assert select_adapter(cached, -1, scores, k) == want
        assert select_adapter(cached, -1, scores, 1) == int(np.argmax(scores))   # k = 1: the availability is not looked at


def test_a_refused_batch_is_undone_by_hand():
    # two blocks, a batch naming three adapters: the third finds both pinned.  Worked by hand: afterwards nothing is
    # cached, both blocks are free (0 comes off first again), nothing was counted.
    c = LruCacheOracle(2)
    assert c.acquire_batch([7, 8, 9]) == BUSY
    assert (c.block, c.order, c.pins, c.free) == ({}, [], {}, [1, 0])
    assert (c.hits, c.requests, c.evictions) == (0, 0, 0)
    # a batch that fits: rows 0 and 2 share an adapter (the second is a hit), row 1 has none
    assert c.acquire_batch([7, -1, 7, 8]) == ([0, -1, 0, 1], [(7, 0), (8, 1)])
    assert (c.hits, c.requests) == (1, 3)
    for a in (7, 7, 8):
        assert c.release(a)
    # 7 stays (a hit), 20 evicts 8 (least recently used of the unpinned), 21 finds nothing: undone, but the eviction stays
    assert c.acquire_batch([7, 20, 21]) == BUSY
    assert c.block == {7: 0} and c.free == [1] and c.pins == {7: 0}
    assert (c.hits, c.requests, c.evictions) == (1, 3, 1)
