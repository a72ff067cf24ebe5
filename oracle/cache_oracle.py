"""Plain, slow model of the adapter memory manager: an LRU cache over a pool of fixed blocks.

TEST INFRASTRUCTURE, NOT PRODUCT CODE (same rule as the rest of this package: only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import it, and it imports nothing of the product).

What is modelled (Sec. 3.3 and Sec. 4.2 of the paper):
  * a memory cache C of at most l adapters, l = the number of blocks of the pre-allocated pool P = {p_1 .. p_l};
  * a request for an adapter that is in C is served from the cache (a hit); otherwise the adapter is assigned to a
    free block of the pool, and when there is none the least recently used adapter is evicted and its block, returned
    to the pool, is the one the new adapter gets (Sec. 4.2 states LRU; Sec. 3.3 words it "least frequently used";
    the implementation section is followed);
  * the free blocks form a stack (Sec. 4.2), here initialised so that blocks come out in the order 0, 1, 2, ...;
  * hit rate H = h_cache / h_total (Sec. 3.3).
Not in the paper, added because loads and kernels run asynchronously on a GPU: a request pins the adapter until it
is released, and a pinned adapter is never the victim.

The recency order is a Python list searched linearly: obviously right, O(l) per request.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

BUSY = "busy"


class LruCacheOracle:
    def __init__(self, capacity: int):
        assert capacity >= 1
        self.capacity = capacity
        self.free: List[int] = list(range(capacity - 1, -1, -1))  # a stack: pop() gives 0 first
        self.order: List[int] = []          # adapter ids, least recently used first
        self.block: Dict[int, int] = {}     # adapter id -> block
        self.pins: Dict[int, int] = {}      # adapter id -> outstanding requests
        self.hits = 0
        self.requests = 0
        self.evictions = 0

    def acquire(self, adapter_id: int) -> Tuple[Optional[int], bool, int]:
        """One request.  Returns (block, hit, evicted adapter id or -1); (None, False, -1) and no change of state
        if the adapter is not cached, no block is free and every cached adapter is pinned."""
        if adapter_id in self.block:
            self.requests += 1
            self.hits += 1
            self.order.remove(adapter_id)
            self.order.append(adapter_id)
            self.pins[adapter_id] += 1
            return self.block[adapter_id], True, -1
        evicted = -1
        if self.free:
            blk = self.free.pop()
        else:
            victim = next((a for a in self.order if self.pins[a] == 0), None)
            if victim is None:
                return None, False, -1
            self.order.remove(victim)
            blk = self.block.pop(victim)
            del self.pins[victim]
            self.evictions += 1
            evicted = victim
        self.requests += 1
        self.order.append(adapter_id)
        self.block[adapter_id] = blk
        self.pins[adapter_id] = 1
        return blk, False, evicted

    def acquire_batch(self, adapter_ids):
        """The requests of one batch in order (negative id: no request).  Returns (blocks per row, misses as
        (adapter id, block) in the order the blocks were assigned), or BUSY with the call undone: its requests
        released and not counted, the adapters it had assigned blocks to no longer cached (nothing was loaded into
        those blocks), their blocks back on the stack, last assigned first; evictions made on the way stay."""
        hits0, requests0 = self.hits, self.requests
        blocks, misses, done = [], [], []
        for a in adapter_ids:
            a = int(a)
            if a < 0:
                blocks.append(-1)
                continue
            blk, hit, _ = self.acquire(a)
            if blk is None:
                for d in done:
                    self.release(d)
                for m, _b in reversed(misses):
                    self.order.remove(m)
                    self.free.append(self.block.pop(m))
                    del self.pins[m]
                self.hits, self.requests = hits0, requests0
                return BUSY
            done.append(a)
            blocks.append(blk)
            if not hit:
                misses.append((a, blk))
        return blocks, misses

    def release(self, adapter_id: int) -> bool:
        if self.pins.get(adapter_id, 0) <= 0:
            return False
        self.pins[adapter_id] -= 1
        return True

    def lookup(self, adapter_id: int) -> int:
        return self.block.get(adapter_id, -1)

    def drop(self, adapter_id: int):
        """Explicit eviction: the block goes back on the stack.  Returns True, False (not cached) or BUSY (pinned)."""
        if adapter_id not in self.block:
            return False
        if self.pins[adapter_id] > 0:
            return BUSY
        self.order.remove(adapter_id)
        self.free.append(self.block.pop(adapter_id))
        del self.pins[adapter_id]
        return True

    def hit_rate(self) -> float:
        return self.hits / self.requests if self.requests else 0.0


def run_trace(capacity: int, trace) -> Tuple[List[bool], List[int], List[int]]:
    """Every request released at once (nothing stays pinned): hit flags, blocks and evicted ids of a whole trace."""
    c = LruCacheOracle(capacity)
    hits, blocks, evicted = [], [], []
    for a in trace:
        b, h, e = c.acquire(int(a))
        c.release(int(a))
        hits.append(h)
        blocks.append(b)
        evicted.append(e)
    return hits, blocks, evicted


def select_adapter(cached, explicit_id: int, scores, k: int) -> int:
    """Adaptive adapter selection, the part after the router (Algorithm 1 of the paper): an explicitly named adapter
    is taken as it is; otherwise the k adapters with the highest confidence scores are gone through in descending
    order of confidence and the first one that is in the memory cache is taken; if none is, the one with the highest
    score (which then has to be loaded).  `cached`: anything with `in`.  Equal scores: the lower adapter id counts as
    the more confident (the paper does not say); a NaN score counts as lower than every number."""
    if explicit_id >= 0:
        return explicit_id
    def key(j):
        s = float(scores[j])
        return (1, 0.0, j) if s != s else (0, -s, j)
    top = sorted(range(len(scores)), key=key)[:max(1, min(int(k), len(scores)))]
    for j in top:
        if j in cached:
            return j
    return top[0]
