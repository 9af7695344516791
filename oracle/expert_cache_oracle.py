"""CPU oracle for the frequency-based cache of sparse (expert) parameters (TEST INFRASTRUCTURE).

This file is the checker, not the product: only ``tests/`` and the bench's
baseline leg may import it.  It shares no code with the C++ implementation.

What it models.  The paper's "Scheduling on Sparse Parameters" (Algorithm 2,
Section 3.2.2) keeps the selectively activated expert states that the next
computation needs in a cache of fixed capacity in the faster memory, "akin to
LFU": a table `hits` counts how often each cached item was requested, every
K requests all counts are multiplied by an attenuation coefficient beta, and
when the cache is full the item to give up is the one "with the lowest hit
frequency that surpasses the hit threshold".  Here the slower memory is pinned
host memory and the faster one a pool of expert-sized slots in HBM; the steps
are those of the algorithm, in its order and notation.

Readings (the algorithm as printed is ambiguous in four places):
 * free space: the printed test `acc_caches + 1 < CPU_size` would leave one
   slot unused for ever; read as `acc_caches < CPU_size`.
 * victim: the printed condition (`hit_a >= threshold` and `hit_a` equal to the
   minimum over ALL items) and the prose (lowest count among those that reach
   the threshold) differ when some item lies below the threshold; the prose is
   taken, because under the printed form a single item that decays below the
   threshold would freeze the cache.  Items below the threshold (new, or
   decayed) are thus protected.
 * the printed `foreach` would evict every item that ties for the minimum and
   fetch p_s once per eviction; read as ONE eviction per request, ties going to
   the item cached earliest.
 * no item reaches the threshold: the algorithm then evicts nothing (on the
   paper's CPU tier the request is served from the SSD without being cached).
   An expert must be in HBM to be computed, so here the item with the lowest
   count overall is given up instead (ties: cached earliest).
One addition: items requested since the last `begin_batch()` are never chosen
as victims, because all experts of one layer evaluation must be resident at
the same time (the capacity must be at least the largest such batch).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple


class SparseParameterCache:
    """`hits`, `threshold`, `beta`, `K`, `steps` and `acc_caches` are Algorithm 2's own names."""

    def __init__(self, size: int, threshold: float, beta: float, K: int):
        if size < 1 or K < 1:
            raise ValueError("size and K must be at least 1")
        self.size = int(size)
        self.threshold = float(threshold)
        self.beta = float(beta)
        self.K = int(K)
        self.steps = 0
        self.acc_caches = 0
        self.hits: Dict[int, float] = {}        # cached item -> (attenuated) number of requests
        self.slot: Dict[int, int] = {}          # cached item -> slot of the pool it occupies
        self.cached_at: Dict[int, int] = {}     # cached item -> sequence number of its insertion
        self.batch: Dict[int, int] = {}         # cached item -> batch number of its last request
        self.cur_batch = 0
        self.inserts = 0

    def begin_batch(self) -> None:
        self.cur_batch += 1

    def schedule(self, p_s: int) -> Tuple[int, bool, Optional[int]]:
        """One SparseSchedule call for item p_s: returns (slot, was cached, evicted item or None)."""
        evicted = None
        if p_s in self.hits:                                   # "Get p_s from the caches; hits[p_s] += 1"
            self.hits[p_s] += 1.0
            hit = True
        else:
            hit = False
            if self.acc_caches < self.size:                    # free space: next unused slot
                slot = self.acc_caches
                self.acc_caches += 1
            else:
                evicted = self._victim()
                slot = self.slot[evicted]
                del self.hits[evicted], self.slot[evicted], self.cached_at[evicted], self.batch[evicted]
            self.hits[p_s] = 1.0
            self.slot[p_s] = slot
            self.cached_at[p_s] = self.inserts
            self.inserts += 1
        self.batch[p_s] = self.cur_batch
        self.steps += 1
        if self.steps == self.K:                               # "hits * beta" (moving average)
            for a in self.hits:
                self.hits[a] *= self.beta
            self.steps = 0
        return self.slot[p_s], hit, evicted

    def _victim(self) -> int:
        free = [a for a in self.hits if self.batch[a] != self.cur_batch]
        if not free:
            raise RuntimeError("every cached item belongs to the current batch: capacity too small")
        above = [a for a in free if self.hits[a] >= self.threshold]
        pool = above if above else free
        return min(pool, key=lambda a: (self.hits[a], self.cached_at[a]))


def run_trace(size: int, threshold: float, beta: float, K: int, trace: List[Tuple[int, bool]]):
    """Feeds (item, starts_a_new_batch) pairs; returns the list of (slot, hit, evicted or -1)."""
    c = SparseParameterCache(size, threshold, beta, K)
    out = []
    for item, new_batch in trace:
        if new_batch:
            c.begin_batch()
        s, h, e = c.schedule(item)
        out.append((s, bool(h), -1 if e is None else e))
    return out
