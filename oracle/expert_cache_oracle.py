"""CPU oracle for the frequency-based cache of sparse (expert) parameters (TEST INFRASTRUCTURE).

This file is the checker, not the product: only ``tests/`` and the bench's
baseline leg may import it.  It shares no code with the C++ implementation.

What it models (Algorithm 2, Section 3.2.2: scheduling of sparse parameters).
A fixed number of places in the faster memory holds the expert states that
were asked for most often, in the manner of a least-frequently-used cache:
  * every request of a resident item raises that item's request count by one;
  * after every `period` requests (of any item) every count is multiplied by
    the attenuation factor `decay`, so that old popularity fades;
  * a request of an item that is not resident brings it in with a count of one,
    into an unused place while there is one, else into the place of a victim;
  * the victim is, among the residents whose count has reached `floor`, the one
    with the smallest count.
Here the slower memory is pinned host memory and the faster one a pool of
expert-sized slots in HBM.

Readings (the algorithm as printed is ambiguous in four places):
 * free space: the printed comparison would leave the last place unused for
   ever; here a place is free as long as fewer than `capacity` are taken.
 * victim: the listing asks for a count at or above the floor that is also the
   minimum over ALL residents, the prose for the smallest count among those at
   or above the floor; the two differ as soon as one resident lies below the
   floor, and under the listing's form such a resident would freeze the cache.
   The prose is taken: residents below the floor (new, or faded) are protected.
 * the listing's loop would give up every resident that ties for the minimum
   and fetch the new item once per victim; read as ONE victim per request, ties
   going to the resident that came in earliest.
 * nobody has reached the floor: the algorithm then gives up nothing (on the
   paper's CPU tier the request is served from the SSD without being cached).
   An expert must be in HBM to be computed, so here the smallest count overall
   goes instead (ties: earliest arrival).
One addition: residents requested since the last `begin_batch()` are never
victims, because all experts of one layer evaluation must be resident at the
same time (the capacity must be at least the largest such batch).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple


@dataclass
class Resident:
    """One occupied place of the pool."""
    item: int
    place: int          # slot of the pool
    count: float        # attenuated number of requests since it came in
    arrival: int        # sequence number of its coming in (tie-break: earliest goes first)
    batch: int          # number of the batch that last asked for it


class SparseParameterCache:
    def __init__(self, capacity: int, floor: float, decay: float, period: int):
        if capacity < 1 or period < 1:
            raise ValueError("capacity and period must be at least 1")
        self.capacity, self.floor, self.decay, self.period = int(capacity), float(floor), float(decay), int(period)
        self.residents: Dict[int, Resident] = {}
        self.places_taken = 0        # places are handed out in index order and never become unused again
        self.arrivals = 0
        self.requests_in_period = 0
        self.batch_no = 0

    # -- the tests read these two views
    @property
    def hits(self) -> Dict[int, float]:
        return {r.item: r.count for r in self.residents.values()}

    def begin_batch(self) -> None:
        self.batch_no += 1

    def evictable(self) -> List[Resident]:
        """Residents that the current batch has not asked for."""
        return [r for r in self.residents.values() if r.batch != self.batch_no]

    def choose_victim(self) -> Resident:
        candidates = self.evictable()
        if not candidates:
            raise RuntimeError("every cached item belongs to the current batch: capacity too small")
        established = [r for r in candidates if r.count >= self.floor]
        return min(established or candidates, key=lambda r: (r.count, r.arrival))

    def admit(self, item: int) -> Optional[int]:
        """Brings `item` in; returns the item that made room for it, if any."""
        gone = None
        if self.places_taken < self.capacity:
            place = self.places_taken
            self.places_taken += 1
        else:
            victim = self.choose_victim()
            place, gone = victim.place, victim.item
            del self.residents[gone]
        self.residents[item] = Resident(item, place, 1.0, self.arrivals, self.batch_no)
        self.arrivals += 1
        return gone

    def fade(self) -> None:
        """Counts of all residents shrink once per `period` requests."""
        self.requests_in_period += 1
        if self.requests_in_period == self.period:
            self.requests_in_period = 0
            for r in self.residents.values():
                r.count *= self.decay

    def schedule(self, item: int) -> Tuple[int, bool, Optional[int]]:
        """One request: returns (place, was resident, item given up or None)."""
        r = self.residents.get(item)
        was_resident = r is not None
        gone = None
        if was_resident:
            r.count += 1.0
            r.batch = self.batch_no
        else:
            gone = self.admit(item)
        self.fade()
        return self.residents[item].place, was_resident, gone


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
