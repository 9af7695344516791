"""Frequency-based expert cache (Algorithm 2 of Section 3.2.2): pins of the oracle, planted mistakes that
those pins must catch, and the C++ policy against the oracle on random traces.  CPU only."""
import numpy as np
import pytest

import paper_2205_10034_amd as M
from oracle.expert_cache_oracle import SparseParameterCache, run_trace


# ----------------------------------------------------------------- pins (take the class under test)
def pin_textbook_lfu(Cache):
    """threshold <= 1 and beta = 1: plain LFU with first-in tie-break, recomputed from the whole request
    history at every step (count = requests of the item since it was last brought in)."""
    rng = np.random.default_rng(3)
    for size, n_items in [(1, 3), (2, 5), (4, 9), (7, 8)]:
        c = Cache(size, 1.0, 1.0, 5)
        history = []                     # (item, was brought in at this step)
        resident = {}                    # item -> slot
        for step in range(300):
            p = int(rng.zipf(1.5) % n_items)
            c.begin_batch()
            slot, hit, gone = c.schedule(p)
            assert hit == (p in resident)
            if p in resident:
                assert slot == resident[p] and gone is None
                history.append((p, False))
                continue
            if len(resident) < size:
                assert gone is None and slot == len(resident)
            else:
                def since_brought_in(a):
                    last = max(i for i, (q, new) in enumerate(history) if q == a and new)
                    return sum(1 for q, _ in history[last:] if q == a), last
                want = min(resident, key=since_brought_in)
                assert gone == want and slot == resident[want]
                del resident[want]
            resident[p] = slot
            history.append((p, True))
            assert len(set(resident.values())) == len(resident) <= size


def pin_decay_worked_example(Cache):
    """One item, K = 3, beta = 0.5: counts 1, 2, 3 -> 1.5, 2.5, 3.5, 4.5 -> 2.25, 3.25."""
    c = Cache(2, 1.0, 0.5, 3)
    seen = []
    for _ in range(7):
        c.schedule(7)
        seen.append(c.hits[7])
    assert seen == [1.0, 2.0, 1.5, 2.5, 3.5, 2.25, 3.25]
    # the period counts requests of any item, and every cached item is attenuated
    c = Cache(3, 1.0, 0.25, 2)
    c.schedule(1); c.schedule(2)
    assert c.hits == {1: 0.25, 2: 0.25}
    c.schedule(1)
    assert c.hits == {1: 1.25, 2: 0.25}


def pin_threshold_protects_items_below_it(Cache):
    """size 2, threshold 2: A A B | C gives up A (the only item at the threshold; B, new, is protected);
    then D finds nobody at the threshold and takes the lowest count overall, first in first out: B."""
    c = Cache(2, 2.0, 1.0, 1000)
    for item in (10, 10, 11):
        c.begin_batch()
        c.schedule(item)
    c.begin_batch()
    assert c.schedule(12) == (0, False, 10)
    c.begin_batch()
    assert c.schedule(13) == (1, False, 11)
    c.begin_batch()
    assert c.schedule(12) == (0, True, None)          # now 12 has two requests: it alone is at the threshold
    c.begin_batch()
    assert c.schedule(14) == (0, False, 12)
    # exactly at the threshold counts as reaching it; among several at the threshold the lowest goes
    c = Cache(3, 2.0, 1.0, 1000)
    for item in (1, 1, 1, 2, 2, 3):
        c.begin_batch()
        c.schedule(item)
    c.begin_batch()
    assert c.schedule(4)[2] == 2


def pin_batch_members_are_never_victims(Cache):
    c = Cache(2, 1.0, 1.0, 1000)
    c.begin_batch()
    for _ in range(5):
        c.schedule(1)                                  # popular
    c.begin_batch()
    c.schedule(2)
    assert c.schedule(3)[2] == 1                       # 2 is of this batch, so popular 1 has to go
    c.begin_batch()
    c.schedule(3)
    c.schedule(2)
    with pytest.raises(Exception):
        c.schedule(4)                                  # both slots belong to the running batch


def pin_invariants_on_random_traces(Cache):
    rng = np.random.default_rng(11)
    for size, thr, beta, K in [(3, 1.0, 0.9, 4), (8, 2.0, 0.5, 7), (16, 3.0, 0.99, 1), (5, 0.0, 0.0, 3)]:
        c = Cache(size, thr, beta, K)
        resident = {}
        batch = set()
        for step in range(2000):
            if step % 3 == 0:
                c.begin_batch()
                batch = set()
            p = int(rng.integers(0, 3 * size))
            if p not in resident and len(resident) == size and len(batch - {p}) >= size:
                continue                               # would not fit beside its own batch
            slot, hit, gone = c.schedule(p)
            assert hit == (p in resident)
            if gone is not None:
                assert gone in resident and gone not in batch and resident[gone] == slot
                del resident[gone]
            if hit:
                assert resident[p] == slot
            resident[p] = slot
            batch.add(p)
            assert len(resident) <= size and len(set(resident.values())) == len(resident)
            assert all(0 <= s < size for s in resident.values())
            assert set(c.hits) == set(resident)


PINS = [pin_textbook_lfu, pin_decay_worked_example, pin_threshold_protects_items_below_it,
        pin_batch_members_are_never_victims, pin_invariants_on_random_traces]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_pin(pin):
    pin(SparseParameterCache)


# ------------------------------------------------------------------------- planted mistakes
class _HighestCountGoes(SparseParameterCache):
    def choose_victim(self):
        cand = self.evictable()
        est = [r for r in cand if r.count >= self.floor]
        return max(est or cand, key=lambda r: (r.count, -r.arrival))


class _LastInFirstOutTies(SparseParameterCache):
    def choose_victim(self):
        cand = self.evictable()
        est = [r for r in cand if r.count >= self.floor]
        return min(est or cand, key=lambda r: (r.count, -r.arrival))


class _ThresholdIgnored(SparseParameterCache):
    def choose_victim(self):
        return min(self.evictable(), key=lambda r: (r.count, r.arrival))


class _ThresholdStrict(SparseParameterCache):
    def choose_victim(self):
        cand = self.evictable()
        est = [r for r in cand if r.count > self.floor]
        return min(est or cand, key=lambda r: (r.count, r.arrival))


class _BatchUnprotected(SparseParameterCache):
    def evictable(self):
        return list(self.residents.values())


class _PrintedFreeSpaceTest(SparseParameterCache):       # the printed comparison: the last place is never used
    def admit(self, item):
        if self.places_taken + 1 >= self.capacity and self.places_taken < self.capacity:
            from oracle.expert_cache_oracle import Resident
            self.places_taken = self.capacity
            ghost = -1 - self.arrivals
            self.residents[ghost] = Resident(ghost, self.capacity - 1, 0.0, -1, -1)
        return super().admit(item)


class _DecayOneStepLate(SparseParameterCache):
    def __init__(self, size, threshold, beta, K):
        super().__init__(size, threshold, beta, K + 1)


class _DecayOnlyTheRequestedItem(SparseParameterCache):
    def schedule(self, item):
        decay, self.decay = self.decay, 1.0
        due = self.requests_in_period + 1 == self.period
        out = super().schedule(item)
        self.decay = decay
        if due:
            self.residents[item].count *= decay
        return out


class _HitCountNotUpdated(SparseParameterCache):
    def schedule(self, item):
        before = self.residents[item].count if item in self.residents else None
        out = super().schedule(item)
        if before is not None and self.requests_in_period != 0:
            self.residents[item].count = before
        return out


class _NewItemStartsAtZero(SparseParameterCache):
    def schedule(self, item):
        new = item not in self.residents
        out = super().schedule(item)
        if new:
            self.residents[item].count -= 1.0 if self.requests_in_period != 0 else self.decay
        return out


MUTANTS = [_HighestCountGoes, _LastInFirstOutTies, _ThresholdIgnored, _ThresholdStrict, _BatchUnprotected,
           _PrintedFreeSpaceTest, _DecayOneStepLate, _DecayOnlyTheRequestedItem, _HitCountNotUpdated,
           _NewItemStartsAtZero]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda m: m.__name__.strip("_"))
def test_pins_catch_planted_mistake(mutant):
    caught = []
    for pin in PINS:
        try:
            pin(mutant)
        except Exception:       # an assertion, or a crash caused by the mistake
            caught.append(pin.__name__)
    assert caught, f"no pin notices {mutant.__name__}"


# ----------------------------------------------------------------- the C++ policy against the oracle
@pytest.mark.parametrize("size,thr,beta,K,n_items,seed", [
    (1, 1.0, 1.0, 1, 4, 0), (4, 1.0, 0.5, 3, 12, 1), (16, 2.0, 0.9, 8, 64, 2), (64, 3.0, 0.75, 32, 256, 3),
    (238, 2.0, 0.9, 128, 1536, 4), (8, 0.0, 0.0, 2, 20, 5), (5, 100.0, 1.0, 1000, 30, 6)])
def test_library_policy_matches_oracle(size, thr, beta, K, n_items, seed):
    rng = np.random.default_rng(seed)
    # bursts of distinct items (one layer's activated experts), popularity skewed
    trace = []
    weights = 1.0 / np.arange(1, n_items + 1) ** 1.1
    weights /= weights.sum()
    while len(trace) < 6000:
        burst = rng.choice(n_items, size=min(size, int(rng.integers(1, 9))), replace=False, p=weights)
        for i, item in enumerate(burst):
            trace.append((int(item), i == 0))
    beta32, thr32 = float(np.float32(beta)), float(np.float32(thr))     # the ABI takes float32
    want = run_trace(size, thr32, beta32, K, trace)
    c = M.ExpertCache(size, thr, beta, K)
    ref = SparseParameterCache(size, thr32, beta32, K)
    for (item, new_batch), w in zip(trace, want):
        if new_batch:
            c.begin_batch()
            ref.begin_batch()
        got = c.schedule(item)
        ref.schedule(item)
        assert got == w
        slot, hits = c.lookup(item)
        assert slot == w[0] and hits == ref.hits[item]                  # bit-identical counts
    st = c.stats()
    assert st["hits"] == sum(1 for w in want if w[1])
    assert st["misses"] == len(want) - st["hits"]
    assert st["evictions"] == sum(1 for w in want if w[2] >= 0)
    assert c.lookup(10 ** 9) == (-1, 0.0)


def test_library_policy_error_paths():
    import ctypes as C
    L = M.lib()
    h = C.c_void_p()
    for bad in [(0, 1.0, 1.0, 1), (4, 1.0, 1.0, 0), (4, 1.0, -1.0, 1), (4, float("nan"), 1.0, 1)]:
        assert L.moe_expert_cache_create(C.byref(h), *bad) == 1
    assert L.moe_expert_cache_create(None, 4, 1.0, 1.0, 1) == 1
    c = M.ExpertCache(2, 1.0, 1.0, 10)
    c.begin_batch()
    c.schedule(1)
    c.schedule(2)
    with pytest.raises(M.MoEError) as e:
        c.schedule(3)
    assert "current batch" in str(e.value)
    with pytest.raises(M.MoEError):
        c.schedule(-5)
    assert L.moe_expert_cache_destroy(None) == 0
