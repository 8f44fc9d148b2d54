"""Pins of the host-only expert-cache model (CPU only): textbook LRU and structural invariants."""
import collections
import random

from oracle.cache_model import DEMAND, PREFETCH, CacheModel


def test_single_expert_demands_are_textbook_lru():
    rnd = random.Random(0)
    for n_slots in (1, 3, 8):
        m = CacheModel(20, n_slots)
        lru = collections.OrderedDict()
        for _ in range(600):
            e = rnd.randrange(20)
            _, hits, misses, _ = m.fetch([e], DEMAND)
            if e in lru:
                lru.move_to_end(e)
                assert (hits, misses) == (1, 0)
            else:
                if len(lru) == n_slots:
                    lru.popitem(last=False)
                lru[e] = True
                assert (hits, misses) == (0, 1)
            assert sorted(x for x in m.slot_expert if x >= 0) == sorted(lru)


def test_invariants_on_random_traces():
    rnd = random.Random(1)
    E, n_slots = 64, 16
    m = CacheModel(E, n_slots)
    last_demand = set()
    for step in range(400):
        if rnd.random() < 0.6:
            ids = rnd.sample(range(E), rnd.randint(0, n_slots))
            before = list(m.slot_expert)
            slots, hits, misses, dropped = m.fetch(ids, DEMAND)
            assert hits + misses == len(ids) and dropped == 0
            assert hits == sum(1 for e in ids if e in before)
            assert all(m.slot_expert[s] == e for e, s in zip(ids, slots))   # every demand is resident
            last_demand = set(ids)
        else:
            ids = rnd.sample(range(E), rnd.randint(0, 30))
            before = list(m.slot_expert)
            slots, hits, misses, dropped = m.fetch(ids, PREFETCH)
            assert hits + misses + dropped == len(ids)
            for e in last_demand:                                           # never evicts the last demand set
                assert (e in before) <= (e in m.slot_expert)
            for e, s in zip(ids, slots):
                assert (s == -1) or m.slot_expert[s] == e
        res = [x for x in m.slot_expert if x >= 0]
        assert len(res) == len(set(res))                                    # no expert in two slots


def test_demand_order_and_victims():
    m = CacheModel(10, 4)
    assert m.fetch([7, 2, 5], DEMAND)[0] == [2, 0, 1]       # misses loaded in ascending id into slots 0,1,2
    assert m.fetch([9], DEMAND)[0] == [3]                   # the empty slot is the oldest
    slots, hits, misses, _ = m.fetch([2, 1], DEMAND)         # 2 hits; 1 evicts the least recent of {5,7} = lowest slot
    assert (hits, misses) == (1, 1) and slots == [0, 1] and m.slot_expert == [2, 1, 7, 9]
    # prefetch may not evict the last demand set {2,1}; 7 and 9 are evictable, oldest first
    slots, hits, misses, dropped = m.fetch([4, 3, 6], PREFETCH)
    assert (hits, misses, dropped) == (0, 2, 1) and slots == [2, 3, -1]
    assert m.slot_expert == [2, 1, 4, 3]
