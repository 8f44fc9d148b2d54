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


# ---------------------------------------------------------------------------------------------
# Second pin, written without the model's bookkeeping: no running stamps, clocks or epochs.  The
# only thing kept is the log of loads (call, expert, slot); who sits where, how recently a slot's
# expert was named and what the latest DEMAND call protects are recomputed, for every decision,
# by scanning the full call history.
def replay_from_history(E, n_slots, history):
    """history: [(ids, mode, limit)] -> [(slots, hits, misses, dropped)] per call, final occupancy"""
    loads = []                                            # (call number, expert, slot), in order

    def occupant(s):
        for call, e, sl in reversed(loads):
            if sl == s:
                return e, call
        return None, 0

    def where(e):
        for s in range(n_slots):
            if occupant(s)[0] == e:
                return s
        return -1

    outs = []
    for c, (ids, mode, limit) in enumerate(history, 1):
        named_now = set(ids)
        protected = set()
        if mode == PREFETCH:
            for past_ids, past_mode, _ in reversed(history[:c - 1]):
                if past_mode == DEMAND:
                    protected = set(past_ids)
                    break

        def last_named(s):
            e, since = occupant(s)
            if e is None:
                return 0
            return max(i for i in range(since, c) if e in history[i - 1][0])

        def victim():
            free = [s for s in range(n_slots)
                    if occupant(s)[0] not in named_now and occupant(s)[0] not in protected]
            return min(free, key=lambda s: (last_named(s), s)) if free else -1

        hits = misses = dropped = 0
        if mode == DEMAND:
            hits = sum(1 for e in ids if where(e) >= 0)
            for e in sorted(ids):
                if where(e) < 0:
                    loads.append((c, e, victim()))
                    misses += 1
            outs.append(([where(e) for e in ids], hits, misses, 0))
            continue
        slots = []
        for e in ids:                                       # the caller's priority order
            if where(e) >= 0:
                hits += 1
                slots.append(where(e))
                continue
            v = victim()
            if v < 0 or (limit is not None and misses >= limit):
                dropped += 1
                slots.append(-1)
                continue
            loads.append((c, e, v))
            misses += 1
            slots.append(v)
        outs.append((slots, hits, misses, dropped))
    return outs, [occupant(s)[0] if occupant(s)[0] is not None else -1 for s in range(n_slots)]


def random_history(rnd, E, n_slots, n_calls, with_limit=True):
    h = []
    for _ in range(n_calls):
        if rnd.random() < 0.5:
            h.append((rnd.sample(range(E), rnd.randint(0, n_slots)), DEMAND, None))
        else:
            lim = rnd.choice([None, None, 0, 1, 2, 3]) if with_limit else None
            h.append((rnd.sample(range(E), rnd.randint(0, min(E, 2 * n_slots))), PREFETCH, lim))
    return h


def first_mismatch_with_history_replay(model_cls, seeds=range(12), n_calls=120):
    """Index of the first call on which model_cls differs from the history replay, or None."""
    for seed in seeds:
        rnd = random.Random(100 + seed)
        E, n_slots = rnd.choice([(12, 3), (20, 5), (9, 8), (30, 6)])
        hist = random_history(rnd, E, n_slots, n_calls)
        ref, final = replay_from_history(E, n_slots, hist)
        m = model_cls(E, n_slots)
        for i, (ids, mode, limit) in enumerate(hist):
            got = m.fetch(ids, mode, limit) if mode == PREFETCH else m.fetch(ids, mode)
            if (list(got[0]), got[1], got[2], got[3]) != (list(ref[i][0]), ref[i][1], ref[i][2], ref[i][3]):
                return seed, i
        if list(m.slot_expert) != final:
            return seed, len(hist)
    return None


def test_model_equals_the_history_replay():
    assert first_mismatch_with_history_replay(CacheModel) is None


# Traces worked by hand from the stated rules (not produced by running anything).
HAND_TRACES = [
    # (E, n_slots, [(ids, mode, limit, expected slots, (hits, misses, dropped), occupancy after)])
    (10, 4, [
        ([7, 2, 5], DEMAND, None, [2, 0, 1], (0, 3, 0), [2, 5, 7, -1]),
        # 5 is resident; 9 may only take the empty slot (the others belong to the last DEMAND);
        # 1 finds nothing: slot 3 now holds an expert of this very call -> dropped
        ([5, 9, 1], PREFETCH, None, [1, 3, -1], (1, 1, 1), [2, 5, 7, 9]),
        # the dropped expert was not queued: an empty prefetch changes nothing
        ([], PREFETCH, None, [], (0, 0, 0), [2, 5, 7, 9]),
        ([1], PREFETCH, None, [3], (0, 1, 0), [2, 5, 7, 1]),
        # DEMAND: 1 hits; 9 evicts the least recently named of {2 (call 1), 5 (call 2), 7 (call 1)},
        # lowest slot among equals = slot 0
        ([9, 1], DEMAND, None, [0, 3], (1, 1, 0), [9, 5, 7, 1]),
        # priority order as given: 6 takes the oldest evictable slot (7, named in call 1), 4 the
        # next (5, named in call 2), 2 is dropped although it has the lowest id
        ([6, 4, 2], PREFETCH, None, [2, 1, -1], (0, 2, 1), [9, 4, 6, 1]),
        # nothing was queued for 2
        ([9], DEMAND, None, [0], (1, 0, 0), [9, 4, 6, 1]),
        ([], PREFETCH, None, [], (0, 0, 0), [9, 4, 6, 1]),
        # the last DEMAND is now {9}: 1 (slot 3, named in call 5) is evictable again and older than
        # 4 and 6 (call 6)
        ([2], PREFETCH, None, [3], (0, 1, 0), [9, 4, 6, 2]),
    ]),
    (10, 4, [
        ([0], DEMAND, None, [0], (0, 1, 0), [0, -1, -1, -1]),
        # at most two copies per call: 3 is dropped although slot 3 is empty
        ([1, 2, 3], PREFETCH, 2, [1, 2, -1], (0, 2, 1), [0, 1, 2, -1]),
        ([1, 3], PREFETCH, 1, [1, 3], (1, 1, 0), [0, 1, 2, 3]),
        # a re-stamped resident (1, call 3) outlives an older one (2, call 2)
        ([4], PREFETCH, None, [2], (0, 1, 0), [0, 1, 4, 3]),
        ([5], PREFETCH, 0, [-1], (0, 0, 1), [0, 1, 4, 3]),
    ]),
]


def run_hand_traces(model_cls):
    """-> None if every hand trace is reproduced, else (trace, call) of the first difference"""
    for ti, (E, n_slots, calls) in enumerate(HAND_TRACES):
        m = model_cls(E, n_slots)
        for ci, (ids, mode, limit, slots, counts, occ) in enumerate(calls):
            got = m.fetch(ids, mode, limit) if mode == PREFETCH else m.fetch(ids, mode)
            if list(got[0]) != slots or tuple(got[1:]) != counts or list(m.slot_expert) != occ:
                return ti, ci
    return None


def test_hand_worked_traces():
    assert run_hand_traces(CacheModel) is None
    for E, n_slots, calls in HAND_TRACES:                   # the history replay reads the rules the same way
        outs, final = replay_from_history(E, n_slots, [(c[0], c[1], c[2]) for c in calls])
        assert [(list(o[0]), (o[1], o[2], o[3])) for o in outs] == [(c[3], c[4]) for c in calls]
        assert final == calls[-1][5]


# ---- planted mistakes: each must be caught by the hand traces and by the history replay --------
class EvictsLastDemand(CacheModel):
    """PREFETCH ignores the protection of the most recent DEMAND call."""
    def _victim(self, needed, protect_epoch):
        return super()._victim(needed, None)


class QueuesInsteadOfDropping(CacheModel):
    """A PREFETCH miss without a slot is kept and loaded first by the next PREFETCH call."""
    def __init__(self, *a):
        super().__init__(*a)
        self.queue = []

    def fetch(self, ids, mode, limit=None):
        if mode != PREFETCH:
            return super().fetch(ids, mode)
        late = [e for e in self.queue if e not in ids and self.slot_of(e) < 0]
        out = super().fetch(list(late) + list(ids), mode, limit)
        k = len(late)
        self.queue = [e for e, s in zip(ids, out[0][k:]) if s < 0]
        return out[0][k:], out[1], out[2] - sum(1 for s in out[0][:k] if s >= 0), out[3] - sum(1 for s in out[0][:k] if s < 0)


class IgnoresPriorityOrder(CacheModel):
    """PREFETCH loads its misses in ascending expert id instead of the given order."""
    def fetch(self, ids, mode, limit=None):
        if mode != PREFETCH:
            return super().fetch(ids, mode)
        order = sorted(ids)
        slots, h, m, d = super().fetch(order, mode, limit)
        back = dict(zip(order, slots))
        return [back[e] for e in ids], h, m, d


class PrefetchHitNotRestamped(CacheModel):
    """A resident expert named by a PREFETCH call keeps its old time stamp."""
    def fetch(self, ids, mode, limit=None):
        if mode != PREFETCH:
            return super().fetch(ids, mode)
        before = {s: self.stamp[s] for s in range(self.n_slots) if self.slot_expert[s] in ids}
        out = super().fetch(ids, mode, limit)
        for s, st in before.items():
            if self.slot_expert[s] in ids and out[0][list(ids).index(self.slot_expert[s])] == s:
                self.stamp[s] = st
        return out


class HighestSlotAmongEquals(CacheModel):
    """Among equally old slots the highest id is evicted."""
    def _victim(self, needed, protect_epoch):
        best = -1
        for s in range(self.n_slots):
            if self.slot_expert[s] in needed:
                continue
            if protect_epoch is not None and self.demand_epoch[s] == protect_epoch:
                continue
            if best < 0 or self.stamp[s] <= self.stamp[best]:
                best = s
        return best


class DemandMissesInGivenOrder(CacheModel):
    """DEMAND loads its misses in the order given instead of ascending expert id."""
    def fetch(self, ids, mode, limit=None):
        if mode != DEMAND:
            return super().fetch(ids, mode, limit)
        ids = list(ids)
        needed = set(ids)
        self.clock += 1
        self.epoch += 1
        hits = misses = 0
        for e in ids:
            s = self.slot_of(e)
            if s >= 0:
                self.stamp[s], self.demand_epoch[s] = self.clock, self.epoch
                hits += 1
        for e in ids:
            if self.slot_of(e) < 0:
                v = self._victim(needed, None)
                self.slot_expert[v], self.stamp[v], self.demand_epoch[v] = e, self.clock, self.epoch
                misses += 1
        return [self.slot_of(e) for e in ids], hits, misses, 0


class LimitCountsHits(CacheModel):
    """The bound on copies per PREFETCH call also counts experts that were already resident."""
    def fetch(self, ids, mode, limit=None):
        if mode != PREFETCH or limit is None:
            return super().fetch(ids, mode, limit)
        n_res = sum(1 for e in ids if self.slot_of(e) >= 0)
        return super().fetch(ids, mode, max(0, limit - n_res))


MUTANTS = [EvictsLastDemand, QueuesInsteadOfDropping, IgnoresPriorityOrder, PrefetchHitNotRestamped,
           HighestSlotAmongEquals, DemandMissesInGivenOrder, LimitCountsHits]


def test_every_planted_mistake_fails_both_pins():
    for mutant in MUTANTS:
        assert first_mismatch_with_history_replay(mutant) is not None, mutant.__name__
        assert run_hand_traces(mutant) is not None, mutant.__name__
