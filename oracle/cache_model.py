"""Host-only model of the HBM expert cache -- TEST INFRASTRUCTURE ONLY.

The paper keeps inactive experts in host DRAM and loads the ones the router selects (Sec. II-B);
for a token that falls back to the big model, the router outputs of its discarded little pass
name the experts to prefetch (Sec. III-B).  The paper fixes no replacement policy; this model is
the reading the library documents, written out as plain integer bookkeeping.  (History: the
reading was fixed first, the library's cache code second, this model third; it is therefore
pinned below by references that share nothing with either.)

* every fetch call advances a logical clock; experts named by the call that are resident
  afterwards carry that time stamp;
* DEMAND (at most n_slots distinct experts): resident ones are hits; the misses are loaded in
  ascending expert id, each into the least recently stamped slot that holds no expert of this
  call (lowest slot id among equals; empty slots are oldest);
* PREFETCH (any number, priority order): resident ones are re-stamped; a miss is loaded only
  into a slot that holds neither an expert of this call nor one of the most recent DEMAND call,
  otherwise it is dropped (never queued for later).  An optional `limit` bounds the copies one
  PREFETCH call may start (the depth of the prefetch queue, Sec. III-B: how far ahead to load is
  adjustable); misses beyond it are dropped as well.

Pins (tests/test_cache_model.py): single-expert DEMAND traces equal a textbook LRU written with
an OrderedDict; a brute-force reference that keeps no running state but recomputes every decision
from the full call history; traces worked by hand from the rules above; structural invariants on
random traces; and each of a list of planted mistakes is shown to fail those pins.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

DEMAND, PREFETCH = 0, 1


class CacheModel:
    def __init__(self, n_experts: int, n_slots: int):
        self.E, self.n_slots = n_experts, n_slots
        self.slot_expert = [-1] * n_slots
        self.stamp = [0] * n_slots
        self.demand_epoch = [None] * n_slots
        self.clock = 0
        self.epoch = 0

    def slot_of(self, e: int) -> int:
        return self.slot_expert.index(e) if e in self.slot_expert else -1

    def _victim(self, needed: set, protect_epoch) -> int:
        best = -1
        for s in range(self.n_slots):
            if self.slot_expert[s] in needed:
                continue
            if protect_epoch is not None and self.demand_epoch[s] == protect_epoch:
                continue
            if best < 0 or self.stamp[s] < self.stamp[best]:
                best = s
        return best

    def fetch(self, ids: Sequence[int], mode: int, limit=None) -> Tuple[List[int], int, int, int]:
        """-> (slot of each id or -1, hits, misses, dropped); `limit` (PREFETCH only): copies this
        call may start at most, None = no bound"""
        ids = list(ids)
        assert len(set(ids)) == len(ids) and all(0 <= e < self.E for e in ids)
        needed = set(ids)
        self.clock += 1
        hits = misses = dropped = 0
        if mode == DEMAND:
            assert len(ids) <= self.n_slots
            self.epoch += 1
            for e in sorted(ids):
                s = self.slot_of(e)
                if s >= 0:
                    self.stamp[s] = self.clock
                    self.demand_epoch[s] = self.epoch
                    hits += 1
            for e in sorted(ids):
                if self.slot_of(e) >= 0:
                    continue
                v = self._victim(needed, None)
                self.slot_expert[v] = e
                self.stamp[v] = self.clock
                self.demand_epoch[v] = self.epoch
                misses += 1
            return [self.slot_of(e) for e in ids], hits, misses, 0
        out = []
        for e in ids:
            s = self.slot_of(e)
            if s >= 0:
                self.stamp[s] = self.clock
                hits += 1
                out.append(s)
                continue
            v = self._victim(needed, self.epoch if self.epoch > 0 else None)
            if v < 0 or (limit is not None and misses >= limit):
                dropped += 1
                out.append(-1)
                continue
            self.slot_expert[v] = e
            self.stamp[v] = self.clock
            misses += 1
            out.append(v)
        return out, hits, misses, dropped
