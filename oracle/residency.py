"""CPU oracle of the residency bookkeeping: which groups are in device memory
after each planning step, which of the selected ones were found there (the
cache hit rate of Section 4, "memory caching distribution and cache hit
rate"), which had to be loaded (Section 3.2: only the selected groups are
loaded; a group selected in consecutive steps is already in device memory).

TEST INFRASTRUCTURE ONLY, like the rest of this package: plain Python over
dictionaries, one operation at a time, nothing shared with the library.

The paper fixes what is counted (hit = a selected group already in device
memory) but not which resident group gives way when device memory is full. The
reading taken here: the one used least recently, where "used" means asked for
by a step's selection; every group of one selection is as recent as the others.

Rules, in the order a step applies them
  fetch(groups)     1. every asked-for group that is resident is marked as used
                       now (so none of them can be displaced by this step);
                    2. in list order, every other asked-for group takes the slot
                       whose last use is oldest; a slot never used is older than
                       any used one; among equally old slots the lowest number;
                       Before the first load of a step, if the last fence is older
                       than the previous step, the step fences for itself: everything
                       up to the previous step counts as fenced from then on;
                    3. returns the slot of every group, and per group one of
                       "hit" (resident from an earlier fetch), "prefetched"
                       (resident because of a prefetch, first time asked for),
                       "miss" (loaded now).
  fence()           from here on the slots handed out so far may be overwritten
                       without waiting (their readers are already queued).
  prefetch(groups)  asked-for groups that are resident stay; every other one, in
                       list order, takes the oldest slot among those whose last
                       use is not after the last fence and that holds none of
                       the asked-for groups; stops when there is none. A slot
                       filled this way is as old as the last fence.
  put(group)        the group's data changed: its device copy, if any, is
                       dropped; the slot keeps its age.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

NEVER = -1


class Residency:
    def __init__(self, n_slots: int):
        self.n_slots = n_slots
        self.group_in: Dict[int, int] = {}      # slot -> group
        self.age: Dict[int, int] = {s: NEVER for s in range(n_slots)}   # slot -> step of last use
        self.ahead = set()                      # slots filled by a prefetch and not yet asked for
        self.step = 0
        self.fenced = NEVER
        self.hits = self.prefetched = self.misses = self.loads = self.evictions = self.requested = 0

    def slot_of(self, group: int) -> int:
        for s, g in self.group_in.items():
            if g == group:
                return s
        return -1

    def resident(self) -> set:
        return set(self.group_in.values())

    def _oldest(self, candidates: Sequence[int]) -> int:
        best = None
        for s in sorted(candidates):
            if best is None or self.age[s] < self.age[best]:
                best = s
        return -1 if best is None else best

    def _load(self, group: int, slot: int):
        if slot in self.group_in:
            self.evictions += 1
        self.group_in[slot] = group
        self.loads += 1

    def fetch(self, groups: Sequence[int]) -> Tuple[List[int], List[str]]:
        assert len(set(groups)) == len(groups) <= self.n_slots
        self.step += 1
        self.requested += len(groups)
        kind = {}
        for g in groups:
            s = self.slot_of(g)
            if s >= 0:
                self.age[s] = self.step
                if s in self.ahead:
                    self.ahead.discard(s)
                    kind[g] = "prefetched"
                    self.prefetched += 1
                else:
                    kind[g] = "hit"
                    self.hits += 1
        for g in groups:
            if g in kind:
                continue
            if self.step > 1 and self.fenced < self.step - 1:
                self.fenced = self.step - 1         # a fetch that has to load fences for itself
            s = self._oldest([s for s in range(self.n_slots) if self.age[s] < self.step])
            assert s >= 0
            self._load(g, s)
            self.ahead.discard(s)
            self.age[s] = self.step
            kind[g] = "miss"
            self.misses += 1
        return [self.slot_of(g) for g in groups], [kind[g] for g in groups]

    def fence(self):
        self.fenced = self.step

    def prefetch(self, groups: Sequence[int]) -> int:
        assert len(set(groups)) == len(groups) <= self.n_slots
        keep = {self.slot_of(g) for g in groups if self.slot_of(g) >= 0}
        n = 0
        for g in groups:
            if self.slot_of(g) >= 0:
                continue
            s = self._oldest([s for s in range(self.n_slots) if s not in keep and self.age[s] <= self.fenced])
            if s < 0:
                break
            self._load(g, s)
            keep.add(s)
            self.age[s] = self.fenced
            self.ahead.add(s)
            n += 1
        return n

    def put(self, group: int):
        s = self.slot_of(group)
        if s >= 0:
            del self.group_in[s]
            self.ahead.discard(s)

    def hit_rate(self) -> float:
        return self.hits / self.requested if self.requested else 0.0
