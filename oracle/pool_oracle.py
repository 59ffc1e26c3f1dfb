"""Reference residency policy for on-demand swapping -- TEST INFRASTRUCTURE ONLY (nothing in the product path
may import this).

The paper (Section 4.1, "On-demand swapping") only says that the compressed deltas a query needs are loaded
when needed while the base model stays resident; it names no replacement policy.  The reading taken: least
recently used, stated here as its plain definition.

  - `n_slots` slots, all free at the start.  A request is a list of distinct experts, at most n_slots of them.
  - An expert that sits in a slot is a hit; every expert of the request counts as used "now" (one time stamp per
    request), so no expert of a request can be evicted for another expert of the same request.
  - Misses are served in the order asked.  The victim is the slot whose time stamp is smallest among the slots
    not used by this request (a free slot has stamp 0, i.e. goes first); the lowest slot index wins ties.
  - A prefetch (loading ahead of need -- the paper does not describe one; this is the plain extension of the rule
    above) is a request that may only overwrite slots the latest acquire did not use and no later prefetch has
    filled: free slots, and slots whose stamp is older than the latest acquire's.  Its resident experts are
    stamped "now" like an acquire's; the others are loaded in the order asked into the oldest such slot, and
    skipped when none is left.  It counts neither hits nor misses.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


class LruPool:
    def __init__(self, n_slots: int):
        self.slot_expert: List[int] = [-1] * n_slots
        self.slot_stamp: List[int] = [0] * n_slots
        self.clock = 0
        self.last_acquire = 0
        self.hits = 0
        self.misses = 0
        self.prefetched = 0

    def slot_of(self, expert: int) -> int:
        return self.slot_expert.index(expert) if expert in self.slot_expert else -1

    def acquire(self, experts: Sequence[int]) -> Tuple[List[int], List[int]]:
        """Returns (slot of every expert in request order, experts that had to be loaded in load order)."""
        assert len(set(experts)) == len(experts) and 0 < len(experts) <= len(self.slot_expert)
        self.clock += 1
        self.last_acquire = self.clock
        for e in experts:
            if e in self.slot_expert:
                self.slot_stamp[self.slot_expert.index(e)] = self.clock
                self.hits += 1
        loaded = []
        for e in experts:
            if e not in self.slot_expert:
                candidates = [s for s in range(len(self.slot_expert)) if self.slot_stamp[s] != self.clock]
                victim = min(candidates, key=lambda s: (self.slot_stamp[s], s))
                self.slot_expert[victim] = e
                self.slot_stamp[victim] = self.clock
                self.misses += 1
                loaded.append(e)
        return [self.slot_expert.index(e) for e in experts], loaded

    def prefetch(self, experts: Sequence[int]) -> List[int]:
        """Returns the experts that were loaded, in load order."""
        assert len(set(experts)) == len(experts) and 0 < len(experts) <= len(self.slot_expert)
        self.clock += 1
        for e in experts:
            if e in self.slot_expert:
                self.slot_stamp[self.slot_expert.index(e)] = self.clock
        loaded = []
        for e in experts:
            if e in self.slot_expert:
                continue
            candidates = [s for s in range(len(self.slot_expert))
                          if self.slot_stamp[s] == 0 or self.slot_stamp[s] < self.last_acquire]
            if not candidates:
                continue
            victim = min(candidates, key=lambda s: (self.slot_stamp[s], s))
            self.slot_expert[victim] = e
            self.slot_stamp[victim] = self.clock
            self.prefetched += 1
            loaded.append(e)
        return loaded
