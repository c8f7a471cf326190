"""CPU oracle of the n-gram cache's life cycle: online insertion, use statistics and eviction.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain Python dictionaries, no shared code with the HIP path.

What the paper fixes:
  * the cache is a set of pairs (target token, [draft tokens]) harvested online; after every speculative step an
    n-gram instance that has not been seen yet is added (Algorithm 1, its last step, the cache update);
  * with a maximum size, "least recently used" evicts the n-gram that has not been accessed for the longest time and
    "least frequently used" removes the n-gram with the lowest access frequency (Appendix, N-gram Cache Scalability).

Readings taken where the paper is silent (mirrored by the library):
  * an *access* is a successful lookup that the translation scan actually uses (the entry becomes a mapped token of
    the proposal), whether or not the target accepts it afterwards;
  * time is a logical clock of the cache: every verification step that uses the cache and every insert call that
    brings at least one pair advances it by one; all entries used in one step carry that step's time; an inserted (or re-inserted) entry carries the
    insert call's time;
  * victims: LRU takes the smallest (last_used, insertion number); LFU the smallest (uses, last_used, insertion
    number).  Eviction happens only when a new key arrives while the cache is full;
  * re-inserting a known key overwrites its target (the last pair wins), refreshes last_used and keeps its uses;
  * without an eviction policy an insert call that would exceed the capacity fails as a whole;
  * an insert call without pairs changes nothing: the clock does not tick (there is no event to date);
  * a saved cache comes back through `load`: the pairs are added in the order given, each with the use count and
    last-use time it was saved with, nothing is evicted, and the clock moves up to the latest of those times, so
    that an export followed by a load into an empty cache continues with the same eviction order.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Tuple

POLICIES = ("none", "lru", "lfu")


class CacheFull(Exception):
    pass


class NgramCache:
    def __init__(self, capacity: int, policy: str = "none"):
        assert policy in POLICIES and capacity >= 0
        self.capacity = capacity
        self.policy = policy
        self.clock = 0
        self._seq = 0
        # key -> [target, uses, last_used, insertion number]
        self.entries: Dict[Tuple[int, ...], List[int]] = {}

    # ------------------------------------------------------------------ views
    def as_dict(self) -> Dict[Tuple[int, ...], int]:
        """The mapping the translation scan looks keys up in."""
        return {k: v[0] for k, v in self.entries.items()}

    def __len__(self) -> int:
        return len(self.entries)

    def snapshot(self) -> Dict[Tuple[int, ...], Tuple[int, int, int]]:
        """key -> (target, uses, last_used)."""
        return {k: (v[0], v[1], v[2]) for k, v in self.entries.items()}

    # ------------------------------------------------------------------ updates
    def _victim(self) -> Tuple[int, ...]:
        if self.policy == "lru":
            return min(self.entries, key=lambda k: (self.entries[k][2], self.entries[k][3]))
        return min(self.entries, key=lambda k: (self.entries[k][1], self.entries[k][2], self.entries[k][3]))

    def insert(self, items: Iterable[Tuple[Tuple[int, ...], int]]) -> int:
        """Adds (key, target) pairs in order; returns the number of evicted entries."""
        items = [(tuple(int(x) for x in k), int(t)) for k, t in items]
        if not items:
            return 0
        if self.policy == "none":
            new_keys = {k for k, _ in items if k not in self.entries}
            if len(self.entries) + len(new_keys) > self.capacity:
                raise CacheFull(f"{len(new_keys)} new keys do not fit into {self.capacity - len(self.entries)} free places")
        elif self.capacity == 0 and items:
            raise CacheFull("capacity 0")
        self.clock += 1
        evicted = 0
        for key, target in items:
            e = self.entries.get(key)
            if e is not None:
                e[0] = target
                e[2] = self.clock
                continue
            if len(self.entries) >= self.capacity:
                del self.entries[self._victim()]
                evicted += 1
            self.entries[key] = [target, 0, self.clock, self._seq]
            self._seq += 1
        return evicted

    def load(self, items: Iterable[Tuple[Tuple[int, ...], int, int, int]]) -> None:
        """Adds (key, target, uses, last_used) in order, keeping the statistics; evicts nothing."""
        items = [(tuple(int(x) for x in k), int(t), int(u), int(l)) for k, t, u, l in items]
        new_keys = {k for k, _, _, _ in items if k not in self.entries}
        if len(self.entries) + len(new_keys) > self.capacity:
            raise CacheFull(f"{len(new_keys)} saved keys do not fit into {self.capacity - len(self.entries)} free places")
        for key, target, uses, last in items:
            e = self.entries.get(key)
            if e is not None:
                e[0], e[1], e[2] = target, uses, last
            else:
                self.entries[key] = [target, uses, last, self._seq]
                self._seq += 1
            self.clock = max(self.clock, last)

    def export(self) -> List[Tuple[Tuple[int, ...], int, int, int]]:
        """(key, target, uses, last_used) in insertion order."""
        return [(k, v[0], v[1], v[2]) for k, v in sorted(self.entries.items(), key=lambda kv: kv[1][3])]

    def record_step(self, used_keys: Iterable[Tuple[int, ...]]) -> None:
        """One verification step used these keys (with multiplicity)."""
        self.clock += 1
        for key in used_keys:
            e = self.entries[tuple(int(x) for x in key)]
            e[1] += 1
            e[2] = self.clock
