"""Reference model of the text-keyed chunk index.  TEST INFRASTRUCTURE ONLY.

A plain Python restatement of the storage module's index (Sec. 3.1: KV caches keyed by
texts; Sec. 3.2: store with text, retrieve by text) with a byte capacity and two
eviction rules.  READING (the paper gives no policy): LRU evicts the entry used longest
ago; LFU evicts the entry with the fewest uses (the insert counts as one use), the one
used longest ago among equals.  An insert under an existing key replaces that entry and
reports it as evicted first; further victims follow in eviction order; if the chunk
cannot fit, or more than max_evicted entries would have to go, nothing changes.
"""
from __future__ import annotations

LRU, LFU = 0, 1


class PoolOracle:
    def __init__(self, capacity: int, policy: int = LRU):
        self.capacity, self.policy = capacity, policy
        self.clock = 0
        self.entries: dict[tuple, dict] = {}      # key -> {value, bytes, uses, stamp}
        self.hits = self.misses = self.inserts = self.evictions = 0

    @property
    def bytes(self) -> int:
        return sum(e["bytes"] for e in self.entries.values())

    def lookup(self, key):
        key = tuple(key)
        e = self.entries.get(key)
        if e is None:
            self.misses += 1
            return None
        self.hits += 1
        self.clock += 1
        e["uses"] += 1
        e["stamp"] = self.clock
        return e["value"]

    def insert(self, key, value, nbytes: int, max_evicted: int = 1 << 30):
        """Returns the list of evicted values, or None if refused."""
        key = tuple(key)
        if nbytes > self.capacity:
            return None
        out = []
        total = self.bytes
        if key in self.entries:
            out.append(key)
            total -= self.entries[key]["bytes"]
        others = [k for k in self.entries if k != key]
        if self.policy == LRU:
            others.sort(key=lambda k: self.entries[k]["stamp"])
        else:
            others.sort(key=lambda k: (self.entries[k]["uses"], self.entries[k]["stamp"]))
        for k in others:
            if total + nbytes <= self.capacity:
                break
            out.append(k)
            total -= self.entries[k]["bytes"]
        if total + nbytes > self.capacity or len(out) > max_evicted:
            return None
        values = [self.entries.pop(k)["value"] for k in out]
        self.evictions += len(out)
        self.clock += 1
        self.entries[key] = {"value": value, "bytes": nbytes, "uses": 1, "stamp": self.clock}
        self.inserts += 1
        return values

    def remove(self, key):
        e = self.entries.pop(tuple(key), None)
        return None if e is None else e["value"]
