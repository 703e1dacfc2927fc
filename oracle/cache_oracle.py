"""Oracle of the schedule cache (TEST INFRASTRUCTURE ONLY, see oracle/__init__.py).

The paper caches the rewritten graph and reuses it when the same structure comes back
(section 4.3).  This library keys a cache of schedules by a fingerprint of the parent
array; the paper fixes no hash, so the definition below is this library's own and the
oracle is that definition written out with Python integers:

    word_i = i * 2^32 + (parent[i] mod 2^32)
    fp[0]  = sum_i mix64((word_i + GOLDEN) mod 2^64)   mod 2^64
    fp[1]  = sum_i mix64(word_i xor KEY1)              mod 2^64

mix64 is the output function of SplitMix64 (Steele, Lea, Flood, "Fast splittable
pseudorandom number generators", OOPSLA 2014) and GOLDEN its increment, so that
mix64(GOLDEN), mix64(2 GOLDEN), ... is the published SplitMix64 stream for seed 0, which
pins mix64 to values outside this repository.  A sum is used because it does not depend
on the order in which a parallel reduction adds; every term depends on the position, so
permuting entries changes the sums.

LruModel is the cache's replacement policy in a dozen lines: least recently used out,
a lookup counts as a use.
"""
from __future__ import annotations

from collections import OrderedDict

import numpy as np

MASK = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
KEY1 = 0xD1B54A32D192ED03


def mix64(z: int) -> int:
    z &= MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def fingerprint(parent) -> tuple:
    """Plain loop over the nodes with Python integers."""
    f0 = f1 = 0
    for i, p in enumerate(np.asarray(parent).tolist()):
        word = (i << 32) | (p & 0xFFFFFFFF)
        f0 = (f0 + mix64(word + GOLDEN)) & MASK
        f1 = (f1 + mix64(word ^ KEY1)) & MASK
    return f0, f1


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def fingerprint_fast(parent) -> tuple:
    """The same sums with wrapping uint64 numpy arithmetic, for forests of millions of nodes
    (checked against fingerprint() in the tests)."""
    p = np.asarray(parent, dtype=np.int32)
    with np.errstate(over="ignore"):
        word = (np.arange(p.shape[0], dtype=np.uint64) << np.uint64(32)) | p.view(np.uint32).astype(np.uint64)
        f0 = _mix64_np(word + np.uint64(GOLDEN)).sum(dtype=np.uint64)
        f1 = _mix64_np(word ^ np.uint64(KEY1)).sum(dtype=np.uint64)
    return int(f0), int(f1)


class LruModel:
    """capacity slots; lookup(key) -> slot or -1 (a hit becomes most recent);
    insert(key) -> (slot, evicted): a free slot while there is one (lowest index first),
    else the slot of the least recently used key, which is dropped."""

    def __init__(self, capacity: int):
        self.capacity = capacity
        self.order = OrderedDict()      # key -> slot, oldest first

    def lookup(self, key) -> int:
        if key not in self.order:
            return -1
        self.order.move_to_end(key)
        return self.order[key]

    def insert(self, key):
        if key in self.order:
            self.order.move_to_end(key)
            return self.order[key], False
        if len(self.order) < self.capacity:
            used = set(self.order.values())
            slot = min(s for s in range(self.capacity) if s not in used)
            self.order[key] = slot
            return slot, False
        _, slot = self.order.popitem(last=False)
        self.order[key] = slot
        return slot, True
