"""Oracle of the host-memory parameter cache of the MEM-PS (paper: Appendix D "MEM-PS
Implementation", cache policy; Section 5; Algorithm 1's collect / update-local-cache / dump
steps).

TEST INFRASTRUCTURE ONLY, like the rest of this package: a plain, slow model written with
Python lists and dicts so that it can be checked against the appendix by eye.  It shares
nothing with the product's implementation (paper_2003_05622_amd/csrc/mem_tier.hpp).

The policy, step by step as the appendix states it:
  * a parameter that is visited is put into an LRU cache (at its most-recently-used end);
  * a parameter evicted from the LRU cache is inserted into an LFU cache;
  * a parameter evicted from the LFU cache is collected: it has to be flushed to the SSD tier
    before its memory is released;
  * the working parameters of the current batch and the parameters fetched ahead for coming
    batches are pinned in the LRU cache: they cannot leave the memory until their batch is
    completed.

Readings where the appendix is silent (the product follows the same ones):
  * capacities are numbers of parameters: lru_capacity and lfu_capacity;
  * evictions happen when a batch completes (nothing can be evicted before, its parameters are
    pinned): while the LRU cache holds more than lru_capacity parameters, its least recently
    visited UNPINNED parameter moves to the LFU cache; while the LFU cache holds more than
    lfu_capacity, its least frequently visited parameter is collected;
  * a parameter's frequency is the number of times it has been visited since it last entered
    the memory; it survives the move between the two caches and is lost with a flush;
  * LFU ties go to the parameter that entered the LFU cache first;
  * a parameter in the LFU cache that is visited moves back to the LRU cache;
  * a parameter visited by several batches (the current one and ones fetched ahead) stays
    pinned until all of them are completed.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np


class MemTierOracle:
    def __init__(self, dim: int, acc_len: int, lru_capacity: int, lfu_capacity: int):
        self.dim, self.acc_len = dim, acc_len
        self.lru_capacity, self.lfu_capacity = lru_capacity, lfu_capacity
        self.lru: List[int] = []            # most recently visited first
        self.lfu: List[int] = []            # in the order they entered the LFU cache
        self.rows: Dict[int, Tuple[np.ndarray, np.ndarray]] = {}
        self.freq: Dict[int, int] = {}
        self.pins: Dict[int, int] = {}      # key -> number of uncompleted batches that visited it
        self.batch_keys: Dict[int, List[int]] = {}
        self.evicted: List[Tuple[int, np.ndarray, np.ndarray]] = []
        self.hits = self.misses = 0

    # -- the visit of Appendix D ---------------------------------------------------------
    def _visit(self, key: int, batch: int) -> None:
        if key in self.lfu:
            self.lfu.remove(key)
        if key in self.lru:
            self.lru.remove(key)
        self.lru.insert(0, key)
        self.freq[key] = self.freq.get(key, 0) + 1
        keys = self.batch_keys.setdefault(batch, [])
        if key not in keys:                 # a batch pins a parameter once, however often it visits it
            keys.append(key)
            self.pins[key] = self.pins.get(key, 0) + 1

    def fetch(self, keys, batch: int):
        """Visits the keys the memory holds; returns (weights, accumulators, found)."""
        keys = [int(k) for k in keys]
        w = np.zeros((len(keys), self.dim), np.float32)
        a = np.zeros((len(keys), self.acc_len), np.float32)
        found = np.zeros(len(keys), bool)
        for i, k in enumerate(keys):
            if k in self.rows:
                self._visit(k, batch)
                w[i], a[i] = self.rows[k]
                found[i] = True
                self.hits += 1
            else:
                self.misses += 1
        return w, a, found

    def store(self, keys, w, a, batch: int, visit: bool) -> None:
        """Puts rows into the memory.  visit=True: the rows come from the tier below (a miss
        being filled): the parameter is visited.  visit=False: updated values of parameters the
        memory already holds (the collect step); a key it does not hold is taken in as a visit."""
        for i, k in enumerate(int(k) for k in keys):
            present = k in self.rows
            self.rows[k] = (np.array(w[i], np.float32), np.array(a[i], np.float32))
            if visit or not present:
                self._visit(k, batch)

    def complete_batch(self, batch: int) -> None:
        for k in self.batch_keys.pop(batch, []):
            self.pins[k] -= 1
            if self.pins[k] == 0:
                del self.pins[k]
        while len(self.lru) > self.lru_capacity:
            victim = None
            for k in reversed(self.lru):        # least recently visited first
                if k not in self.pins:
                    victim = k
                    break
            if victim is None:
                break                            # everything left is pinned
            self.lru.remove(victim)
            self.lfu.append(victim)
        while len(self.lfu) > self.lfu_capacity:
            victim = min(self.lfu, key=lambda k: self.freq[k])    # min() keeps the first of equals
            self.lfu.remove(victim)
            wv, av = self.rows.pop(victim)
            del self.freq[victim]
            self.evicted.append((victim, wv, av))

    def take_evicted(self):
        out, self.evicted = self.evicted, []
        return out
