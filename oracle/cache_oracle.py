"""TEST INFRASTRUCTURE -- not part of the product path.

Plain numpy/Python statement of the vectorised feature cache of the paper (section 4.3,
"Vectorized cache"): a dynamic cache whose entries are looked up and updated a whole batch
at a time.

  * one "recent score" per entry, 0 = most recently used; initially all 0; every update
    decrements all scores by 1; an access resets the entry's score to 0; replacement evicts
    the entries with the lowest scores (LRU);
  * LFU: the score is an access count instead;
  * FIFO: a ring buffer whose pointer moves by the number of replaced entries;
  * at most a fraction lambda of the capacity is replaced per update (default 0.2).

Where the paper is silent, the readings are:
  R1  a batch is looked up against the cache as it was BEFORE the batch (vectorised: no entry
      inserted by the batch can be hit by the same batch);
  R2  a fetch always returns the true feature row (hit: from the cache, miss: from the
      backing store), so the cache is transparent;
  R3  duplicates: every occurrence of a cached id counts as an access (LFU adds 1 per
      occurrence); a missed id is inserted once, missed ids are taken in the order of their
      first occurrence in the batch;
  R4  number inserted per update: m = min(#distinct missed ids, floor(lambda * capacity));
  R5  victims: the m entries with the lowest score, ties broken by the lower slot index
      (empty slots compete like any other entry: their scores only ever decrease, so they
      go first); the i-th victim in ascending slot order receives the i-th missed id;
  R6  a new entry starts with score 0 (LRU) or 1 (LFU: its first access);
  R7  order inside one update: scores are decremented / reset (accesses of the batch), then
      the victims are chosen, so an entry hit by the batch has the highest score.

Pins: tests/test_cache_oracle.py (batch size 1 equals a textbook LRU / FIFO, the paper's
score rules on a hand-worked sequence, transparency, the lambda cap, map invariants).
"""
from __future__ import annotations

import numpy as np

LRU, LFU, FIFO = 0, 1, 2


class VectorCache:
    def __init__(self, num_ids: int, capacity: int, dim: int, policy: int = LRU, lam: float = 0.2):
        assert capacity >= 1 and 0 < lam <= 1
        self.num_ids, self.capacity, self.dim, self.policy, self.lam = num_ids, capacity, dim, policy, lam
        self.slot_of = np.full(num_ids, -1, np.int32)
        self.id_of = np.full(capacity, -1, np.int32)
        self.score = np.zeros(capacity, np.int32)
        self.data = np.zeros((capacity, dim), np.float32)
        self.ring = 0
        self.hits = self.misses = self.replaced = 0

    @property
    def max_replace(self) -> int:
        return int(np.floor(np.float32(self.lam) * np.float32(self.capacity)))

    def fetch(self, ids: np.ndarray, store: np.ndarray):
        """Returns (rows [B, dim], hit [B] bool) and updates the cache."""
        ids = np.asarray(ids, np.int32)
        slots = self.slot_of[ids]                       # R1: state before the batch
        hit = slots >= 0
        out = np.empty((len(ids), self.dim), np.float32)
        out[hit] = self.data[slots[hit]]                # R2
        out[~hit] = store[ids[~hit]]
        self.hits += int(hit.sum())
        self.misses += int((~hit).sum())

        # accesses of the batch (R3, R7)
        if self.policy == LRU:
            self.score -= 1
            self.score[slots[hit]] = 0
        elif self.policy == LFU:
            np.add.at(self.score, slots[hit], 1)

        # distinct missed ids in order of first occurrence (R3), capped (R4)
        missed = ids[~hit]
        _, first = np.unique(missed, return_index=True)
        new_ids = missed[np.sort(first)]
        m = min(len(new_ids), self.max_replace)
        if m == 0:
            return out, hit
        new_ids = new_ids[:m]
        if self.policy == FIFO:
            victims = (self.ring + np.arange(m)) % self.capacity
            self.ring = int((self.ring + m) % self.capacity)
        else:
            order = np.lexsort((np.arange(self.capacity), self.score))      # by score, then slot (R5)
            victims = np.sort(order[:m])
        for s, i in zip(victims, new_ids):
            old = self.id_of[s]
            if old >= 0:
                self.slot_of[old] = -1
            self.id_of[s] = i
            self.slot_of[i] = s
            self.data[s] = store[i]
            self.score[s] = 1 if self.policy == LFU else 0                   # R6
        self.replaced += m
        return out, hit
