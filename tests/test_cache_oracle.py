"""Pins for the feature-cache oracle (oracle/cache_oracle.py): with batches of one access it must
be a textbook LRU / FIFO cache, the score rules of the paper's section 4.3 are checked on a
hand-worked sequence, and properties that hold for any input are checked on random batches."""
from collections import OrderedDict, deque

import numpy as np
import pytest

from oracle import cache_oracle as CO


def make_store(n, d, seed=0):
    return np.random.default_rng(seed).standard_normal((n, d)).astype(np.float32)


def test_batch_of_one_is_textbook_lru():
    n, cap = 50, 7
    store = make_store(n, 4)
    c = CO.VectorCache(n, cap, 4, CO.LRU, lam=1.0)
    ref = OrderedDict()
    rng = np.random.default_rng(1)
    for i in rng.zipf(1.3, 3000) % n:
        out, hit = c.fetch([i], store)
        assert np.array_equal(out[0], store[i])
        assert bool(hit[0]) == (i in ref)
        if i in ref:
            ref.move_to_end(i)
        else:
            if len(ref) == cap:
                ref.popitem(last=False)
            ref[i] = True
        assert set(c.id_of[c.id_of >= 0]) == set(ref)


def test_batch_of_one_is_textbook_fifo():
    n, cap = 40, 5
    store = make_store(n, 3)
    c = CO.VectorCache(n, cap, 3, CO.FIFO, lam=1.0)
    ref = deque()
    rng = np.random.default_rng(2)
    for i in rng.integers(0, n, 2000):
        out, hit = c.fetch([i], store)
        assert bool(hit[0]) == (i in ref)
        if i not in ref:
            if len(ref) == cap:
                ref.popleft()
            ref.append(i)
        assert set(c.id_of[c.id_of >= 0]) == set(ref)


def test_score_rules_hand_worked():
    # capacity 4, lambda 0.5: at most 2 replacements per update
    store = make_store(10, 2)
    c = CO.VectorCache(10, 4, 2, CO.LRU, lam=0.5)
    assert list(c.score) == [0, 0, 0, 0]                       # "initially, all recent scores are 0"
    _, hit = c.fetch([5, 6, 7], store)                         # three distinct misses, two may enter
    assert not hit.any()
    assert list(c.id_of) == [5, 6, -1, -1]                     # ties on the score: lowest slots first
    assert list(c.score) == [0, 0, -1, -1]                     # all decremented, new entries start at 0
    _, hit = c.fetch([5, 7, 7, 8], store)
    assert list(hit) == [True, False, False, False]
    # all decremented (-1,-1,-2,-2), the access resets slot 0, the two lowest are replaced
    assert list(c.id_of) == [5, 6, 7, 8] and list(c.score) == [0, -1, 0, 0]
    _, hit = c.fetch([9, 6], store)
    assert list(hit) == [False, True]
    # scores before replacement: (-1, 0, -1, -1): slot 0 is the lowest-numbered of the lowest
    assert list(c.id_of) == [9, 6, 7, 8] and list(c.score) == [0, 0, -1, -1]
    assert c.slot_of[5] == -1 and c.slot_of[9] == 0 and (c.hits, c.misses, c.replaced) == (2, 7, 5)


def test_lfu_counts_hand_worked():
    store = make_store(10, 2)
    c = CO.VectorCache(10, 2, 2, CO.LFU, lam=1.0)
    c.fetch([1, 2], store)
    assert list(c.id_of) == [1, 2] and list(c.score) == [1, 1]
    c.fetch([1, 1, 3], store)                                  # two more accesses of id 1; id 3 replaces id 2
    assert list(c.id_of) == [1, 3] and list(c.score) == [3, 1]
    c.fetch([4, 3, 3], store)                                  # id 3 now has 3 accesses, tie with id 1: lower slot goes
    assert list(c.id_of) == [4, 3] and list(c.score) == [1, 3]


@pytest.mark.parametrize("policy", [CO.LRU, CO.LFU, CO.FIFO])
def test_properties_on_random_batches(policy):
    n, cap, d = 500, 64, 5
    store = make_store(n, d, 3)
    c = CO.VectorCache(n, cap, d, policy, lam=0.2)
    rng = np.random.default_rng(4)
    for it in range(200):
        b = int(rng.integers(1, 90))
        ids = (rng.zipf(1.2, b) % n).astype(np.int32)
        before = c.replaced
        cached_before = set(c.id_of[c.id_of >= 0])
        out, hit = c.fetch(ids, store)
        assert np.array_equal(out, store[ids])                                 # transparent
        assert np.array_equal(hit, np.array([i in cached_before for i in ids]))   # looked up before the update
        assert c.replaced - before <= int(np.floor(np.float32(0.2) * np.float32(cap)))   # lambda cap
        assert c.replaced - before == min(len(set(ids[~hit])), 12)
        occ = c.id_of >= 0
        assert np.array_equal(c.slot_of[c.id_of[occ]], np.nonzero(occ)[0])     # the two maps are inverse
        assert (c.slot_of >= 0).sum() == occ.sum()
        assert np.array_equal(c.data[occ], store[c.id_of[occ]])               # cached rows are the true rows
