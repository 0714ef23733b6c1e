"""Pins of the cache-policy simulator: with one block touched per call it is
textbook LRU (checked against an OrderedDict LRU); with several it obeys the
stated batch rules."""
from collections import OrderedDict

import numpy as np

from oracle.lru import LruBank


def textbook_lru(trace, capacity):
    """Classic LRU: returns (hits, misses, final resident set)."""
    od, hits, misses = OrderedDict(), 0, 0
    for b in trace:
        if b in od:
            hits += 1
            od.move_to_end(b)
        else:
            misses += 1
            if len(od) == capacity:
                od.popitem(last=False)
            od[b] = True
    return hits, misses, set(od)


def test_single_touch_calls_are_textbook_lru():
    rng = np.random.default_rng(0)
    for capacity in (1, 3, 8):
        trace = rng.zipf(1.3, 600) % 40
        bank = LruBank(40, capacity)
        for b in trace:
            bank.call([int(b)])
        hits, misses, resident = textbook_lru(trace.tolist(), capacity)
        assert (bank.hits, bank.misses) == (hits, misses)
        assert {b for b in bank.slot_block if b >= 0} == resident
        for b, s in enumerate(bank.page_table):
            assert (s >= 0) == (b in resident)
            if s >= 0:
                assert bank.slot_block[s] == b


def test_batch_rules():
    bank = LruBank(100, 4)
    bank.call([7, 3, 9])                     # cold: inserted in ascending id into slots 0,1,2
    assert bank.slot_block == [3, 7, 9, -1] and (bank.hits, bank.misses) == (0, 3)
    bank.call([3, 50])                       # 3 hit (refreshed), 50 takes the never-used slot
    assert bank.slot_block == [3, 7, 9, 50] and (bank.hits, bank.misses) == (1, 4)
    bank.call([60, 61])                      # evicts the two oldest: 7 (slot 1) and 9 (slot 2)
    assert bank.slot_block == [3, 60, 61, 50]
    assert bank.page_table[7] == -1 and bank.page_table[9] == -1 and bank.page_table[60] == 1
    bank.call([1, 2, 3, 4, 5, 6])            # 3 hits and stays; 5 misses, 3 older slots: lowest 3 ids go in
    assert bank.slot_block == [3, 1, 2, 4]
    assert bank.last_misses == 5 and bank.last_touched == 6
    assert bank.page_table[3] == 0 and bank.page_table[5] == -1 and bank.page_table[6] == -1
