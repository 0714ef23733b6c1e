"""Plain simulation of the hot-block cache policy (one bank).  TEST
INFRASTRUCTURE ONLY.

Policy (Sec. 4 "KV Cache Offloading": a GPU key bank acting as a cache, a page
table from global key index to bank index, LRU eviction; Alg. 4: the misses of
a layer call are collected and inserted after it).  Granularity and tie rules
are this build's reading: blocks of block_tokens tokens; all touches of one
call share the call's stamp; after the call the missed blocks, in ascending
block id, replace the slots with the oldest stamps (lowest slot on a tie,
never-used slots first); a slot touched in this same call is never evicted
(both blocks were just used: a tie, and swapping them buys nothing); if more
blocks were missed than there are such slots only the lowest-numbered ones are
inserted.
"""
from __future__ import annotations

from typing import Iterable, List


class LruBank:
    def __init__(self, n_blocks_total: int, n_slots: int):
        self.page_table: List[int] = [-1] * n_blocks_total
        self.slot_block: List[int] = [-1] * n_slots
        self.slot_stamp: List[int] = [0] * n_slots
        self.stamp = 1
        self.hits = 0
        self.misses = 0
        self.last_misses = 0
        self.last_touched = 0

    def call(self, touched: Iterable[int]) -> None:
        """One layer call touching the given global block ids, then the update."""
        touched = sorted(set(int(t) for t in touched))
        missed = [b for b in touched if self.page_table[b] < 0]
        for b in touched:
            s = self.page_table[b]
            if s >= 0:
                self.slot_stamp[s] = self.stamp
        self.hits += len(touched) - len(missed)
        self.misses += len(missed)
        self.last_misses, self.last_touched = len(missed), len(touched)
        eligible = [s for s in range(len(self.slot_block)) if self.slot_stamp[s] != self.stamp]
        n_ins = min(len(missed), len(eligible))
        order = sorted(eligible, key=lambda s: (self.slot_stamp[s], s))
        victims = sorted(order[:n_ins])
        for b, s in zip(missed[:n_ins], victims):
            old = self.slot_block[s]
            if old >= 0:
                self.page_table[old] = -1
            self.slot_block[s] = b
            self.page_table[b] = s
            self.slot_stamp[s] = self.stamp
        self.stamp += 1
