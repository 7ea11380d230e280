"""Plain CPU model of the two-tier KV block store (Sec. 3.1 KV cache manager, Sec. 3.4 unified slot
pool with least-recently-used replacement).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests and the benchmark's checking legs may import this
module.  It shares no code with the HIP path.

What it models.  Every (page, KV head) pair of every layer -- a "slice": one key slice and one value
slice, 8 KiB -- lives in host memory and has a global id.  The GPU holds one pool of `num_slots` slots
shared by all layers (Sec. 3.4); a slot holds one slice.  Attention over a slice that has a slot reads
the slot; over one that has none it reads host memory.  After a layer's attention the store is brought
up to date with the slices that attention actually used (the selected blocks, not anything read ahead
of the stop), the paper's LRU policy at the granularity the GPU works at:

  * the update has a time stamp `now` = one more than the last update's;
  * a used slice that has a slot: the slot's stamp becomes `now` (a hit);
  * the used slices without a slot (misses), in the order (stream, rank in the stream's criticality
    order), are given slots taken from the candidates in the order (stamp, slot index) ascending: empty
    slots (stamp 0) first, then the least recently used;
  * never a candidate: a slot stamped `now` (used by this very update), and a slot whose slice lies in
    the caller's `busy` id range (the layer whose attention runs while this update does: its slots are
    being read);
  * if there are more misses than candidates the first misses in that order get the slots and the
    rest stay in host memory.

(The GPU path lets ages saturate at 65535 updates; the model does not, and no test runs that long.)

With one used slice per update and no busy range this is textbook LRU; tests/test_tier_oracle.py pins it to
the textbook's worked reference string and to an independent ordered-dictionary LRU on random traces.
A slice used by two streams in one update (a page shared between requests) is outside the model: it
asserts that each update's used ids are distinct.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class UpdateStats:
    hits: int
    misses: int
    promoted: int
    evicted: int


def used_slices(block_table: np.ndarray, order: np.ndarray, blocks_read: np.ndarray, num_kv_heads: int,
                slice_base: int) -> np.ndarray:
    """Global ids of the slices a decode call used, in (stream, rank) order.

    block_table [B][max_blocks] physical page per logical block; order [B][H][max_blocks] ranked logical
    blocks per stream; blocks_read [B][H] how many of them the stream's attention used.  A slice's id is
    slice_base + page * H + h.
    """
    B, H = blocks_read.shape
    assert H == num_kv_heads
    ids = []
    for r in range(B):
        for h in range(H):
            n = int(blocks_read[r, h])
            logical = order[r, h, :n].astype(np.int64)
            assert (logical >= 0).all()
            pages = block_table[r, logical].astype(np.int64)
            ids.append(slice_base + pages * H + h)
    return np.concatenate(ids) if ids else np.zeros(0, dtype=np.int64)


class TierModel:
    def __init__(self, total_slices: int, num_slots: int):
        self.slot_of = np.full(total_slices, -1, dtype=np.int64)   # slice id -> slot, -1 = host memory only
        self.owner = np.full(num_slots, -1, dtype=np.int64)        # slot -> slice id, -1 = empty
        self.stamp = np.zeros(num_slots, dtype=np.int64)           # slot -> time of last use, 0 = never
        self.clock = 0

    def resident(self, ids) -> np.ndarray:
        return self.slot_of[np.asarray(ids, dtype=np.int64)] >= 0

    def update(self, used_ids, busy_first: int = 0, busy_count: int = 0) -> UpdateStats:
        used = np.asarray(used_ids, dtype=np.int64)
        assert len(np.unique(used)) == len(used), "a slice used twice in one update is outside the model"
        now = self.clock + 1
        misses = []
        hits = 0
        for i in used:
            slot = self.slot_of[i]
            if slot >= 0:
                self.stamp[slot] = now
                hits += 1
            else:
                misses.append(int(i))
        cand = []
        for slot in range(len(self.owner)):
            if self.stamp[slot] >= now:
                continue
            o = self.owner[slot]
            if o >= 0 and busy_first <= o < busy_first + busy_count:
                continue
            cand.append((int(self.stamp[slot]), slot))
        cand.sort()
        take = min(len(misses), len(cand))
        evicted = 0
        for j in range(take):
            slot = cand[j][1]
            old = self.owner[slot]
            if old >= 0:
                self.slot_of[old] = -1
                evicted += 1
            self.owner[slot] = misses[j]
            self.slot_of[misses[j]] = slot
            self.stamp[slot] = now
        self.clock = now
        return UpdateStats(hits, len(misses), take, evicted)
