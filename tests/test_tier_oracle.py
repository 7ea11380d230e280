"""CPU pins of the two-tier block store model (oracle/tier_oracle.py): textbook LRU fault counts, an
independent ordered-dictionary LRU on random traces, and the properties of the batched update that the
GPU path is compared against (Sec. 3.4: unified slot pool, LRU eviction)."""
import os
from collections import OrderedDict

import numpy as np
import pytest

from oracle.tier_oracle import TierModel, used_slices

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "lru_reference_strings.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = [int(x) for x in line.split()]
        out.append((f[0], f[1], f[2:]))
    return out


@pytest.mark.parametrize("frames,faults,refs", _cases())
def test_textbook_reference_strings(frames, faults, refs):
    t = TierModel(total_slices=16, num_slots=frames)
    got = sum(t.update([r]).misses for r in refs)
    assert got == faults


def _dict_lru(capacity, refs):
    d, faults, resident_after = OrderedDict(), 0, []
    for r in refs:
        if r in d:
            d.move_to_end(r)
        else:
            faults += 1
            if len(d) == capacity:
                d.popitem(last=False)
            d[r] = True
        resident_after.append(frozenset(d))
    return faults, resident_after


@pytest.mark.parametrize("seed", range(6))
def test_single_access_updates_are_exact_lru(seed):
    rng = np.random.default_rng(seed)
    n_ids, cap = 40, int(rng.integers(1, 12))
    refs = (rng.zipf(1.4, size=400) % n_ids).tolist()
    want_faults, want_sets = _dict_lru(cap, refs)
    t = TierModel(n_ids, cap)
    faults = 0
    for r, want in zip(refs, want_sets):
        faults += t.update([r]).misses
        assert frozenset(np.nonzero(t.slot_of >= 0)[0].tolist()) == want
    assert faults == want_faults


def _consistent(t):
    res = np.nonzero(t.slot_of >= 0)[0]
    assert len(set(t.slot_of[res].tolist())) == len(res)
    for i in res:
        assert t.owner[t.slot_of[i]] == i
    for s, o in enumerate(t.owner):
        if o >= 0:
            assert t.slot_of[o] == s


def test_pool_that_holds_everything_never_misses_twice():
    t = TierModel(100, 64)
    ids = list(range(10, 60))
    s0 = t.update(ids)
    assert (s0.hits, s0.misses, s0.promoted, s0.evicted) == (0, 50, 50, 0)
    for _ in range(3):
        s = t.update(ids[::-1])
        assert (s.hits, s.misses, s.promoted, s.evicted) == (50, 0, 0, 0)
    _consistent(t)
    # empty slots are handed out in slot order, misses in the order given
    assert [t.slot_of[i] for i in ids] == list(range(50))


def test_more_misses_than_slots_keeps_the_first_and_never_evicts_what_the_update_used():
    t = TierModel(100, 8)
    t.update([0, 1, 2, 3])
    s = t.update([3, 2, 50, 51, 52, 53, 54, 55, 56])          # 2 hits, 7 misses, 6 candidates (4 empty + slices 0, 1)
    assert (s.hits, s.misses, s.promoted, s.evicted) == (2, 7, 6, 2)
    assert t.resident([2, 3, 50, 51, 52, 53, 54, 55]).all() and not t.resident([0, 1, 56]).any()
    _consistent(t)


def test_oldest_goes_first_and_ties_go_by_slot_index():
    t = TierModel(100, 4)
    t.update([10, 11])      # slots 0, 1 at time 1
    t.update([12, 13])      # slots 2, 3 at time 2
    t.update([11])          # slice 11 (slot 1) refreshed at time 3
    t.update([20])          # evicts slice 10 (slot 0, time 1)
    assert t.slot_of[20] == 0 and not t.resident([10])[0]
    t.update([21, 22])      # candidates by (stamp, slot): slot 2 (t2), slot 3 (t2), slot 1 (t3)
    assert t.slot_of[21] == 2 and t.slot_of[22] == 3 and t.resident([11])[0]
    _consistent(t)


def test_busy_range_is_not_evicted():
    t = TierModel(100, 4)
    t.update([40, 41, 42, 43])
    s = t.update([1, 2, 3], busy_first=40, busy_count=2)      # only the slots of slices 42, 43 may go
    assert (s.promoted, s.evicted) == (2, 2)
    assert t.resident([40, 41, 1, 2]).all() and not t.resident([42, 43, 3]).any()
    _consistent(t)


def test_used_slices_follow_stream_then_rank_order():
    table = np.array([[5, 6, 7, 8], [9, 10, 11, 12]], dtype=np.int32)
    order = np.array([[[2, 0, 1, 3], [3, 2, 1, 0]], [[0, 1, 2, 3], [1, 0, -1, -1]]], dtype=np.int32)
    read = np.array([[2, 1], [0, 2]], dtype=np.int32)
    ids = used_slices(table, order, read, num_kv_heads=2, slice_base=1000)
    # request 0 head 0: blocks 2, 0 -> pages 7, 5; head 1: block 3 -> page 8; request 1 head 1: blocks 1, 0 -> pages 10, 9
    assert ids.tolist() == [1000 + 7 * 2, 1000 + 5 * 2, 1000 + 8 * 2 + 1, 1000 + 10 * 2 + 1, 1000 + 9 * 2 + 1]


def test_a_slice_used_twice_in_one_update_is_refused():
    t = TierModel(10, 4)
    with pytest.raises(AssertionError):
        t.update([1, 1])
