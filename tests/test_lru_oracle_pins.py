"""Pins of the LRU cache model (oracle/lru_oracle.py) -- CPU only.

The model is checked against things it does not define itself: the textbook per-item LRU (an ordered dict)
on access sequences where the two must coincide, the defining invariant of LRU (nothing outside the cache
was used more recently than anything inside), capacity and bookkeeping identities, and the stated tie rules
on a hand-worked example.
"""
from collections import OrderedDict

import numpy as np
import pytest

from oracle.lru_oracle import LruCache


def _textbook(capacity, sequence):
    od, trace = OrderedDict(), []
    for r in sequence:
        if r in od:
            od.move_to_end(r)
            trace.append(True)
        else:
            if len(od) == capacity:
                od.popitem(last=False)
            od[r] = True
            trace.append(False)
    return trace, set(od)


@pytest.mark.parametrize("capacity,space,n,seed", [(4, 9, 400, 0), (16, 40, 2000, 1), (1, 3, 50, 2), (8, 8, 100, 3)])
def test_single_row_calls_are_the_textbook_lru(capacity, space, n, seed):
    rng = np.random.default_rng(seed)
    seq = [int(x) for x in rng.zipf(1.3, size=n) % space]
    want_trace, want_set = _textbook(capacity, seq)
    c = LruCache(capacity, age_max=10 ** 9)
    got = [c.access([r]) == (1, 0) for r in seq]
    assert got == want_trace
    assert set(c.where) == want_set
    assert c.misses == want_trace.count(False) and c.requested == n


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_nothing_outside_was_used_more_recently_than_anything_inside(seed):
    rng = np.random.default_rng(seed)
    C = 24
    c = LruCache(C, age_max=10 ** 9)
    last_use = {}
    for step in range(1, 200):
        rows = set(int(x) for x in rng.integers(0, 90, size=rng.integers(1, 13)))
        c.access(rows)
        for r in rows:
            last_use[r] = step
        inside = set(c.where)
        assert rows <= inside and len(inside) <= C
        assert len(inside) == min(C, len(last_use))                      # never an empty slot beside an evicted row
        outside = set(last_use) - inside
        if inside and outside:
            assert max(last_use[r] for r in outside) <= min(last_use[r] for r in inside)
        # the two maps agree
        assert all(c.slot_row[s] == r for r, s in c.where.items())
        assert sum(x is not None for x in c.slot_row) == len(inside)


def test_bookkeeping_identities():
    rng = np.random.default_rng(5)
    c = LruCache(10)
    total = 0
    for _ in range(300):
        rows = set(int(x) for x in rng.integers(0, 50, size=6))
        hits, misses = c.access(list(rows) + list(rows)[:2])             # duplicates in a call count once
        assert hits + misses == len(rows)
        total += len(rows)
    assert c.misses - c.written_back == len(c.where) == 10               # every miss either filled an empty slot or replaced a row
    assert c.requested == total
    with pytest.raises(ValueError):
        LruCache(3).access([1, 2, 3, 4])


def test_tie_rules_on_a_worked_example():
    c = LruCache(4)
    c.access([10, 20])            # step 1: slots 0, 1 (empty slots are the oldest; lower index first)
    assert c.where == {10: 0, 20: 1}
    c.access([30, 40])            # step 2: slots 2, 3
    c.access([10])                # step 3: slot 0 refreshed
    # step 4: two misses; ages now: slot0 = 1, slot1 = 3, slot2 = slot3 = 2 -> slot 1 (strictly older) first, then
    # the lower of the two slots of equal age
    c.access([5, 7])
    assert c.where == {10: 0, 5: 1, 7: 2, 40: 3}
    assert c.written_back == 2


def test_ages_beyond_the_horizon_are_equal():
    c = LruCache(3, age_max=3)
    c.access([1])                 # slot 0, step 1
    c.access([2])                 # slot 1, step 2
    c.access([3])                 # slot 2, step 3
    c.access([3])                 # step 4
    c.access([3])                 # step 5: ages 4, 3, 0 -> rows cap at age_max - 1 = 2: slot order decides, not true age
    c.access([9])                 # replaces slot 0 (row 1), as true LRU would
    assert c.where == {9: 0, 2: 1, 3: 2}
    c2 = LruCache(3, age_max=3)
    for r in ([2], [1], [3], [3], [3]):   # now the truly oldest row (2) sits in slot 0 as well
        c2.access(r)
    c2.access([3, 7])             # one miss: slot 0 again, by slot order
    assert c2.where == {7: 0, 1: 1, 3: 2}
