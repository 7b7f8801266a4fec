"""Pins of the cache-manager oracle (oracle/manager.py) and parity of the library's manager with it.

Section 4.2 of the paper: metadata per cache entry, the compound eviction score with the
coefficients 0.45 / 0.10 / 0.45, reference counters, the sparing of queued requests' adapters,
dynamic sizing.  All host-side: runs without a GPU (the library's cache is created host-only)."""
from __future__ import annotations

import collections
import math

import numpy as np
import pytest

from oracle.manager import CacheManager


def _single_class(n_slots, weights, window=0):
    return CacheManager([128], [n_slots], 1000, weights, window)


def test_hand_worked_scores_with_the_papers_coefficients():
    """Three cached adapters, 20 requests in all; scores worked out by hand from the formula."""
    m = CacheManager([128], [3], 1, (0.45, 0.10, 0.45))
    for _ in range(10):
        m.acquire(1, 8, pin=False)      # requests 1..10: adapter 1, rank 8
    for _ in range(5):
        m.acquire(3, 64, pin=False)     # 11..15: adapter 3, rank 64
    for _ in range(5):
        m.acquire(2, 128, pin=False)    # 16..20: adapter 2, rank 128
    # now: adapter 1: freq 10, last 10; adapter 3: freq 5, last 15; adapter 2: freq 5, last 20; now = 20
    s = m.scores()
    slot = {e.adapter_id: i for i, e in enumerate(m.entries)}
    # ages 10, 5, 0 -> largest 10; frequencies / 10; ranks / 128:
    #   adapter 1: 0.45 * 1.0 + 0.10 * 0.0 + 0.45 * 0.0625 = 0.478125
    #   adapter 3: 0.45 * 0.5 + 0.10 * 0.5 + 0.45 * 0.5    = 0.5
    #   adapter 2: 0.45 * 0.5 + 0.10 * 1.0 + 0.45 * 1.0    = 0.775
    assert s[slot[1]] == pytest.approx(0.478125, abs=1e-15)
    assert s[slot[3]] == pytest.approx(0.5, abs=1e-15)
    assert s[slot[2]] == pytest.approx(0.775, abs=1e-15)
    # the small, old adapter goes first although it is the most frequently used one: size and
    # frequency weigh the same, recency little
    assert m.victim() == slot[1]


def test_recency_only_is_textbook_lru():
    rng = np.random.default_rng(3)
    m = _single_class(8, (0.0, 1.0, 0.0))
    lru = collections.OrderedDict()  # textbook: move to the end on use, pop from the front
    for _ in range(3000):
        a = int(rng.zipf(1.3)) % 40
        slot, hit = m.acquire(a, 16, pin=False)
        assert hit == (a in lru)
        if a in lru:
            lru.move_to_end(a)
        else:
            if len(lru) == 8:
                old, _ = lru.popitem(last=False)
                assert old not in m.where          # the oracle evicted the same adapter
            lru[a] = True
        assert set(m.where) == set(lru)


def test_frequency_only_evicts_the_least_used_and_size_only_the_smallest():
    rng = np.random.default_rng(5)
    ranks = {a: int(rng.choice([8, 16, 32, 64, 128])) for a in range(30)}
    for weights, key in (((1.0, 0.0, 0.0), lambda e: e.freq), ((0.0, 0.0, 1.0), lambda e: e.rank)):
        m = _single_class(6, weights)
        for _ in range(1500):
            a = int(rng.integers(0, 30))
            before = {e.adapter_id: key(e) for e in m.entries if e is not None}
            full = len(before) == 6
            slot, hit = m.acquire(a, ranks[a], pin=False)
            if not hit and full:
                gone = set(before) - set(m.where)
                assert len(gone) == 1
                assert before[gone.pop()] == min(before.values())


def test_entries_in_use_stay_and_queued_ones_go_last():
    rng = np.random.default_rng(7)
    m = CacheManager([8, 32, 128], [3, 3, 2], 64)
    running = collections.deque()
    for step in range(4000):
        a = int(rng.zipf(1.2)) % 60
        rank = [8, 16, 32, 64, 128][a % 5]
        queued = [int(q) for q in rng.integers(0, 60, size=3)]
        pinned_before = {e.adapter_id for e in m.entries if e is not None and e.refcount > 0}
        cached_before = {e.adapter_id: i for i, e in enumerate(m.entries) if e is not None}
        slot, hit = m.acquire(a, rank, pin=True, queued=queued)
        if slot < 0:
            # nothing may go: every large-enough slot holds an entry in use
            assert all(e is not None and e.refcount > 0 for i, e in enumerate(m.entries) if m.slot_class_rank[i] >= rank)
        else:
            assert m.slot_class_rank[slot] >= rank
            running.append(slot)
            gone = set(cached_before) - set(m.where)
            assert not (gone & pinned_before)
            if gone & set(queued):
                # a queued adapter went: then no other unreferenced entry in a large-enough slot was left
                others = [b for b, i in cached_before.items()
                          if b not in pinned_before and b not in queued and m.slot_class_rank[i] >= rank]
                assert not others
        while len(running) > 4:
            m.release(running.popleft())
    assert m.hits + m.misses > 0 and m.evictions > 0


def test_free_slots_come_from_the_smallest_class_that_fits():
    m = CacheManager([8, 32, 128], [1, 1, 1], 64)
    assert m.acquire(1, 8)[0] == 0
    assert m.acquire(2, 8)[0] == 1      # class 8 is full: the rank-8 adapter takes the class-32 slot
    assert m.acquire(3, 64)[0] == 2
    assert m.acquire(4, 64) == (-1, False)  # the only slot that holds rank 64 is in use
    m.release(2)
    assert m.acquire(4, 64) == (2, False) and 3 not in m.where


def test_frequency_window_halves_all_counts():
    m = _single_class(2, (1.0, 0.0, 0.0), window=4)
    for _ in range(3):
        m.acquire(1, 8, pin=False)
    assert m.entries[0].freq == 3.0
    m.acquire(2, 8, pin=False)          # request 4: every count is halved, then this use is added
    assert m.entries[0].freq == 1.5 and m.entries[1].freq == 1.0


def test_trim_stops_when_the_budget_is_met_and_spares_entries_in_use():
    m = CacheManager([8, 128], [2, 3], 100)
    for a, r in ((1, 8), (2, 4), (3, 128), (4, 60), (5, 100)):
        m.acquire(a, r, pin=(a == 3))
    assert m.resident_bytes() == (8 + 8 + 128 + 64 + 104) * 100
    n, ok = m.trim(200 * 100)
    assert ok and m.resident_bytes() <= 200 * 100
    assert 3 in m.where                 # in use: never evicted
    # evicting one entry fewer would not have met the budget: the last victim was needed
    assert n >= 1
    n2, ok2 = m.trim(0)
    assert not ok2 and set(m.where) == {3}
    assert math.isinf(m.scores()[0])


# ---- the library against the oracle --------------------------------------------------------

def _lib_cache(B, class_rank, class_slots):
    cfg = B.make_config([(64, 128), (128, 64)], 2, list(class_rank), list(class_slots), B.LORA_BF16, 64, 16,
                        flags=B.LORA_CACHE_HOST_ONLY)
    rc, h = B.lora_cache_create(cfg, 0, 0)
    assert rc == B.LORA_OK
    return h


@pytest.mark.parametrize("weights,window", [((0.45, 0.10, 0.45), 0), ((0.0, 1.0, 0.0), 0), ((1 / 3, 1 / 3, 1 / 3), 0),
                                            ((0.45, 0.10, 0.45), 50)])
def test_library_manager_takes_the_oracles_decisions(weights, window):
    from paper_2411_17741_amd import binding as B

    class_rank, class_slots = [8, 32, 128], [4, 3, 3]
    h = _lib_cache(B, class_rank, class_slots)
    try:
        assert B.lora_cache_set_policy(h, *weights, window) == B.LORA_OK
        per_row = 2 * (64 + 128) * 2 * 2   # two projections of (h_in + h_out) bf16, two layers
        m = CacheManager(class_rank, class_slots, per_row, weights, window)
        rng = np.random.default_rng(11)
        running = collections.deque()
        for step in range(3000):
            a = int(rng.zipf(1.2)) % 80
            rank = [8, 16, 24, 64, 128][a % 5]
            queued = [int(q) for q in rng.integers(0, 80, size=int(rng.integers(0, 4)))]
            pin = bool(rng.integers(0, 4))
            want_slot, want_hit = m.acquire(a, rank, pin=pin, queued=queued)
            rc, slot, hit = B.lora_cache_acquire(h, a, rank, 1.0, pin, queued)
            if want_slot < 0:
                assert rc == B.LORA_E_NOMEM
            else:
                assert (rc, slot, bool(hit)) == (B.LORA_OK, want_slot, want_hit)
                if pin:
                    running.append(slot)
            while len(running) > 5:
                s = running.popleft()
                m.release(s)
                assert B.lora_cache_slot_ref(h, s, -1) == B.LORA_OK
            if step % 97 == 0:
                scores = m.scores()
                for i, e in enumerate(m.entries):
                    rc, v = B.lora_cache_score(h, i)
                    if e is None:
                        assert rc == B.LORA_E_STATE
                    else:
                        assert rc == B.LORA_OK and v == scores[i]      # the same doubles
                rc, v = B.lora_cache_choose_victim(h, 0, queued)
                want = m.victim(0, queued)
                assert (v if rc == B.LORA_OK else -1) == want
                assert B.lora_cache_resident_bytes(h) == (B.LORA_OK, m.resident_bytes())
            if step % 501 == 500:
                budget = m.resident_bytes() // 2
                want_n, want_ok = m.trim(budget, queued)
                rc, n = B.lora_cache_trim(h, budget, queued)
                assert n == want_n and (rc == B.LORA_OK) == want_ok
        rc, st = B.lora_cache_stats(h)
        assert (st.hits, st.misses, st.evictions) == (m.hits, m.misses, m.evictions)
        assert m.evictions > 100
    finally:
        B.lora_cache_destroy(h)


def test_library_manager_argument_checks_and_fill_after_a_miss():
    from paper_2411_17741_amd import binding as B

    h = _lib_cache(B, [8, 32], [1, 1])
    try:
        assert B.lora_cache_get_policy(h) == (B.LORA_OK, (0.45, 0.10, 0.45, 0))
        assert B.lora_cache_set_policy(h, -1.0, 0.0, 0.0) == B.LORA_E_INVAL
        assert B.lora_cache_set_policy(h, float("nan"), 0.0, 0.0) == B.LORA_E_INVAL
        assert B.lora_cache_acquire(h, 5, 64)[0] == B.LORA_E_INVAL        # above the largest class
        rc, slot, hit = B.lora_cache_acquire(h, 5, 8, 2.0)
        assert (rc, slot, hit) == (B.LORA_OK, 0, 0)
        rc, info = B.lora_cache_slot_info(h, 0)
        assert (info.state, info.adapter_id, info.rank, info.refcount, info.alpha) == (B.LORA_SLOT_FILLING, 5, 8, 1, 2.0)
        # the miss bound the slot: its parts are then loaded with the same (id, rank, alpha)
        for layer in range(2):
            for proj in range(2):
                assert B.lora_cache_fill_slot(h, 0, 5, 8, 2.0, layer, proj, 0, 0, 0) == B.LORA_OK
        assert B.lora_cache_slot_info(h, 0)[1].state == B.LORA_SLOT_READY
        assert B.lora_cache_fill_slot(h, 0, 6, 8, 2.0, 0, 0, 0, 0, 0) == B.LORA_E_STATE   # another adapter
        assert B.lora_cache_acquire(h, 5, 16)[0] == B.LORA_E_INVAL        # cached with another rank
        assert B.lora_cache_acquire(h, 5, 8) == (B.LORA_OK, 0, 1)
        assert B.lora_cache_slot_info(h, 0)[1].refcount == 2
        assert B.lora_cache_score(h, 1)[0] == B.LORA_E_STATE
        assert B.lora_cache_choose_victim(h, 0)[0] == B.LORA_E_NOMEM      # the only entry is in use
    finally:
        B.lora_cache_destroy(h)
