"""CPU ORACLE (test infrastructure, not part of the product): the adapter cache manager.

Plain-Python restatement of the cache management of paper section 4.2, kept
free of anything the GPU library uses.  Only `tests/` imports it.

What the paper fixes:

* every cache entry carries: adapter id, rank, last-used time, usage frequency
  within a time frame, and a reference counter of the running requests that
  use it;
* an entry whose reference counter is not zero is never evicted;
* entries of requests that wait in the queues are kept as long as memory
  allows: they are considered for eviction only when nothing else is left;
* the eviction score is  F * frequency + R * recency + S * size  with
  F, R, S = 0.45, 0.10, 0.45; the entry with the lowest score goes first;
  larger adapters cost more to reload, so size raises the score;
* the cache is resized on demand: entries are evicted, in score order, until
  what the rest of the system needs is free;
* waiting requests may have their adapters prefetched.

What it leaves open, and the reading taken (the library takes the same one,
stated in its header): the three terms have no units in the paper, so each is
scaled to [0, 1] over the cached entries -- frequency divided by the largest
cached frequency, recency = 1 - age / largest age with age counted in requests
since the entry's last use, size = rank / largest cached rank.  "Within a time
frame": all frequencies are halved every `freq_window` requests (0: never).
Ties go to the lower slot.

The pool is the library's: slots grouped in rank classes, an adapter goes to a
free slot of the smallest class that holds its rank, and only entries in slots
that are large enough can make room for it.

Pins (tests/test_oracle_manager.py): a hand-worked score table with the
paper's coefficients; with weights (0, 1, 0) the victims are those of a
textbook LRU list; with (1, 0, 0) the victim has the lowest use count, with
(0, 0, 1) the lowest rank; reference counters and queued adapters are honoured
on random traces; trimming stops exactly when the budget is met.
"""
from __future__ import annotations

import math
from typing import Dict, Iterable, List, Optional, Sequence, Tuple


class Entry:
    __slots__ = ("adapter_id", "rank", "freq", "last", "refcount")

    def __init__(self, adapter_id: int, rank: int):
        self.adapter_id = adapter_id
        self.rank = rank
        self.freq = 0.0
        self.last = 0
        self.refcount = 0


class CacheManager:
    """Slots are numbered class by class in the order of `class_rank` (ascending)."""

    def __init__(self, class_rank: Sequence[int], class_slots: Sequence[int], bytes_per_rank_row: int,
                 weights: Tuple[float, float, float] = (0.45, 0.10, 0.45), freq_window: int = 0):
        self.slot_class_rank: List[int] = []
        for r, n in zip(class_rank, class_slots):
            self.slot_class_rank += [int(r)] * int(n)
        self.entries: List[Optional[Entry]] = [None] * len(self.slot_class_rank)
        self.where: Dict[int, int] = {}
        self.bytes_per_rank_row = int(bytes_per_rank_row)  # pool bytes of one storage row over all layers and projections
        self.w_freq, self.w_recency, self.w_size = weights
        self.freq_window = int(freq_window)
        self.now = 0
        self.hits = self.misses = self.evictions = 0

    # -- the score -------------------------------------------------------------------------
    def scores(self) -> List[float]:
        cached = [e for e in self.entries if e is not None]
        out = [math.inf] * len(self.entries)
        if not cached:
            return out
        max_f = max(e.freq for e in cached)
        max_age = max(self.now - e.last for e in cached)
        max_rank = max(e.rank for e in cached)
        for i, e in enumerate(self.entries):
            if e is None:
                continue
            frequency = e.freq / max_f if max_f > 0 else 0.0
            recency = 1.0 - (self.now - e.last) / max_age if max_age > 0 else 1.0
            size = e.rank / max_rank
            out[i] = self.w_freq * frequency + self.w_recency * recency + self.w_size * size
        return out

    def victim(self, rank: int = 0, queued: Iterable[int] = ()) -> int:
        """Slot whose entry goes next to make room for an adapter of `rank`; -1 if none may go."""
        queued = set(queued)
        score = self.scores()
        for spare_queued in (True, False):
            best = -1
            for i, e in enumerate(self.entries):
                if e is None or e.refcount > 0 or self.slot_class_rank[i] < rank:
                    continue
                if spare_queued and e.adapter_id in queued:
                    continue
                if best < 0 or score[i] < score[best]:
                    best = i
            if best >= 0:
                return best
        return -1

    # -- requests --------------------------------------------------------------------------
    def _free_slot(self, rank: int) -> int:
        for i, e in enumerate(self.entries):  # slots ascend by class, so the first fit is the smallest class
            if e is None and self.slot_class_rank[i] >= rank:
                return i
        return -1

    def _touch(self, e: Entry, pin: bool) -> None:
        self.now += 1
        if self.freq_window > 0 and self.now % self.freq_window == 0:
            for o in self.entries:
                if o is not None:
                    o.freq *= 0.5
        e.freq += 1.0
        e.last = self.now
        if pin:
            e.refcount += 1

    def acquire(self, adapter_id: int, rank: int, pin: bool = True, queued: Iterable[int] = ()) -> Tuple[int, bool]:
        """-> (slot, hit); slot = -1 if every large-enough entry is in use."""
        if adapter_id in self.where:
            slot = self.where[adapter_id]
            self.hits += 1
            self._touch(self.entries[slot], pin)
            return slot, True
        slot = self._free_slot(rank)
        if slot < 0:
            slot = self.victim(rank, queued)
            if slot < 0:
                return -1, False
            self._drop(slot)
        self.misses += 1
        e = Entry(adapter_id, rank)
        self.entries[slot] = e
        self.where[adapter_id] = slot
        self._touch(e, pin)
        return slot, False

    def release(self, slot: int) -> None:
        e = self.entries[slot]
        assert e is not None and e.refcount > 0
        e.refcount -= 1

    def _drop(self, slot: int) -> None:
        e = self.entries[slot]
        del self.where[e.adapter_id]
        self.entries[slot] = None
        self.evictions += 1

    # -- sizing ----------------------------------------------------------------------------
    @staticmethod
    def _storage_rows(rank: int) -> int:
        return (rank + 7) // 8 * 8

    def resident_bytes(self) -> int:
        return sum(self._storage_rows(e.rank) * self.bytes_per_rank_row for e in self.entries if e is not None)

    def trim(self, max_bytes: int, queued: Iterable[int] = ()) -> Tuple[int, bool]:
        """Evict in score order until at most max_bytes are held -> (entries evicted, budget met)."""
        n = 0
        while self.resident_bytes() > max_bytes:
            slot = self.victim(0, queued)
            if slot < 0:
                return n, False
            self._drop(slot)
            n += 1
        return n, True
