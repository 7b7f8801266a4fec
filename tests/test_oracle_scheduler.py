"""Pins of the scheduler oracle (oracle/scheduler.py) and parity of the library's scheduler with it.

Section 4.3 of the paper: weighted request size, size-ranged queues with token quotas, the
two-phase batch admission, number of queues and boundaries from K-means, least quota per queue.
All host-side: runs without a GPU."""
from __future__ import annotations

import itertools
import math

import numpy as np
import pytest

from oracle import scheduler as S


# ---- request size --------------------------------------------------------------------------------

def test_request_size_hand_worked():
    # (0.4 * 512/2048 + 0.6 * 256/1024) * 64/128 = (0.1 + 0.15) * 0.5
    assert S.wrs(512, 256, 64, 2048, 1024, 128) == pytest.approx(0.125, abs=1e-15)
    # the largest request in every respect has size A + B = 1
    assert S.wrs(2048, 1024, 128, 2048, 1024, 128) == pytest.approx(1.0, abs=1e-15)
    # output weighs 1.5 times the input; the rank scales the whole
    assert S.wrs(0, 1024, 128, 2048, 1024, 128) == pytest.approx(0.6, abs=1e-15)
    assert S.wrs(2048, 0, 128, 2048, 1024, 128) == pytest.approx(0.4, abs=1e-15)
    assert S.wrs(2048, 1024, 8, 2048, 1024, 128) == pytest.approx(1.0 / 16, abs=1e-15)


def test_queue_boundaries_are_inclusive_below():
    b = [0.1, 0.4]
    assert [S.queue_of(v, b) for v in (0.0, 0.0999, 0.1, 0.3, 0.4, 2.0)] == [0, 0, 1, 1, 2, 2]
    assert S.queue_of(0.7, []) == 0


# ---- batch admission: the two situations of the paper's scheduler figure ---------------------------

def _three_queues():
    # request size = 0.4 * input / 1000 (no output, full rank): small < 0.1 <= medium < 0.25 <= large
    return S.Scheduler([300, 600, 1000], [0.1, 0.25], 1000, 1000, 128, 0)


def test_batch_without_spare_tokens():
    s = _three_queues()
    for i in range(4):
        assert s.submit(10 + i, 100, 0, 1, 128) == 0       # small: 100 tokens each
    for i in range(2):
        assert s.submit(20 + i, 300, 0, 2, 128) == 1       # medium: 300 each
    for i in range(2):
        assert s.submit(30 + i, 700, 0, 3, 128) == 2       # large: 700 each
    # small admits three (the fourth does not fit its 300), medium both, large one; no queue ran
    # empty with tokens to spare except medium, which used its quota up: nothing to redistribute
    assert s.generate_batch() == [10, 11, 12, 20, 21, 30]
    assert s.free == [0, 0, 300]
    assert [len(q) for q in s.queues] == [1, 0, 1]


def test_batch_with_spare_tokens_redistributed_smallest_first():
    s = _three_queues()
    for i in range(4):
        s.submit(10 + i, 100, 0, 1, 128)
    assert s.submit(20, 250, 0, 2, 128) == 1                # medium has one request only
    for i in range(2):
        s.submit(30 + i, 700, 0, 3, 128)
    # phase 1: small 3, medium 1 (350 of its 600 unused, queue empty -> spare), large 1;
    # phase 2: the fourth small request takes 100 of the spare 350; the second large one needs 700: stays
    assert s.generate_batch() == [10, 11, 12, 20, 30, 13]
    assert s.free == [0, 250, 300]
    # the borrowed tokens go back to the queue they belong to
    s.finish(13)
    assert s.free == [0, 350, 300]
    s.finish(10)
    assert s.free == [100, 350, 300]
    assert s.waiting_adapters() == [3]


def test_first_request_that_does_not_fit_blocks_its_queue():
    s = S.Scheduler([500], [], 1000, 1000, 128, 2)
    s.submit(1, 100, 100, 7, 50)     # 100 + 100 + 50 * 2 = 300
    s.submit(2, 200, 100, 7, 8)      # 316: does not fit the 200 left
    s.submit(3, 10, 10, 7, 8)        # would fit, but arrival order is kept
    assert s.generate_batch() == [1]
    assert s.generate_batch() == []
    s.finish(1)
    assert s.generate_batch() == [2, 3]


def test_quotas_are_conserved_and_order_is_kept_on_a_random_trace():
    rng = np.random.default_rng(1)
    quotas = [4000, 8000, 12000, 16000]
    s = S.Scheduler(quotas, [0.02, 0.08, 0.3], 2048, 1024, 128, 4)
    running, arrival, rid = [], {}, 0
    for step in range(600):
        for _ in range(int(rng.integers(0, 6))):
            q = s.submit(rid, int(rng.integers(1, 2048)), int(rng.integers(1, 1024)), int(rng.integers(0, 50)),
                         int(rng.choice([8, 16, 32, 64, 128])))
            arrival[rid] = (q, rid)
            rid += 1
        heads = [q[0].req_id if q else None for q in s.queues]
        batch = s.generate_batch()
        # arrival order within every queue: the admitted requests of a queue are a prefix of it, in order
        for q in range(4):
            mine = [r for r in batch if arrival[r][0] == q]
            assert mine == sorted(mine)
            if mine:
                assert min(mine) == heads[q]
        running += batch
        lent = [0] * 4
        for r in s.running.values():
            assert sum(t for _, t in r.borrowed) == s.needed(r)
            for q, t in r.borrowed:
                lent[q] += t
        assert [f + l for f, l in zip(s.free, lent)] == quotas and min(s.free) >= 0
        for _ in range(int(rng.integers(0, 5))):
            if running:
                s.finish(running.pop(int(rng.integers(0, len(running)))))
    assert rid > 1000 and len(s.running) == len(running)


# ---- number of queues, boundaries --------------------------------------------------------------

def _brute_force_wcss(values, k):
    """Smallest within-cluster sum of squares over every assignment of the values to k labels."""
    best = math.inf
    for labels in itertools.product(range(k), repeat=len(values)):
        if len(set(labels)) != k:
            continue
        total = 0.0
        for c in range(k):
            group = [v for v, l in zip(values, labels) if l == c]
            mean = sum(group) / len(group)
            total += sum((v - mean) ** 2 for v in group)
        best = min(best, total)
    return best


def test_clustering_is_the_k_means_optimum():
    rng = np.random.default_rng(2)
    for trial in range(6):
        values = [float(v) for v in rng.random(7) ** 2]
        for k in (1, 2, 3, 4):
            got, centroids = S.kmeans_1d(values, k)
            assert got == pytest.approx(_brute_force_wcss(values, k), rel=1e-9, abs=1e-15)
            assert centroids == sorted(centroids) and len(centroids) == k
    # all values alike: one queue, whatever k_max is
    assert S.fit_queues([0.5] * 10, 4) == (1, [])


def test_boundaries_are_midpoints_between_centroids():
    sizes = [0.01, 0.012, 0.011, 0.2, 0.21, 0.22, 0.8, 0.85]
    k, bounds = S.fit_queues(sizes, 4)
    assert k == 3
    c = [(0.01 + 0.012 + 0.011) / 3, (0.2 + 0.21 + 0.22) / 3, (0.8 + 0.85) / 2]
    assert bounds == pytest.approx([(c[0] + c[1]) / 2, (c[1] + c[2]) / 2], rel=1e-12)
    # two well separated groups
    k, bounds = S.fit_queues([1.0, 1.1, 0.9, 5.0, 5.2, 4.8], 4)
    assert k == 2 and bounds == pytest.approx([3.0], rel=1e-12)


# ---- quotas --------------------------------------------------------------------------------------

def test_least_quota_meets_the_slo_exactly_in_the_queueing_model():
    S_max, D, slo, lam = 4096.0, 2.0, 5.0, 0.5
    tok = S.min_quota(S_max, D, slo, lam)
    assert tok == 5735                                      # 4096 * 2 * (1/5 + 1/2) = 5734.4, rounded up
    # M/M/1: service rate mu = tokens / (S * D); time in system 1 / (mu - lambda) <= SLO, and one
    # token less would break it
    assert 1.0 / (tok / (S_max * D) - lam) <= slo
    assert 1.0 / ((tok - 1) / (S_max * D) - lam) > slo


def test_quota_assignment():
    assert S.assign_quotas(100000, [1000, 2000, 3000], [1, 1, 2]) == [24500, 25500, 50000]
    assert S.assign_quotas(5999, [1000, 2000, 3000], [1, 1, 2]) is None
    q = S.assign_quotas(6010, [1000, 2000, 3000], [1, 1, 1])     # 10 left: 3 each, the odd token to queue 0
    assert q == [1004, 2003, 3003] and sum(q) == 6010


# ---- the library against the oracle --------------------------------------------------------------

def test_library_scheduler_takes_the_oracles_decisions():
    from paper_2411_17741_amd import binding as B

    rng = np.random.default_rng(4)
    quotas, bounds = [3000, 6000, 9000, 20000], [0.015, 0.07, 0.25]
    rc, h = B.lora_sched_create(quotas, bounds, 2048, 1024, 128, 4)
    assert rc == B.LORA_OK
    try:
        s = S.Scheduler(quotas, bounds, 2048, 1024, 128, 4)
        running, rid = [], 0
        for step in range(800):
            for _ in range(int(rng.integers(0, 7))):
                args = (rid, int(rng.integers(0, 2049)), int(rng.integers(0, 1025)), int(rng.integers(0, 50)),
                        int(rng.choice([8, 16, 32, 64, 128])))
                assert B.lora_sched_submit(h, *args) == (B.LORA_OK, s.submit(*args))
                assert B.lora_sched_wrs(args[1], args[2], args[4], 2048, 1024, 128) == S.wrs(args[1], args[2], args[4], 2048, 1024, 128)
                rid += 1
            want = s.generate_batch()
            assert B.lora_sched_generate_batch(h) == (B.LORA_OK, want)
            running += want
            for q in range(4):
                assert B.lora_sched_queue_state(h, q) == (B.LORA_OK, s.free[q], len(s.queues[q]))
            if step % 50 == 0:
                assert B.lora_sched_waiting_adapters(h) == (B.LORA_OK, s.waiting_adapters())
            for _ in range(int(rng.integers(0, 6))):
                if running:
                    r = running.pop(int(rng.integers(0, len(running))))
                    s.finish(r)
                    assert B.lora_sched_finish(h, r) == B.LORA_OK
        assert rid > 2000
        assert B.lora_sched_finish(h, -5) == B.LORA_E_NOTFOUND
        if running:
            assert B.lora_sched_submit(h, running[0], 1, 1, 1, 8)[0] == B.LORA_E_INVAL   # the id is still running
    finally:
        B.lora_sched_destroy(h)


def test_library_batch_capacity_and_argument_checks():
    from paper_2411_17741_amd import binding as B

    rc, h = B.lora_sched_create([1000], [], 100, 100, 128, 0)
    assert rc == B.LORA_OK
    try:
        for i in range(5):
            assert B.lora_sched_submit(h, i, 10, 10, 1, 8) == (B.LORA_OK, 0)
        assert B.lora_sched_submit(h, 0, 10, 10, 1, 8)[0] == B.LORA_E_INVAL      # already waiting
        assert B.lora_sched_submit(h, 9, -1, 10, 1, 8)[0] == B.LORA_E_INVAL
        assert B.lora_sched_submit(h, 9, 1, 10, 1, 0)[0] == B.LORA_E_INVAL
        assert B.lora_sched_generate_batch(h, cap=2) == (B.LORA_OK, [0, 1])      # the rest stays queued
        assert B.lora_sched_queue_state(h, 0) == (B.LORA_OK, 960, 3)
        assert B.lora_sched_generate_batch(h) == (B.LORA_OK, [2, 3, 4])
        assert B.lora_sched_queue_state(h, 1)[0] == B.LORA_E_INVAL
    finally:
        B.lora_sched_destroy(h)
    assert B.lora_sched_create([100, 100], [0.5, 0.1][:1], 0, 100, 128, 0)[0] == B.LORA_E_INVAL   # max_input < 1
    assert B.lora_sched_create([100, 100, 100], [0.5, 0.1], 100, 100, 128, 0)[0] == B.LORA_E_INVAL  # descending
    assert B.lora_sched_create([-1], [], 100, 100, 128, 0)[0] == B.LORA_E_INVAL
    assert math.isnan(B.lora_sched_wrs(1, 1, 1, 0, 1, 1))


def test_library_queue_fit_and_quotas_match_the_oracle():
    from paper_2411_17741_amd import binding as B

    rng = np.random.default_rng(6)
    for trial in range(20):
        n = int(rng.integers(1, 300))
        centres = rng.random(int(rng.integers(1, 5)))
        sizes = [float(abs(centres[int(rng.integers(0, len(centres)))] + 0.02 * rng.standard_normal())) for _ in range(n)]
        k, bounds = S.fit_queues(sizes, 4)
        rc, k2, bounds2 = B.lora_sched_fit_queues(sizes, 4)
        assert rc == B.LORA_OK and k2 == k
        assert bounds2 == pytest.approx(bounds, rel=1e-9, abs=1e-12)
    assert B.lora_sched_fit_queues([0.5] * 10, 4) == (B.LORA_OK, 1, [])
    assert B.lora_sched_fit_queues([], 4)[0] == B.LORA_E_INVAL
    for args in ((4096.0, 2.0, 5.0, 0.5), (100.0, 0.3, 1.0, 12.0), (1.0, 1.0, 1.0, 0.0)):
        assert B.lora_sched_min_quota(*args) == S.min_quota(*args)
    assert B.lora_sched_min_quota(0.0, 1.0, 1.0, 1.0) == -1
    for total, least, w in ((100000, [1000, 2000, 3000], [1, 1, 2]), (6010, [1000, 2000, 3000], [1, 1, 1]), (7, [0, 0], [0.3, 0.7])):
        assert B.lora_sched_assign_quotas(total, least, w) == (B.LORA_OK, S.assign_quotas(total, least, w))
    assert B.lora_sched_assign_quotas(5999, [1000, 2000, 3000], [1, 1, 2])[0] == B.LORA_E_NOMEM
