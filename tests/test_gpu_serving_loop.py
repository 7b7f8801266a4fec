"""The pieces together on the GPU: the scheduler (section 4.3) forms the batch of every iteration, the
cache manager (section 4.2) finds or loads the adapters of the admitted requests -- evicting by score
when the pool is full --, and the batch (prompts of the new requests, one token of every other
running request) goes through lora_apply; every iteration's output is checked against the fp64
oracle with the adapters the requests name."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from oracle import manager as OM
from oracle import scheduler as OS

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = {"rel_fro": 1e-2, "max_abs_over_rms": 2e-2, "delta_rel_fro": 2e-2}


def _bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def test_scheduler_cache_manager_and_apply_over_iterations():
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H
    from paper_2411_17741_amd.pool import LoraPool

    rng = np.random.default_rng(12)
    h_in, h_out, scale = 256, 384, 2.0
    class_rank, class_slots = [8, 32, 128], [2, 2, 2]            # six slots for twenty adapters
    n_adapters = 20
    ranks = rng.choice([8, 16, 32, 64, 128], size=n_adapters)
    weights = {a: (_bf16(rng.normal(0, 0.05, (h_in, ranks[a]))), _bf16(rng.normal(0, 0.05, (ranks[a], h_out))), 1.0 + 0.25 * (a % 3))
               for a in range(n_adapters)}
    pool = LoraPool([(h_in, h_out)], 1, class_rank, class_slots, B.LORA_BF16, max_tokens=4096, max_segments=256)
    quotas, bounds = [600, 1200, 2400], [0.01, 0.05]
    rc, sched = B.lora_sched_create(quotas, bounds, 256, 8, 128, 1)
    assert rc == B.LORA_OK
    o_sched = OS.Scheduler(quotas, bounds, 256, 8, 128, 1)
    o_cache = OM.CacheManager(class_rank, class_slots, (h_in + h_out) * 2)
    try:
        running = {}     # req id -> [adapter, slot, tokens still to produce, prompt length if not yet run]
        rid = refused = checked = 0
        for it in range(14):
            for _ in range(int(rng.poisson(3.0))):
                a = int(min(n_adapters - 1, rng.zipf(1.3) - 1))
                args = (rid, int(rng.integers(4, 200)), int(rng.integers(1, 7)), a + 100, int(ranks[a]))
                assert B.lora_sched_submit(sched, *args) == (B.LORA_OK, o_sched.submit(*args))
                rid += 1
            rc, batch = B.lora_sched_generate_batch(sched)
            assert (rc, batch) == (B.LORA_OK, o_sched.generate_batch())
            rc, queued = B.lora_sched_waiting_adapters(sched)
            assert (rc, queued) == (B.LORA_OK, o_sched.waiting_adapters())
            for r in batch:
                req = o_sched.running[r]
                a = req.adapter_id - 100
                want_slot, want_hit = o_cache.acquire(req.adapter_id, req.rank, True, queued)
                rc, slot, hit = B.lora_cache_acquire(pool.handle, req.adapter_id, req.rank, weights[a][2], True, queued)
                if want_slot < 0:
                    # every slot that fits is held by a running request: the request is squashed and gives its tokens back
                    assert rc == B.LORA_E_NOMEM
                    o_sched.finish(r)
                    assert B.lora_sched_finish(sched, r) == B.LORA_OK
                    refused += 1
                    continue
                assert (rc, slot, bool(hit)) == (B.LORA_OK, want_slot, want_hit)
                if not hit:
                    pool.fill(slot, req.adapter_id, req.rank, weights[a][2], 0, 0, weights[a][0], weights[a][1])
                running[r] = [a, slot, req.output_len, req.input_len]
            if not running:
                continue
            # this iteration's batch: the prompt of a request that has not run yet, else one token
            seg_len = [st[3] if st[3] else 1 for st in running.values()]
            seg_off = np.concatenate([[0], np.cumsum(seg_len)]).astype(np.int32)
            seg_slot = np.asarray([st[1] for st in running.values()], np.int32)
            seg_adapter = np.asarray([st[0] for st in running.values()], np.int32)
            seg_rank = ranks[seg_adapter].astype(np.int32)
            T = int(seg_off[-1])
            x, base = _bf16(rng.normal(0, 1, (T, h_in))), _bf16(rng.normal(0, 1, (T, h_out)))
            xd, yd = H.to_device(x, B.LORA_BF16), H.to_device(base, B.LORA_BF16)
            pool.apply(0, 0, xd, yd, seg_off, seg_slot, seg_rank, scale)
            pool.check_fault()
            pool.fills_done()
            ref = oracle.lora_apply(x, base, seg_off, seg_adapter, {a: weights[a] for a in set(seg_adapter.tolist())}, scale)
            m = H.error_metrics(yd.float().cpu().numpy(), ref, base)
            for k, lim in TOL.items():
                assert m[k] <= lim, f"iteration {it}: {k} = {m[k]:.3e} > {lim}"
            checked += 1
            for r in list(running):
                st = running[r]
                st[3] = 0
                st[2] -= 1
                if st[2] == 0:
                    o_sched.finish(r)
                    o_cache.release(st[1])
                    assert B.lora_sched_finish(sched, r) == B.LORA_OK
                    assert B.lora_cache_slot_ref(pool.handle, st[1], -1) == B.LORA_OK
                    del running[r]
        rc, stats = B.lora_cache_stats(pool.handle)
        assert (stats.hits, stats.misses, stats.evictions) == (o_cache.hits, o_cache.misses, o_cache.evictions)
        assert checked >= 10 and stats.misses > 6 and stats.evictions > 0 and stats.hits > 0
    finally:
        B.lora_sched_destroy(sched)
        pool.close()
