#!/usr/bin/env python3
"""Benchmark of the batched heterogeneous-rank LoRA apply on one MI355X.

A step = one pass of the whole hot path over one batch, the way a serving iteration runs
it: index the batch once (host), upload its work lists, then run shrink + expand for every
projection of every layer copy the pool holds, reading the adapters from the cache pool.
The layer copies are distinct memory and the activations rotate over several buffer sets, so
that slabs and activations come from HBM and not from the 256 MB Infinity Cache.  Inputs are
resident in HBM before the timed region starts.  value = tokens x layers / time: the rate at
which tokens pass one layer's LoRA apply.

Prints ONE JSON line: tokens/s per layer, the roofline figure of the dominant kernel (HIP
events around each kernel, in a second pass of the same steps) and the CPU oracle's rate on a
bounded sample of the same workload.

    python bench.py [--workload decode|prefill|mixed|stress] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E
WORKLOAD_TEXT = {
    "decode": "decode: 64 one-token requests, one 4096->4096 bf16 projection, pool of 100 adapters (ranks 8..128), Zipf(1.0)",
    "prefill": "prefill: 8 prompts lognormal(6,0.8) in [32,2048], one 4096->4096 bf16 projection, distinct adapters of rank 16/64/128",
    "mixed": "mixed: 224 decode + 32 prompts, 7B-shaped layer (q,k,v,o,gate,up,down) bf16, pool of 500, Zipf(1.2)",
    "stress": "stress: 512 decode + 4x512 prompt tokens, 13B-shaped layer bf16, pool of 1000 in 4 layer copies, Zipf(1.2)",
    "decode_heavy": "decode_heavy (extra, not one of the task's configurations): 1024 one-token requests, one 4096->4096 bf16 projection, pool of 500 adapters (ranks 8..128), Zipf(1.0)",
    "decode_qkv": "decode_qkv (extra): the decode configuration's batch on the projections q, k, v (4096->4096 bf16 each, same activations), applied as one group",
    "decode_paper": "decode_paper (extra): one-token requests, one 4096->4096 bf16 projection, the paper's adapter population: --adapters N_a, N_a/5 of each rank 8..128, rank uniform, power law within the rank",
}
# HBM bytes per launch (average over a layer's launches of that kernel) from rocprofv3 counter runs of this same
# script (FETCH_SIZE and WRITE_SIZE, each in a run of its own, scaled by what the same counters read for a plain
# 256 MiB copy).  A counter run cannot happen inside this process, so the figures measured for the same workloads
# are carried here; the line names their source, and they are left out when the flags change what is launched.
TRAFFIC_SOURCE = "profiles/kernel_traffic_all_workloads.txt"
MEASURED_TRAFFIC = {("decode", "gemv_fused"): 24.74e6, ("decode_qkv", "gemv_fused"): 71.81e6, ("prefill", "mfma_shrink"): 66.64e6,
                    ("prefill", "mfma_expand"): 121.58e6, ("mixed", "mfma_expand"): 558.77e6, ("mixed", "mfma_shrink"): 404.12e6,
                    ("mixed", "gemv_fused"): 177.94e6, ("stress", "gemv_fused"): 356.77e6, ("stress", "mfma_expand"): 103.75e6,
                    ("stress", "mfma_shrink"): 73.25e6}
DEFAULT_LAYERS = {"decode": 32, "prefill": 8, "mixed": 2, "stress": 4, "decode_heavy": 8, "decode_paper": 32, "decode_qkv": 16}
DEFAULT_STEPS = {"decode": 100, "prefill": 60, "mixed": 20, "stress": 20, "decode_heavy": 40, "decode_paper": 100, "decode_qkv": 100}


def algorithmic_bytes(inst, w, esize=2):
    """Bytes each kernel kind must move per projection: every distinct slab it needs once at its
    true rank, its tokens' x rows once, its tokens' base_out rows read and written once.  The
    T x rank intermediate is not counted.  Consecutive projections that read the same x share one
    tile-shrink launch (as lora_apply_plan_multi groups them, up to 4): x counts once per group."""
    tok_n = lambda items: sum(it[1] for it in items)
    slabs = lambda items: {it[2]: it[3] for it in items}
    out = []
    group_len = 0
    for i, pr in enumerate(inst.projs):
        first_of_group = i == 0 or inst.projs[i - 1].x_key != pr.x_key or group_len == 4
        group_len = 1 if first_of_group else group_len + 1
        g, t = slabs(w["groups"]), slabs(w["tiles"])
        ng, nt = tok_n(w["groups"]), tok_n(w["tiles"])
        out.append({
            "gemv_shrink": esize * (sum(g.values()) * pr.h_in + ng * pr.h_in),
            "gemv_expand": esize * (sum(g.values()) * pr.h_out + 2 * ng * pr.h_out),
            "mfma_shrink": esize * (sum(t.values()) * pr.h_in + (nt * pr.h_in if first_of_group else 0)),
            "mfma_expand": esize * (sum(t.values()) * pr.h_out + 2 * nt * pr.h_out),
            "mfma_reduce": 0,
        })
        out[-1]["gemv_fused"] = out[-1]["gemv_shrink"] + out[-1]["gemv_expand"]
    return out


MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def fused_base(args, inst, pi, xs, ys, n_layers, n_sets, steps, stream) -> dict:
    """y = x.W + s.(x.A).B in one pass per projection (lora_linear_plan), next to the same work done as a
    vendor-library matmul followed by the apply on its output."""
    import torch
    from paper_2411_17741_amd import binding as B

    h, sh, dev = pi.pool.handle, stream.cuda_stream, xs[0][inst.projs[0].x_key].device
    n_proj = len(inst.projs)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4321)
    wts = [[(torch.randn((p.h_out, p.h_in), generator=gen, device=dev) * 0.02).to(torch.bfloat16) for p in inst.projs] for _ in range(2)]

    ws = torch.empty((inst.T * max(p.h_out for p in inst.projs),), dtype=torch.float32, device=dev)  # fp32 adapter term of the GEMV tokens

    def step(s: int, fused: bool) -> None:
        rc, plan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, sh)
        B.check(rc, "lora_plan_create")
        for l in range(n_layers):
            for p in range(n_proj):
                x, y, wt = xs[l % n_sets][inst.projs[p].x_key], ys[l % n_sets][p], wts[(s + l) % 2][p]
                if fused:
                    B.check(B.lora_linear_plan(h, plan, l, p, x.data_ptr(), wt.data_ptr(), y.data_ptr(), inst.scale, sh,
                                               workspace=ws.data_ptr(), workspace_bytes=ws.numel() * 4), "lora_linear_plan")
                else:
                    torch.matmul(x, wt.t(), out=y)
                    B.check(B.lora_apply_plan(h, plan, l, p, x.data_ptr(), y.data_ptr(), inst.scale, sh), "lora_apply_plan")
        B.check(B.lora_plan_destroy(h, plan))

    def timed(fused: bool) -> float:
        for s in range(args.warmup):
            step(s, fused)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            step(args.warmup + s, fused)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_fused, ms_split = timed(True), timed(False)
    B.check(B.lora_cache_set_timing(h, 1))
    n_t = max(1, min(steps, 40 // n_layers))
    for s in range(n_t):
        step(args.warmup + s, True)
    torch.cuda.synchronize()
    rc, tm = B.lora_cache_read_timing(h)
    B.check(rc)
    B.check(B.lora_cache_set_timing(h, 0))
    kernels = {k: {"launches": int(n), "avg_us": ms * 1e3 / n} for k, (ms, n) in tm.items() if n}
    flops_layer = sum(2.0 * inst.T * p.h_in * p.h_out for p in inst.projs)
    lin = kernels["linear"]
    achieved = flops_layer / n_proj / (lin["avg_us"] * 1e-6) / 1e12  # average launch: one projection
    out = {
        "metric": "lora_linear_tokens_per_s_per_layer", "value": inst.T / (ms_fused / n_layers * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": args.warmup, "ms_per_step": ms_fused, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT.get(inst.name, inst.name) + "; base projection fused (lora_linear_plan), random base weights",
                   "tokens": inst.T, "projections": n_proj, "layers_per_step": n_layers, "ms_per_layer": ms_fused / n_layers,
                   "vendor_matmul_then_apply_ms_per_layer": ms_split / n_layers},
        "roofline": {"bound": "mfma", "kernel": "linear", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_PEAK_TFLOPS, "traffic": None, "avg_launch_us": lin["avg_us"],
                     "flops_per_launch": flops_layer / n_proj},
        "cpu_baseline": None,
        "kernels": kernels,
    }
    return out


def prefetch_sweep(args) -> int:
    """Queue-driven prefetch (paper section 4.2: the adapters of waiting requests are loaded before their
    batch runs) measured as fill/apply overlap on the host link.  A stream of decode batches over the
    paper's adapter population (N_a/5 adapters per rank, rank uniform, power law within the rank) runs
    against a pool that holds only part of the adapters.  Iteration k acquires the adapters of its batch
    (pinned; a miss is loaded from pinned host memory on a side stream, and the apply waits for it), then
    -- at depth d > 0 -- acquires unpinned and loads what batch k+d will need, and applies.  Prints one
    JSON line: time per iteration, demand misses and bytes loaded for every depth."""
    import torch
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd.pool import LoraPool

    depths = [int(d) for d in args.prefetch_depths.split(",")]
    n_tok, n_a, n_layers = args.tokens if args.tokens != 64 else 256, args.adapters if args.adapters != 100 else 200, args.layers or 8
    ranks = [8, 16, 32, 64, 128]
    per_rank = n_a // 5
    slots_per_rank = args.slots_per_rank or per_rank - max(2, per_rank // 13)
    projs = [(4096, 4096)] * 4
    steps, warmup = args.steps or 40, max(args.warmup, 8)
    n_iter = warmup + steps + max(depths) + 1
    rng = np.random.default_rng(7)
    # the request stream: per token a rank class, then an adapter of that rank by a power law (exponent 1.2: the paper states none)
    w = 1.0 / np.arange(1, per_rank + 1) ** 1.2
    cdf = np.cumsum(w / w.sum())
    perm = [rng.permutation(per_rank) for _ in ranks]
    batches = []
    for _ in range(n_iter):
        cls = rng.integers(0, 5, size=n_tok)
        pos = np.minimum(np.searchsorted(cdf, rng.random(n_tok)), per_rank - 1)
        batches.append(np.asarray([c * per_rank + perm[c][k] for c, k in zip(cls, pos)], np.int64))
    need = [np.unique(b) for b in batches]
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    # every part of every adapter has host memory of its own in one pinned arena (what is loaded does not matter
    # here, where from does: parts that shared host memory would be served from the GPU's caches, not over the link)
    part_bytes = {r: 2 * 4096 * r * 2 for r in ranks}  # A [4096][r] + B [r][4096], bf16
    adapter_bytes = [n_layers * 4 * part_bytes[ranks[a // per_rank]] for a in range(n_a)]
    arena = torch.empty(sum(adapter_bytes), dtype=torch.uint8, pin_memory=True)
    arena.view(torch.int16)[:] = 0x3c00  # a small bf16 number everywhere
    parts_of, off = [], arena.data_ptr()
    for a in range(n_a):
        r = ranks[a // per_rank]
        entries = []
        for l in range(n_layers):
            for p in range(4):
                entries.append((l, p, off, off + part_bytes[r] // 2))
                off += part_bytes[r]
        parts_of.append(entries)
    parts_c = [B.make_fill_parts(e) for e in parts_of]
    x = torch.randn((n_tok, 4096), generator=gen, device=dev).to(torch.bfloat16)
    ys = [torch.randn((n_tok, 4096), generator=gen, device=dev).to(torch.bfloat16) for _ in range(n_layers * 4)]
    seg_offsets = np.arange(n_tok + 1, dtype=np.int32)
    stream, side = torch.cuda.current_stream(), torch.cuda.Stream()
    sh = stream.cuda_stream
    out = {}
    for d in depths:
        pool = LoraPool(projs, n_layers, ranks, [slots_per_rank] * 5, B.LORA_BF16, max_tokens=n_tok, max_segments=n_tok + 8, n_plans=4,
                        flags=B.LORA_CACHE_DIRECT_FILL if args.direct_fill else 0)
        h = pool.handle
        B.check(B.lora_cache_set_fencing(h, 1))
        descs = B.make_descs([(l, p, x.data_ptr(), ys[l * 4 + p].data_ptr()) for l in range(n_layers) for p in range(4)])
        counts = {"demand_miss": 0, "demand_hit": 0, "prefetched": 0, "refused": 0, "bytes": 0, "t_fill": 0.0}

        def load(a, slot):
            r = ranks[a // per_rank]
            t_f = time.perf_counter()
            if args.fill_by_part:
                for l, p, pa, pb in parts_of[a]:
                    B.check(B.lora_cache_fill_slot(h, slot, 1000 + a, r, 1.0, l, p, pa, pb, side.cuda_stream), "fill")
            else:
                B.check(B.lora_cache_fill_slot_parts(h, slot, 1000 + a, r, 1.0, parts_c[a], side.cuda_stream), "fill")
            counts["t_fill"] += time.perf_counter() - t_f
            counts["bytes"] += adapter_bytes[a]

        def iteration(k):
            queued = np.concatenate(need[k + 1:k + 1 + d]) + 1000 if d else None
            slot_of = {}
            for a in need[k]:
                a = int(a)
                rc, slot, hit = B.lora_cache_acquire(h, 1000 + a, ranks[a // per_rank], 1.0, True, queued)
                if rc == B.LORA_E_NOMEM:  # every slot of the class is held by this batch: the request runs without its adapter
                    counts["refused"] += 1
                    slot_of[a] = -1
                    continue
                B.check(rc, "acquire")
                slot_of[a] = slot
                counts["demand_hit" if hit else "demand_miss"] += 1
                if not hit:
                    load(a, slot)
            if d:
                for a in need[k + d]:
                    a = int(a)
                    rc, slot, hit = B.lora_cache_acquire(h, 1000 + a, ranks[a // per_rank], 1.0, False, queued)
                    if rc != B.LORA_E_NOMEM:  # no slot to spare: the adapter will be a demand miss
                        B.check(rc, "acquire")
                    if rc == B.LORA_OK and not hit:
                        counts["prefetched"] += 1
                        load(a, slot)
            seg_slot = np.asarray([slot_of[int(a)] for a in batches[k]], np.int32)
            seg_rank = np.asarray([ranks[int(a) // per_rank] for a in batches[k]], np.int32)
            rc, plan = B.lora_plan_create(h, n_tok, seg_offsets, seg_slot, seg_rank, sh)
            B.check(rc, "lora_plan_create")
            B.check(B.lora_apply_plan_multi(h, plan, descs, 2.0, sh), "lora_apply_plan_multi")
            B.check(B.lora_plan_destroy(h, plan))
            for a, slot in slot_of.items():
                if slot >= 0:
                    B.check(B.lora_cache_slot_ref(h, slot, -1))

        for k in range(warmup):
            iteration(k)
        torch.cuda.synchronize()
        for key in counts:
            counts[key] = 0
        t0 = time.perf_counter()
        for k in range(warmup, warmup + steps):
            iteration(k)
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        t_all = time.perf_counter() - t0
        pool.check_fault()
        out[str(d)] = {"ms_per_iteration": t_all * 1e3 / steps, "host_enqueue_ms_per_iteration": t_host * 1e3 / steps,
                       "host_ms_in_fill_calls_per_iteration": counts["t_fill"] * 1e3 / steps,
                       "demand_misses_per_iteration": counts["demand_miss"] / steps, "demand_hit_rate": counts["demand_hit"] / max(1, counts["demand_hit"] + counts["demand_miss"]),
                       "prefetched_per_iteration": counts["prefetched"] / steps, "refused_per_iteration": counts["refused"] / steps,
                       "loaded_MB_per_iteration": counts["bytes"] / steps / 1e6,
                       "host_link_GBs": counts["bytes"] / t_all / 1e9}
        pool.close()
    best = min(out.values(), key=lambda r: r["ms_per_iteration"])
    print(json.dumps({
        "metric": "lora_apply_tokens_per_s_per_layer", "value": n_tok / (best["ms_per_iteration"] * 1e-3 / n_layers), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": best["ms_per_iteration"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"decode batches of {n_tok} one-token requests over {n_a} adapters (N_a/5 per rank 8..128, power law 1.2 within the rank), "
                               f"pool of {slots_per_rank} slots per rank, q,k,v,o 4096->4096 bf16, {n_layers} layers; misses loaded from pinned host memory "
                               "on a side stream; queue-driven prefetch at the listed depths", "tokens": n_tok, "layers_per_step": n_layers},
        "prefetch_depth": out, "roofline": None, "cpu_baseline": None}))
    return 0



def serve_replay(args) -> int:
    """Scheduler, cache manager, loads and applies together (paper sections 4.2-4.3) on Poisson arrivals:
    every iteration the new requests are submitted, the scheduler forms the batch (lora_sched_generate_batch),
    the adapters of the admitted requests are acquired (a miss is loaded whole from pinned host memory on a
    side stream), the adapters of waiting requests are prefetched, and the batch -- the prompts of the new
    requests, one token of every other running request -- goes through the apply of every projection and
    layer.  Inputs are synthetic: prompt lengths lognormal(6, 0.8) in [32, 2048], output lengths
    lognormal(3.5, 0.8) in [1, 256], the paper's adapter population.  The time to first token of a request
    is taken from the start of its arrival's iteration to the end of the iteration that ran its prompt.
    Run once with the queues fitted to the request sizes and once with a single queue.  Host-inclusive:
    the loop is Python calling the C ABI, synchronised every iteration.  One JSON line."""
    import torch
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd.pool import LoraPool

    n_a, n_layers = args.adapters if args.adapters != 100 else 200, args.layers or 4
    ranks = [8, 16, 32, 64, 128]
    per_rank = n_a // 5
    slots_per_rank = args.slots_per_rank or (3 * per_rank) // 4
    projs = [(4096, 4096)] * 4
    n_iter, warm = args.steps or 300, 40
    rate, total_tokens, max_batch_tokens = args.arrivals, args.token_budget, 32768
    rng = np.random.default_rng(11)
    w = 1.0 / np.arange(1, per_rank + 1) ** 1.2
    cdf = np.cumsum(w / w.sum())
    perm = [rng.permutation(per_rank) for _ in ranks]
    arrivals = []  # per iteration: [(input, output, adapter)]
    for _ in range(n_iter + warm):
        reqs = []
        for _ in range(int(rng.poisson(rate))):
            c = int(rng.integers(0, 5))
            k = int(min(np.searchsorted(cdf, rng.random()), per_rank - 1))
            reqs.append((int(np.clip(rng.lognormal(6.0, 0.8), 32, 2048)), int(np.clip(rng.lognormal(3.5, 0.8), 1, 256)), c * per_rank + int(perm[c][k])))
        arrivals.append(reqs)
    flat = [r for it in arrivals for r in it]
    sizes = [B.lora_sched_wrs(i, o, ranks[a // per_rank], 2048, 256, 128) for i, o, a in flat]

    dev = torch.device("cuda:0")
    part_bytes = {r: 2 * 4096 * r * 2 for r in ranks}
    adapter_bytes = [n_layers * 4 * part_bytes[ranks[a // per_rank]] for a in range(n_a)]
    arena = torch.empty(sum(adapter_bytes), dtype=torch.uint8, pin_memory=True)
    arena.view(torch.int16)[:] = 0x3c00
    parts_c, off = [], arena.data_ptr()
    for a in range(n_a):
        r, entries = ranks[a // per_rank], []
        for l in range(n_layers):
            for p in range(4):
                entries.append((l, p, off, off + part_bytes[r] // 2))
                off += part_bytes[r]
        parts_c.append(B.make_fill_parts(entries))
    x = torch.zeros((max_batch_tokens, 4096), device=dev, dtype=torch.bfloat16)
    y = torch.zeros((max_batch_tokens, 4096), device=dev, dtype=torch.bfloat16)
    stream, side = torch.cuda.current_stream(), torch.cuda.Stream()
    sh = stream.cuda_stream

    def run(k_max):
        rc, K, bounds = B.lora_sched_fit_queues(sizes, k_max)
        B.check(rc, "fit_queues")
        q_of = np.searchsorted(np.asarray(bounds), np.asarray(sizes), side="right") if bounds else np.zeros(len(sizes), int)
        need = np.asarray([i + o + ranks[a // per_rank] for i, o, a in flat])
        least = [int(need[q_of == q].max()) if (q_of == q).any() else 0 for q in range(K)]
        weights = [float(need[q_of == q].sum()) + 1.0 for q in range(K)]   # tokens the queue's requests ask for
        rc, quotas = B.lora_sched_assign_quotas(total_tokens, least, weights)
        B.check(rc, "assign_quotas")
        rc, sched = B.lora_sched_create(quotas, bounds, 2048, 256, 128, 1)
        B.check(rc, "sched_create")
        pool = LoraPool(projs, n_layers, ranks, [slots_per_rank] * 5, B.LORA_BF16, max_tokens=max_batch_tokens, max_segments=4096, n_plans=2,
                        flags=B.LORA_CACHE_DIRECT_FILL)
        h = pool.handle
        B.check(B.lora_cache_set_fencing(h, 1))
        descs = B.make_descs([(l, p, x.data_ptr(), y.data_ptr()) for l in range(n_layers) for p in range(4)])
        info, running = {}, {}   # request id -> (input, output, adapter, arrival time); -> [slot, outputs left, prompt pending]
        ttft, ttft_small, batch_tokens, refused = [], [], [], 0
        rid = 0
        small_cut = float(np.median(sizes))
        torch.cuda.synchronize()
        t_begin = None
        tokens_done = 0
        for it in range(n_iter + warm):
            if it == warm:
                t_begin = time.perf_counter()
                ttft, ttft_small, batch_tokens, tokens_done = [], [], [], 0
                B.lora_cache_stats(h)
            t_it = time.perf_counter()
            for (i, o, a) in arrivals[it]:
                B.check(B.lora_sched_submit(sched, rid, i, o, 1000 + a, ranks[a // per_rank])[0], "submit")
                info[rid] = (i, o, a, t_it)
                rid += 1
            rc, batch = B.lora_sched_generate_batch(sched)
            B.check(rc, "generate_batch")
            rc, queued = B.lora_sched_waiting_adapters(sched)
            queued_np = np.asarray(queued, np.int64) if queued else None
            fresh = []
            for r in batch:
                i, o, a, t_arr = info[r]
                rc, slot, hit = B.lora_cache_acquire(h, 1000 + a, ranks[a // per_rank], 1.0, True, queued_np)
                if rc == B.LORA_E_NOMEM:   # every slot that fits is held by running requests: the request gives its tokens back
                    B.check(B.lora_sched_finish(sched, r))
                    refused += 1
                    continue
                B.check(rc, "acquire")
                if not hit:
                    B.check(B.lora_cache_fill_slot_parts(h, slot, 1000 + a, ranks[a // per_rank], 1.0, parts_c[a], side.cuda_stream), "fill")
                running[r] = [slot, o, i]
                fresh.append(r)
            for aid in (queued[:args.prefetch] if queued else []):   # the adapters of the requests at the head of the queues
                a = aid - 1000
                rc, slot, hit = B.lora_cache_acquire(h, aid, ranks[a // per_rank], 1.0, False, queued_np)
                if rc == B.LORA_OK and not hit:
                    B.check(B.lora_cache_fill_slot_parts(h, slot, aid, ranks[a // per_rank], 1.0, parts_c[a], side.cuda_stream), "fill")
            if running:
                lens = [st[2] if st[2] else 1 for st in running.values()]
                T = int(sum(lens))
                if T > max_batch_tokens:
                    raise RuntimeError(f"batch of {T} tokens exceeds the {max_batch_tokens} the run allows for")
                seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
                seg_slot = np.asarray([st[0] for st in running.values()], np.int32)
                seg_rank = np.asarray([ranks[info[r][2] // per_rank] for r in running], np.int32)
                rc, plan = B.lora_plan_create(h, T, seg_off, seg_slot, seg_rank, sh)
                B.check(rc, "lora_plan_create")
                B.check(B.lora_apply_plan_multi(h, plan, descs, 2.0, sh), "lora_apply_plan_multi")
                B.check(B.lora_plan_destroy(h, plan))
                stream.synchronize()
                tokens_done += T
                batch_tokens.append(T)
            t_end = time.perf_counter()
            for r in fresh:
                d = (t_end - info[r][3]) * 1e3
                ttft.append(d)
                if sizes[r] < small_cut:
                    ttft_small.append(d)
            for r in list(running):
                st = running[r]
                st[2] = 0
                st[1] -= 1
                if st[1] <= 0:
                    B.check(B.lora_sched_finish(sched, r))
                    B.check(B.lora_cache_slot_ref(h, st[0], -1))
                    del running[r]
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_begin
        pool.check_fault()
        rc, stats = B.lora_cache_stats(h)
        waiting = sum(B.lora_sched_queue_state(sched, q)[2] for q in range(K))
        B.lora_sched_destroy(sched)
        pool.close()
        pct = lambda v, p: float(np.percentile(v, p)) if len(v) else None
        return {"queues": K, "boundaries": bounds, "quotas": quotas, "ms_per_iteration": elapsed * 1e3 / n_iter,
                "tokens_per_s_per_layer": tokens_done / elapsed, "mean_batch_tokens": float(np.mean(batch_tokens)) if batch_tokens else 0.0,
                "ttft_ms": {"p50": pct(ttft, 50), "p99": pct(ttft, 99)}, "ttft_ms_smaller_half": {"p50": pct(ttft_small, 50), "p99": pct(ttft_small, 99)},
                "requests_admitted": len(ttft), "requests_refused": refused, "requests_still_waiting": waiting,
                "cache": {"hits": int(stats.hits), "misses": int(stats.misses), "evictions": int(stats.evictions), "loaded_MB": stats.bytes_filled / 1e6}}

    fitted = run(4)
    single = run(1)
    print(json.dumps({
        "metric": "lora_apply_tokens_per_s_per_layer", "value": fitted["tokens_per_s_per_layer"], "unit": "tokens/s", "n_gpus": 1,
        "steps": n_iter, "warmup": warm, "ms_per_step": fitted["ms_per_iteration"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"serving replay: Poisson({rate}) requests per iteration, prompts lognormal(6,0.8) in [32,2048], outputs lognormal(3.5,0.8) in [1,256], "
                               f"{n_a} adapters (N_a/5 per rank 8..128, power law 1.2 within the rank), pool of {slots_per_rank} slots per rank, "
                               f"q,k,v,o 4096->4096 bf16, {n_layers} layers, token budget {total_tokens}, prefetch of {args.prefetch} waiting adapters; host-inclusive",
                   "layers_per_step": n_layers},
        "queues_fitted": fitted, "single_queue": single, "roofline": None, "cpu_baseline": None}))
    return 0



def run_workload(args, workload: str, steps: int = 0, cpu_baseline: bool = True, fused_base_only: bool = False, extras: bool = True) -> dict:
    """One workload measured: the record the JSON line is made of."""
    import torch
    import workloads as wl
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H

    steps = steps or DEFAULT_STEPS[workload]
    n_layers = args.layers or DEFAULT_LAYERS[workload]
    if workload == "decode_paper":
        inst = wl.decode_paper(seed=0, n_adapters=args.adapters, n_decode=args.tokens)
    elif workload == "decode_qkv" and args.tokens != 64:
        inst = wl.decode_qkv(seed=0, n_decode=args.tokens)
    else:
        inst = wl.CONFIGS[workload](seed=0)
    t_setup = time.time()
    pi = H.PooledInstance(inst, n_layers=n_layers, mfma_min_tokens=args.mfma_min_tokens, flags={"auto": 0, "fused": B.LORA_CACHE_FUSED_GEMV, "split": B.LORA_CACHE_SPLIT_GEMV}[args.gemv] | (B.LORA_CACHE_DIRECT_FILL if args.direct_fill else 0) | (B.LORA_CACHE_NO_OVERLAP if args.no_overlap else 0))
    h = pi.pool.handle
    dev = torch.device("cuda:0")

    # activation sets: enough of them that one rotation exceeds the Infinity Cache
    x_keys = sorted({p.x_key: p.h_in for p in inst.projs}.items())
    set_bytes = 2 * inst.T * (sum(w for _, w in x_keys) + sum(p.h_out for p in inst.projs))
    n_sets = args.sets or int(min(16, max(2, -(-768 * 2**20 // max(1, set_bytes)))))
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    xs, ys = [], []
    for _ in range(n_sets):
        xs.append({k: (torch.randn((inst.T, w), generator=gen, device=dev) * inst.sigma_x).to(torch.bfloat16) for k, w in x_keys})
        ys.append([(torch.randn((inst.T, p.h_out), generator=gen, device=dev) * inst.sigma_base).to(torch.bfloat16) for p in inst.projs])
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    B.check(B.lora_cache_set_fencing(h, 1))
    n_proj = len(inst.projs)

    if fused_base_only:
        out = fused_base(args, inst, pi, xs, ys, n_layers, n_sets, steps, stream)
        pi.close()
        return out

    descs = B.make_descs([(l, p, xs[l % n_sets][inst.projs[p].x_key].data_ptr(), ys[l % n_sets][p].data_ptr())
                          for l in range(n_layers) for p in range(n_proj)])

    def step(s: int) -> None:
        rc, plan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, sh)
        B.check(rc, "lora_plan_create")
        B.check(B.lora_apply_plan_multi(h, plan, descs, inst.scale, sh), "lora_apply_plan_multi")
        B.check(B.lora_plan_destroy(h, plan))

    # one cold call of the one-call form (index + upload + apply; first launch of the kernels in this process)
    torch.cuda.synchronize()
    t_c = time.perf_counter()
    B.check(B.lora_apply(h, 0, 0, xs[0][inst.projs[0].x_key].data_ptr(), ys[0][0].data_ptr(), inst.T, inst.seg_offsets,
                         pi.seg_slot, pi.seg_rank, inst.scale, sh), "lora_apply")
    torch.cuda.synchronize()
    cold_call_us = (time.perf_counter() - t_c) * 1e6

    # a GPU that has been idle runs its first second of work at about half speed (the same bench as the
    # first process on a fresh box: 0.83 ms per step, 0.46 ms with 1.4 s of steps before it): about a
    # second of untimed steps comes first, then the W warm-up steps, then the K timed ones
    prewarm_steps, t_pre = 0, time.perf_counter()
    while time.perf_counter() - t_pre < args.prewarm_s and prewarm_steps < 20000:
        for s in range(8):
            step(s)
        torch.cuda.synchronize()
        prewarm_steps += 8
    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step(args.warmup + s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps
    ms_per_layer = ms_per_step / n_layers
    tokens_per_s = inst.T / (ms_per_layer * 1e-3)

    # the same steps once more, each between two events: spread of the step time
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record(stream)
    for s in range(steps):
        step(args.warmup + s)
        evs[s + 1].record(stream)
    torch.cuda.synchronize()
    per_layer_us = np.sort([evs[i].elapsed_time(evs[i + 1]) * 1e3 / n_layers for i in range(steps)])
    spread = {"p10": float(per_layer_us[int(0.1 * (steps - 1))]), "median": float(np.median(per_layer_us)),
              "p90": float(per_layer_us[int(0.9 * (steps - 1))])}

    # the applies of a step recorded into a HIP graph once and replayed (what a decode loop does with its iteration):
    # same kernels, no host work per launch.  One plan, made outside the capture; fencing off while capturing.
    graph_replay = None
    if extras and not args.no_graph:
        rc, gplan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, sh)
        B.check(rc, "lora_plan_create")
        B.check(B.lora_apply_plan_multi(h, gplan, descs, inst.scale, sh), "lora_apply_plan_multi")  # eager once: fills seen as done
        torch.cuda.synchronize()
        B.check(B.lora_cache_set_fencing(h, 0))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, capture_error_mode="thread_local"):
            B.check(B.lora_apply_plan_multi(h, gplan, descs, inst.scale, torch.cuda.current_stream().cuda_stream), "lora_apply_plan_multi (capture)")
        B.check(B.lora_cache_set_fencing(h, 1))
        n_rep = max(5, steps)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        for _ in range(n_rep):
            g.replay()
        torch.cuda.synchronize()
        graph_replay = {"us_per_layer": (time.perf_counter() - t_g) * 1e6 / n_rep / n_layers, "replays": n_rep,
                        "eager_us_per_layer": ms_per_layer * 1e3}
        del g
        B.check(B.lora_plan_destroy(h, gplan))

    # host side of a step: indexing alone, and plan creation (index + validation + staging + enqueue of the upload)
    def host_us(fn, n=50):
        ts = []
        for _ in range(n):
            t1 = time.perf_counter()
            fn()
            ts.append((time.perf_counter() - t1) * 1e6)
        return float(np.median(ts))

    index_us = host_us(lambda: B.lora_index(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, B.LORA_MFMA_MIN_TOKENS, counts_only=True))

    def make_and_drop_plan():
        rc, plan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, sh)
        B.check(rc)
        B.check(B.lora_plan_destroy(h, plan))

    plan_us = host_us(make_and_drop_plan)
    torch.cuda.synchronize()

    # the work lists the library's plan holds (for the byte counts): same indexer, the plan's own threshold
    rc, plan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, sh)
    B.check(rc)
    rc, plan_info = B.lora_plan_info(plan)
    B.check(rc)
    B.check(B.lora_plan_destroy(h, plan))
    rc, w = B.lora_index(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, plan_info.mfma_min_tokens)
    B.check(rc)
    assert len(w["tiles"]) == plan_info.n_tiles
    per_proj = algorithmic_bytes(inst, w)
    step_bytes = sum(sum(b for k, b in v.items() if k != "gemv_fused") for v in per_proj)
    step_flops = sum(2 * it[1] * it[3] * (p.h_in + p.h_out) for p in inst.projs for it in (w["tiles"] + w["groups"]))

    roofline = None
    kernels = {}
    if not args.no_kernel_timing:
        # second pass over the same steps with an event pair around every kernel.  The host-side measurements above
        # left the GPU idle (its first work after that runs slower): a second of untimed steps first, then
        # the steps once with the event pairs on and unread, so that the pool of events has its size
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < min(1.0, args.prewarm_s):
            for s in range(4):
                step(s)
            torch.cuda.synchronize()
        n_steps_timed = max(1, min(steps, 400 // n_layers))
        B.check(B.lora_cache_set_timing(h, 1))
        for s in range(n_steps_timed):
            step(s)
        torch.cuda.synchronize()
        B.check(B.lora_cache_read_timing(h)[0])  # (reading hands the event pairs back to the pool)
        n_timed = n_steps_timed * n_layers  # layer passes
        for s in range(n_steps_timed):
            step(args.warmup + s)
        torch.cuda.synchronize()
        rc, tm = B.lora_cache_read_timing(h)
        B.check(rc)
        B.check(B.lora_cache_set_timing(h, 0))
        for kind, (ms, n) in tm.items():
            if n:
                kbytes = sum(v[kind] for v in per_proj) * n_timed  # all projections, all timed layer passes
                kernels[kind] = {"launches": int(n), "avg_us": ms * 1e3 / n, "algorithmic_bytes_per_launch": kbytes / n,
                                 "achieved_GBs": kbytes / (ms * 1e-3) / 1e9 if ms > 0 else None}
        dom = max(kernels, key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches"])
        roofline = {
            "bound": "hbm", "kernel": dom, "achieved": kernels[dom]["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": kernels[dom]["achieved_GBs"] / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC.get((workload, dom)) if args.gemv == "auto" and not args.mfma_min_tokens else None,
            "traffic_source": TRAFFIC_SOURCE if args.gemv == "auto" and not args.mfma_min_tokens and (workload, dom) in MEASURED_TRAFFIC else None,
            "avg_launch_us": kernels[dom]["avg_us"], "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes_per_launch"],
        }

    # stress only: adapters that miss are loaded from pinned host memory on a side stream while the applies run.
    # Loaded here are pool adapters the batch does not name (no ordering between the two streams), over and over,
    # for as long as a few steps take; reported: the fill rate alone and overlapped, the step time overlapped.
    fill_overlap = None
    if workload == "stress":
        unused = [a for a in range(len(inst.ranks)) if a not in set(int(u) for u in inst.used_adapters())][:6]
        host = []
        for a in unused:
            for p in range(n_proj):
                A, Bm = inst.adapter_weights(a, p)
                host.append((a, p, torch.from_numpy(A).to(torch.bfloat16).pin_memory(), torch.from_numpy(Bm).to(torch.bfloat16).pin_memory()))
        side = torch.cuda.Stream()
        part_bytes = sum((ta.numel() + tb.numel()) * 2 for _, _, ta, tb in host) * n_layers

        def enqueue_fills(rounds):
            for _ in range(rounds):
                for a, p, ta, tb in host:
                    for l in range(n_layers):
                        B.check(B.lora_cache_fill_slot(h, int(pi.slot_of[a]), int(inst.adapter_ids[a]), int(inst.ranks[a]),
                                                       float(inst.alpha[a]), l, p, ta.data_ptr(), tb.data_ptr(), side.cuda_stream))

        def timed(fill_rounds, n_steps):
            torch.cuda.synchronize()
            f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            f0.record(side)
            a0.record(stream)
            enqueue_fills(fill_rounds)
            f1.record(side)
            for s_ in range(n_steps):
                step(s_)
            a1.record(stream)
            torch.cuda.synchronize()
            return f0.elapsed_time(f1), a0.elapsed_time(a1)

        enqueue_fills(1)  # binds the slots, creates their events
        fill_alone_ms, _ = timed(2, 0)
        _, apply_alone_ms = timed(0, 6)
        rounds = max(1, int(round(2 * apply_alone_ms / fill_alone_ms)))  # about as much fill time as 6 steps take
        fill_ov_ms, apply_ov_ms = timed(rounds, 6)
        fill_overlap = {
            "adapters": len(unused), "bytes_per_round": part_bytes,
            "fill_GBs_alone": 2 * part_bytes / (fill_alone_ms * 1e-3) / 1e9,
            "fill_GBs_overlapped": rounds * part_bytes / (fill_ov_ms * 1e-3) / 1e9,
            "ms_per_layer_alone": apply_alone_ms / 6 / n_layers, "ms_per_layer_overlapped": apply_ov_ms / 6 / n_layers,
            "apply_slowdown": apply_ov_ms / apply_alone_ms,
        }

    cpu = None
    if cpu_baseline:
        import oracle

        # bounded sample: evenly spaced tokens of the batch, each as its own one-token segment
        n_samp = min(inst.T, 64 if workload == "decode" else 256)
        rows = np.unique(np.linspace(0, inst.T - 1, n_samp).astype(np.int64))
        ta = inst.token_adapter()[rows]
        off = np.arange(len(rows) + 1, dtype=np.int32)
        data = []
        for p in range(n_proj):
            ads = {int(a): (*inst.adapter_weights(int(a), p), float(inst.alpha[a])) for a in np.unique(ta[ta >= 0])}
            data.append((inst.x(p, rows).astype(np.float64), inst.base_out(p, rows).astype(np.float64), ads))
        reps, t_cpu = 0, 0.0
        while reps < 400 and t_cpu < 10.0:  # about 10 s of host work
            t1 = time.perf_counter()
            for x_, b_, ads in data:
                oracle.lora_apply(x_, b_, off, ta, ads, inst.scale)
            t_cpu += time.perf_counter() - t1
            reps += 1
        cpu = {"value": len(rows) * reps / t_cpu, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{len(rows)} evenly spaced tokens of the batch, all {n_proj} projection(s), {reps} repetition(s), fp64"}

    out = {
        "metric": "lora_apply_tokens_per_s_per_layer", "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[workload], "tokens": inst.T, "segments": inst.n_seg, "projections": n_proj,
                   "pool_adapters": int(inst.n_adapters), "distinct_adapters": int(len(inst.used_adapters())), "layers_per_step": n_layers, "activation_sets": n_sets,
                   "library_limits": "h_in and h_out multiples of 64, rank 1..128",
                   "ms_per_layer": ms_per_layer, "us_per_layer_spread": spread, "cold_single_call_us": cold_call_us,
                   "host_index_us": index_us, "host_plan_create_us": plan_us, "graph_replay": graph_replay,
                   "mfma_min_tokens": plan_info.mfma_min_tokens, "tiles": len(w["tiles"]), "gemv_shrink_items": plan_info.n_gemv_shrink_items, "gemv_groups": len(w["groups"])},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "fill_overlap": fill_overlap,
        "prewarm_steps": prewarm_steps,
        "layer": {"algorithmic_bytes": step_bytes, "flops": step_flops, "achieved_GBs": step_bytes / (ms_per_layer * 1e-3) / 1e9,
                  "hbm_frac": step_bytes / (ms_per_layer * 1e-3) / 1e9 / HBM_PEAK_GBS,
                  "achieved_TFLOPs": step_flops / (ms_per_layer * 1e-3) / 1e12, "setup_s": t_setup},
        "kernels": kernels,
    }
    pi.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="", choices=[""] + list(WORKLOAD_TEXT),
                    help="one workload alone; default: the decode configuration as the headline with the prefill, mixed and stress "
                         "configurations (and the decode batch on q,k,v as one group) as sub-records of the same line")
    ap.add_argument("--layers", type=int, default=0, help="layer copies of the pool to rotate over")
    ap.add_argument("--sets", type=int, default=0, help="activation buffer sets to rotate over")
    ap.add_argument("--gemv", default="auto", choices=["auto", "fused", "split"], help="GEMV shrink and expand as one launch, two, or chosen by size")
    ap.add_argument("--mfma-min-tokens", type=int, default=0, help="tokens of one slot from which the matrix-core tile path is taken (0: library default)")
    ap.add_argument("--direct-fill", action="store_true", help="fills read pinned host memory from the repack kernel (LORA_CACHE_DIRECT_FILL)")
    ap.add_argument("--adapters", type=int, default=100, help="decode_paper: number of adapters N_a (a multiple of 5)")
    ap.add_argument("--tokens", type=int, default=64, help="decode_paper, decode_qkv: one-token requests in the batch")
    ap.add_argument("--fused-base", action="store_true", help="time lora_linear_plan (base projection and adapter update in one pass; "
                    "random base weights) instead of the apply on a given base output; prints its own JSON line")
    ap.add_argument("--prefetch-depths", default="", help="e.g. 0,1,2,4: run the queue-driven prefetch experiment instead (own JSON line); "
                    "uses --tokens (default 256), --adapters (default 200), --layers (default 8), --slots-per-rank, --direct-fill, --fill-by-part")
    ap.add_argument("--serve", action="store_true", help="replay Poisson arrivals through scheduler, cache manager, loads and applies (own JSON line); "
                    "uses --arrivals, --token-budget, --prefetch, --adapters (default 200), --layers (default 4), --slots-per-rank, --steps (iterations)")
    ap.add_argument("--arrivals", type=float, default=1.0, help="--serve: mean requests arriving per iteration")
    ap.add_argument("--token-budget", type=int, default=65536, help="--serve: tokens the scheduler's queues share")
    ap.add_argument("--prefetch", type=int, default=8, help="--serve: adapters of waiting requests prefetched per iteration")
    ap.add_argument("--fill-by-part", action="store_true", help="prefetch experiment: one lora_cache_fill_slot call per (layer, projection) "
                    "instead of one lora_cache_fill_slot_parts call per adapter")
    ap.add_argument("--slots-per-rank", type=int, default=0, help="prefetch experiment: pool slots per rank class (default: all but 3 of the 40 adapters of a rank)")
    ap.add_argument("--prewarm-s", type=float, default=1.0, help="seconds of untimed steps before the warm-up steps (a cold GPU ramps its clocks)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the graph-replay timing of the step")
    ap.add_argument("--no-overlap", action="store_true", help="the GEMV launch of an apply behind its tile kernels instead of beside them (LORA_CACHE_NO_OVERLAP): "
                    "per-kernel durations of a trace then stand for the kernels alone")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1\n")
        return 2

    import torch

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible; the library has no CPU path\n")
        return 2
    import workloads as wl
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H

    if args.prefetch_depths:
        return prefetch_sweep(args)
    if args.serve:
        return serve_replay(args)
    if args.workload:  # one workload, as named
        out = run_workload(args, args.workload, args.steps, cpu_baseline=not args.no_cpu_baseline, fused_base_only=args.fused_base)
        print(json.dumps(out))
        return 0
    # default: the decode configuration is the headline (the metric's bandwidth half is quoted on it); the other
    # configurations ride along as sub-records of the same line, each measured the same way with fewer steps
    out = run_workload(args, "decode", args.steps, cpu_baseline=not args.no_cpu_baseline)
    keep = ("value", "ms_per_step", "steps", "roofline", "kernels", "layer", "fill_overlap")
    out["configs"] = {}
    for name in ("prefill", "mixed", "stress", "decode_qkv"):
        rec = run_workload(args, name, 0, cpu_baseline=False)
        sub = {k: rec[k] for k in keep if rec.get(k) is not None}
        sub["workload"] = rec["config"]["workload"]
        for k in ("tokens", "projections", "layers_per_step", "ms_per_layer", "distinct_adapters", "tiles", "gemv_shrink_items", "graph_replay"):
            if k in rec["config"]:
                sub[k] = rec["config"][k]
        sub["tokens_per_s_per_layer"] = sub.pop("value")
        if name == "prefill":  # the metric's matrix-core half: base projection and adapter update in one kernel
            fb = run_workload(args, name, 0, cpu_baseline=False, fused_base_only=True)
            sub["fused_base"] = {"ms_per_layer": fb["config"]["ms_per_layer"],
                                 "vendor_matmul_then_apply_ms_per_layer": fb["config"]["vendor_matmul_then_apply_ms_per_layer"],
                                 "roofline": fb["roofline"], "kernels": fb["kernels"]}
        out["configs"][name] = sub
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
