"""Replay a synthetic request trace through the library's cache manager under three eviction
policies (section 4.2 and the caching-policy comparison of section 5 of the paper): recency only
(LRU), equal weights (FairShare) and the paper's 0.45 / 0.10 / 0.45.

Host-only: no GPU, no adapter weights; what is counted is hits and the bytes a miss would load
over the host link (q, k, v, o of a 32-layer 7B-shaped model at 16 bit).

The trace stands in for the paper's production trace, which is not public in this form:
N adapters, ranks uniform over {8, 16, 32, 64, 128}, popularity Zipf(alpha) over all adapters through
a seeded permutation, `running` requests in flight at any time (each holds a reference to its
adapter until it ends, in arrival order), the adapters of the next `queued` arrivals known to the
manager.  The cache has one rank class per rank with `slots_per_class` slots each.

    python -m paper_2411_17741_amd.tools.policy_trace [--adapters 500] [--alpha 1.2] [--slots 12] [--requests 200000]
"""
from __future__ import annotations

import argparse
import collections

import numpy as np

from paper_2411_17741_amd import binding as B

RANKS = (8, 16, 32, 64, 128)
POLICIES = (("LRU", (0.0, 1.0, 0.0)), ("FairShare", (1 / 3, 1 / 3, 1 / 3)), ("Chameleon", (0.45, 0.10, 0.45)))


def make_trace(n_adapters: int, alpha: float, n_requests: int, seed: int):
    rng = np.random.default_rng(seed)
    ranks = rng.choice(RANKS, size=n_adapters)
    p = 1.0 / np.arange(1, n_adapters + 1) ** alpha
    p /= p.sum()
    order = rng.permutation(n_adapters)
    ids = order[rng.choice(n_adapters, size=n_requests, p=p)]
    return ranks, ids


def replay(weights, window, ranks, ids, slots_per_class: int, running: int, queued: int):
    cfg = B.make_config([(4096, 4096)] * 4, 32, list(RANKS), [slots_per_class] * len(RANKS), B.LORA_BF16, 64, 64,
                        flags=B.LORA_CACHE_HOST_ONLY)
    rc, h = B.lora_cache_create(cfg, 0, 0)
    B.check(rc, "lora_cache_create")
    try:
        B.check(B.lora_cache_set_policy(h, *weights, window))
        in_flight = collections.deque()
        loaded = refused = 0
        by_rank = {r: [0, 0] for r in RANKS}  # requests, misses
        for i, a in enumerate(ids):
            rank = int(ranks[a])
            rc, slot, hit = B.lora_cache_acquire(h, int(a) + 1, rank, 1.0, True, ids[i + 1:i + 1 + queued] + 1)
            if rc == B.LORA_E_NOMEM:
                refused += 1  # every slot that fits is held by a running request: the request would wait
            else:
                B.check(rc, "lora_cache_acquire")
                by_rank[rank][0] += 1
                if not hit:
                    by_rank[rank][1] += 1
                    loaded += 4 * 32 * B.lora_adapter_bytes(4096, 4096, rank, B.LORA_BF16)
                in_flight.append(slot)
            while len(in_flight) > running:
                B.check(B.lora_cache_slot_ref(h, in_flight.popleft(), -1))
        rc, st = B.lora_cache_stats(h)
        return st.hits / max(1, st.hits + st.misses), loaded, refused, by_rank
    finally:
        B.lora_cache_destroy(h)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--adapters", type=int, default=500)
    ap.add_argument("--alpha", type=float, default=1.2)
    ap.add_argument("--slots", type=int, default=12, help="slots per rank class")
    ap.add_argument("--requests", type=int, default=200000)
    ap.add_argument("--running", type=int, default=32)
    ap.add_argument("--queued", type=int, default=16)
    ap.add_argument("--window", type=int, default=0, help="requests after which use counts are halved (0: never)")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    ranks, ids = make_trace(args.adapters, args.alpha, args.requests, args.seed)
    print(f"{args.adapters} adapters, Zipf({args.alpha}), {args.requests} requests, {args.slots} slots per rank class "
          f"({args.slots * len(RANKS)} of {args.adapters} adapters fit), {args.running} running, {args.queued} queued known")
    print(f"{'policy':10s} {'hit rate':>9s} {'loaded GB':>10s} {'refused':>8s}   miss rate by rank " + " ".join(f"{r:>6d}" for r in RANKS))
    for name, w in POLICIES:
        hit, loaded, refused, by_rank = replay(w, args.window, ranks, ids, args.slots, args.running, args.queued)
        print(f"{name:10s} {hit:9.4f} {loaded / 1e9:10.1f} {refused:8d}   " + " " * 18 +
              " ".join(f"{by_rank[r][1] / max(1, by_rank[r][0]):6.3f}" for r in RANKS))


if __name__ == "__main__":
    main()
