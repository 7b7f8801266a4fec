"""CPU ORACLE (test infrastructure, not part of the product): the request scheduler of paper section 4.3.

Plain Python, written from the paper's description; only `tests/` imports it.

What the paper fixes:

* request size:  WRS = (A * input / max_input + B * output / max_output) * rank / max_rank,
  A = 0.4, B = 0.6, output = the predicted output length;
* K queues ordered by request size; queue 1 takes sizes below boundary 1, queue i sizes from
  boundary i-1 (inclusive) up to boundary i (exclusive);
* boundaries are the midpoints between consecutive centroids of a K-means clustering of the
  request sizes, K <= 4;
* every queue owns a quota of tokens; a request needs its input tokens + its output tokens + the
  tokens its adapter's memory amounts to; an admitted request borrows what it needs and gives it
  back when it ends;
* a batch is formed in two phases (the paper's batch-generation listing): first every queue, from
  the smallest requests up, admits requests in arrival order while its own free quota lasts and
  stops at the first that does not fit; a queue that ran empty puts its unused quota into a common
  spare bucket; then, again from the smallest requests up, each queue admits further requests out
  of the bucket in the same way, until the bucket is empty;
* the least quota of a queue whose largest request has S tokens, takes D to process, arrives at rate
  lambda and must meet an SLO is  S * D * (1 / SLO + lambda);  every queue gets its least quota and the
  rest of the tokens is split in proportion to given weights.

Readings where the paper is silent or at odds with itself (the library takes the same ones):

* tokens of the spare bucket remember the queue they came from: they are drawn in queue order and
  go back to that queue when the borrowing request ends, so the quotas are conserved;
* "the K with minimal WCSS" cannot be meant literally (the within-cluster sum of squares never grows
  with K): K is the one whose step from K-1 removes the largest fraction of the remaining sum of
  squares (1 if all sizes are equal);
* the clustering is the exact one-dimensional K-means optimum (clusters are runs of the sorted
  sizes), not a randomly initialised iteration;
* quotas are whole tokens: least quotas are rounded up, proportional shares down, and the tokens
  left by the rounding go to the queues one each from the smallest requests up.

Pins (tests/test_oracle_scheduler.py): hand-worked WRS values and batches (the two situations the
paper's scheduler figure walks through), brute force over all splits for the clustering, the
M/M/1 sojourn time 1 / (mu - lambda) = SLO at the least quota, conservation of quotas on random
traces, first-come-first-served order within a queue.
"""
from __future__ import annotations

import math
from collections import deque
from typing import Dict, List, Sequence, Tuple


def wrs(input_len: int, output_len: int, rank: int, max_input: int, max_output: int, max_rank: int,
        a: float = 0.4, b: float = 0.6) -> float:
    return (a * (input_len / max_input) + b * (output_len / max_output)) * (rank / max_rank)


def queue_of(size: float, boundaries: Sequence[float]) -> int:
    q = 0
    for bound in boundaries:
        if size >= bound:
            q += 1
    return q


# ---- number of queues and boundaries ------------------------------------------------------------

def _sse(values: Sequence[float]) -> float:
    if not values:
        return 0.0
    mean = sum(values) / len(values)
    return sum((v - mean) ** 2 for v in values)


def kmeans_1d(values: Sequence[float], k: int) -> Tuple[float, List[float]]:
    """Optimal K-means of numbers on a line -> (within-cluster sum of squares, centroids ascending).

    In one dimension the optimal clusters are runs of the sorted values, so the optimum is found by
    trying, for every prefix and every number of clusters, every place for the last cut."""
    xs = sorted(values)
    n = len(xs)
    k = min(k, n)
    best = [[math.inf] * (n + 1) for _ in range(k + 1)]
    cut = [[0] * (n + 1) for _ in range(k + 1)]
    best[0][0] = 0.0
    for c in range(1, k + 1):
        for end in range(c, n + 1):
            for start in range(c - 1, end):
                cost = best[c - 1][start] + _sse(xs[start:end])
                if cost < best[c][end]:
                    best[c][end] = cost
                    cut[c][end] = start
    centroids = []
    end = n
    for c in range(k, 0, -1):
        start = cut[c][end]
        centroids.append(sum(xs[start:end]) / (end - start))
        end = start
    return best[k][n], centroids[::-1]


def fit_queues(sizes: Sequence[float], k_max: int = 4) -> Tuple[int, List[float]]:
    """-> (number of queues, boundaries between them)."""
    k_max = min(k_max, len(set(sizes)))
    wcss = [None] + [kmeans_1d(sizes, k)[0] for k in range(1, k_max + 1)]
    k_best, drop_best = 1, 0.0
    for k in range(2, k_max + 1):
        if wcss[k - 1] <= 0.0:
            break
        drop = (wcss[k - 1] - wcss[k]) / wcss[k - 1]
        if drop > drop_best:
            k_best, drop_best = k, drop
    centroids = kmeans_1d(sizes, k_best)[1]
    return k_best, [(centroids[i] + centroids[i + 1]) / 2 for i in range(k_best - 1)]


# ---- quotas --------------------------------------------------------------------------------------

def min_quota(max_request_tokens: float, duration: float, slo: float, arrival_rate: float) -> int:
    return math.ceil(max_request_tokens * duration * (1.0 / slo + arrival_rate))

def assign_quotas(total_tokens: int, least: Sequence[int], weights: Sequence[float]) -> List[int]:
    """Every queue its least quota, the rest in proportion to the weights; None if the total is too small."""
    rest = total_tokens - sum(least)
    if rest < 0:
        return None
    wsum = sum(weights)
    quota = [int(l) + int(math.floor(rest * (w / wsum))) for l, w in zip(least, weights)]
    left = total_tokens - sum(quota)
    i = 0
    while left > 0:
        quota[i % len(quota)] += 1
        left -= 1
        i += 1
    return quota


# ---- the queues ----------------------------------------------------------------------------------

class Request:
    __slots__ = ("req_id", "input_len", "output_len", "adapter_id", "rank", "queue", "borrowed")

    def __init__(self, req_id, input_len, output_len, adapter_id, rank, queue):
        self.req_id, self.input_len, self.output_len = req_id, input_len, output_len
        self.adapter_id, self.rank, self.queue = adapter_id, rank, queue
        self.borrowed: List[Tuple[int, int]] = []  # (queue the tokens belong to, tokens)


class Scheduler:
    def __init__(self, quotas: Sequence[int], boundaries: Sequence[float], max_input: int, max_output: int,
                 max_rank: int, tokens_per_rank: int, a: float = 0.4, b: float = 0.6):
        assert len(quotas) == len(boundaries) + 1
        self.free = [int(q) for q in quotas]
        self.quota = [int(q) for q in quotas]
        self.boundaries = list(boundaries)
        self.norm = (max_input, max_output, max_rank)
        self.tokens_per_rank = tokens_per_rank
        self.a, self.b = a, b
        self.queues: List[deque] = [deque() for _ in quotas]
        self.running: Dict[int, Request] = {}

    def submit(self, req_id: int, input_len: int, output_len: int, adapter_id: int, rank: int) -> int:
        size = wrs(input_len, output_len, rank, *self.norm, self.a, self.b)
        q = queue_of(size, self.boundaries)
        self.queues[q].append(Request(req_id, input_len, output_len, adapter_id, rank, q))
        return q

    def needed(self, r: Request) -> int:
        return r.input_len + r.output_len + r.rank * self.tokens_per_rank

    def _put_batch(self, q: int, sources: List[List[int]], batch: List[Request]) -> int:
        """Admit requests of queue q in arrival order out of `sources` ([queue, tokens] pairs, drawn in
        order); stop at the first that does not fit.  -> tokens consumed."""
        consumed = 0
        while self.queues[q]:
            r = self.queues[q][0]
            need = self.needed(r)
            if sum(t for _, t in sources) < need:
                break
            take = need
            for src in sources:
                part = min(take, src[1])
                if part > 0:
                    src[1] -= part
                    self.free[src[0]] -= part
                    r.borrowed.append((src[0], part))
                    take -= part
            consumed += need
            self.queues[q].popleft()
            self.running[r.req_id] = r
            batch.append(r)
        return consumed

    def generate_batch(self) -> List[int]:
        batch: List[Request] = []
        bucket: List[List[int]] = []
        for q in range(len(self.queues)):            # phase 1: every queue out of its own free quota
            own = [[q, self.free[q]]]
            self._put_batch(q, own, batch)
            if not self.queues[q] and own[0][1] > 0:
                bucket.append(own[0])                # what an emptied queue did not use is spare
        for q in range(len(self.queues)):            # phase 2: the spare tokens, smallest requests first
            if sum(t for _, t in bucket) == 0:
                break
            self._put_batch(q, bucket, batch)
        return [r.req_id for r in batch]

    def finish(self, req_id: int) -> None:
        r = self.running.pop(req_id)
        for q, tokens in r.borrowed:
            self.free[q] += tokens

    def waiting_adapters(self) -> List[int]:
        """Adapters of the requests still in the queues (what the cache manager spares and prefetches)."""
        return [r.adapter_id for q in self.queues for r in q]
