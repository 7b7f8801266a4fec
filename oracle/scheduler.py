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
* a batch is formed in two passes (the paper's batch-generation algorithm): first every queue, from
  the smallest requests up, admits requests in arrival order while its own free quota lasts and
  stops at the first that does not fit; a queue that ran empty leaves its unused quota as spare
  tokens; then, again from the smallest requests up, each queue admits further requests out
  of the spare tokens in the same way, until none are left;
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

import bisect
import functools
import itertools
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

    In one dimension the optimal clusters are runs of the sorted values.  Stated as a recursion on what
    is left: the best way to put the values from position `i` on into `c` clusters is the best choice of
    where the first of them ends, plus the best way to put the rest into c - 1 (memoised)."""
    xs = sorted(values)
    n = len(xs)
    k = min(k, n)
    # sums and sums of squares up to a position: the sum of squares of a run around its own mean in closed form
    s1 = [0.0] + list(itertools.accumulate(xs))
    s2 = [0.0] + list(itertools.accumulate(x * x for x in xs))

    def spread(i: int, j: int) -> float:  # of xs[i:j], j > i
        return max(0.0, (s2[j] - s2[i]) - (s1[j] - s1[i]) ** 2 / (j - i))

    @functools.lru_cache(maxsize=None)
    def rest(i: int, c: int) -> Tuple[float, Tuple[int, ...]]:
        """-> (sum of squares, ends of the clusters) for xs[i:] in c clusters."""
        if c == 1:
            return spread(i, n), (n,)
        options = ((spread(i, j) + rest(j, c - 1)[0], j) for j in range(i + 1, n - c + 2))
        cost, j = min(options)  # ties: the earliest end
        return cost, (j,) + rest(j, c - 1)[1]

    if n == 0:
        return 0.0, []
    cost, ends = rest(0, k)
    starts = (0,) + ends[:-1]
    # the cost once more from the clusters themselves, around their means (no cancellation)
    exact = sum(_sse(xs[i:j]) for i, j in zip(starts, ends))
    return exact, [sum(xs[i:j]) / (j - i) for i, j in zip(starts, ends)]


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

    def _fitting(self, q: int, tokens: int) -> int:
        """How many requests at the head of queue q can be admitted, in arrival order, out of `tokens`:
        the longest prefix whose needs add up to no more than that (admission stops at the first request
        that does not fit, later ones do not overtake it)."""
        upto = list(itertools.accumulate(self.needed(r) for r in self.queues[q]))
        return bisect.bisect_right(upto, tokens)

    def generate_batch(self) -> List[int]:
        """One batch, as section 4.3 describes its formation (two passes over the queues, smallest requests first).

        The first pass is per queue and independent of the others: a queue admits what fits its own free quota.
        The second pass hands out what emptied queues left over.  Those leftovers are laid end to end, queue after
        queue, as one line of tokens; every request admitted in the second pass takes the next stretch of that line,
        and owes each queue the part of its stretch that lies in that queue's leftover."""
        batch: List[Request] = []

        def admit(r: Request) -> None:
            self.running[r.req_id] = r
            batch.append(r)

        lots: List[Tuple[int, int]] = []  # (owner queue, tokens), in queue order
        for q in range(len(self.queues)):
            for _ in range(self._fitting(q, self.free[q])):
                r = self.queues[q].popleft()
                r.borrowed.append((q, self.needed(r)))
                self.free[q] -= self.needed(r)
                admit(r)
            if not self.queues[q] and self.free[q] > 0:
                lots.append((q, self.free[q]))

        ends = list(itertools.accumulate(t for _, t in lots))  # where each lot ends on the line
        line = ends[-1] if ends else 0
        at = 0  # tokens of the line handed out so far
        for q in range(len(self.queues)):
            if at == line:
                break
            for _ in range(self._fitting(q, line - at)):
                r = self.queues[q].popleft()
                lo, hi = at, at + self.needed(r)
                for (owner, tokens), end in zip(lots, ends):
                    part = min(hi, end) - max(lo, end - tokens)  # overlap of [lo, hi) with this lot
                    if part > 0:
                        r.borrowed.append((owner, part))
                        self.free[owner] -= part
                at = hi
                admit(r)
        return [r.req_id for r in batch]

    def finish(self, req_id: int) -> None:
        r = self.running.pop(req_id)
        for q, tokens in r.borrowed:
            self.free[q] += tokens

    def waiting_adapters(self) -> List[int]:
        """Adapters of the requests still in the queues (what the cache manager spares and prefetches)."""
        return [r.adapter_id for q in self.queues for r in q]
