"""Seeded instance generator (inputs only; see the package docstring).

Every array is produced from a Philox stream keyed by (seed, purpose, index), in
row blocks, so that any single adapter or any subset of token rows can be
regenerated alone and is bit-identical to the same rows of the full array.
Values are drawn in fp32 and, for bf16 instances, rounded to nearest-even bf16
and handed out as fp32 arrays holding exactly representable bf16 values (plus a
helper to get the 16-bit patterns for upload).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

ROW_BLOCK = 256  # rows drawn from one stream; sampling regenerates whole blocks

# stream purposes
_P_X, _P_BASE, _P_A, _P_B, _P_RANK, _P_POP, _P_LEN, _P_ORDER, _P_MISS, _P_W = range(10)


# ---------------------------------------------------------------------------
# number formats
# ---------------------------------------------------------------------------
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the fp32 values they denote."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 -> fp32 array whose every value is exactly a bf16 number."""
    return bf16_from_bits(bf16_bits(a))


def _rng(seed: int, purpose: int, *idx: int) -> np.random.Generator:
    ss = np.random.SeedSequence([int(seed) & 0xFFFFFFFF, int(purpose)] + [int(i) & 0xFFFFFFFF for i in idx])
    return np.random.Generator(np.random.Philox(ss))


# ---------------------------------------------------------------------------
@dataclass
class Projection:
    name: str
    h_in: int
    h_out: int
    x_key: int  # projections with the same x_key read the same activation tensor


@dataclass
class Instance:
    name: str
    dtype: str  # "f32" | "bf16"
    seed: int
    projs: List[Projection]
    ranks: np.ndarray  # [n_adapters] int32, rank of pool adapter a
    adapter_ids: np.ndarray  # [n_adapters] int64, caller-visible ids
    alpha: np.ndarray  # [n_adapters] float32, per-adapter factor kept in the cache entry
    scale: float
    seg_offsets: np.ndarray  # [n_seg+1] int32
    seg_adapter: np.ndarray  # [n_seg] int32 index into the pool, -1 = no adapter
    sigma_w: float = 0.02
    sigma_x: float = 1.0
    sigma_base: float = 1.28
    n_layers: int = 1
    miss_adapters: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    note: str = ""

    # -- structure ----------------------------------------------------------
    @property
    def T(self) -> int:
        return int(self.seg_offsets[-1])

    @property
    def n_seg(self) -> int:
        return int(len(self.seg_adapter))

    @property
    def n_adapters(self) -> int:
        return int(len(self.ranks))

    @property
    def seg_rank(self) -> np.ndarray:
        r = np.where(self.seg_adapter >= 0, self.ranks[np.maximum(self.seg_adapter, 0)], 0)
        return r.astype(np.int32)

    def used_adapters(self) -> np.ndarray:
        lens = np.diff(self.seg_offsets)
        m = (self.seg_adapter >= 0) & (lens > 0)
        return np.unique(self.seg_adapter[m]).astype(np.int32)

    def token_adapter(self) -> np.ndarray:
        """[T] pool index per token, as handed to the generator (-1 = none)."""
        return np.repeat(self.seg_adapter, np.diff(self.seg_offsets)).astype(np.int32)

    # -- values -------------------------------------------------------------
    def _q(self, a: np.ndarray) -> np.ndarray:
        return bf16_round(a) if self.dtype == "bf16" else np.ascontiguousarray(a, np.float32)

    def adapter_weights(self, a: int, p: int) -> Tuple[np.ndarray, np.ndarray]:
        """(A [h_in][r], B [r][h_out]) of pool adapter `a` for projection `p`."""
        pr, r = self.projs[p], int(self.ranks[a])
        A = _rng(self.seed, _P_A, a, p).standard_normal((pr.h_in, r), dtype=np.float32) * np.float32(self.sigma_w)
        B = _rng(self.seed, _P_B, a, p).standard_normal((r, pr.h_out), dtype=np.float32) * np.float32(self.sigma_w)
        return self._q(A), self._q(B)

    def _rows(self, purpose: int, key: int, width: int, sigma: float, rows: Optional[Sequence[int]]) -> np.ndarray:
        T = self.T
        if rows is None:
            nblk = (T + ROW_BLOCK - 1) // ROW_BLOCK
            out = np.empty((T, width), np.float32)

            def fill(b: int) -> None:
                lo, hi = b * ROW_BLOCK, min(T, (b + 1) * ROW_BLOCK)
                blk = _rng(self.seed, purpose, key, b).standard_normal((ROW_BLOCK, width), dtype=np.float32)
                out[lo:hi] = self._q(blk[: hi - lo] * np.float32(sigma))

            if nblk > 4:
                with ThreadPoolExecutor(max_workers=8) as ex:
                    list(ex.map(fill, range(nblk)))
            else:
                for b in range(nblk):
                    fill(b)
            return out
        rows = np.asarray(rows, np.int64)
        out = np.empty((len(rows), width), np.float32)
        cache: Dict[int, np.ndarray] = {}
        for i, t in enumerate(rows):
            b = int(t) // ROW_BLOCK
            if b not in cache:
                blk = _rng(self.seed, purpose, key, b).standard_normal((ROW_BLOCK, width), dtype=np.float32)
                cache = {b: self._q(blk * np.float32(sigma))}
            out[i] = cache[b][int(t) - b * ROW_BLOCK]
        return out

    def x(self, p: int, rows: Optional[Sequence[int]] = None) -> np.ndarray:
        """Activations [T][h_in] read by projection p (or only `rows` of them)."""
        pr = self.projs[p]
        return self._rows(_P_X, pr.x_key, pr.h_in, self.sigma_x, rows)

    def base_out(self, p: int, rows: Optional[Sequence[int]] = None) -> np.ndarray:
        """Base-model output x.W [T][h_out] that the adapter delta is added to.

        Drawn directly as N(0, sigma_base) (the spread x.W has for W ~ N(0, 0.02)
        and h_in = 4096) instead of multiplying by a materialised W.
        """
        pr = self.projs[p]
        return self._rows(_P_BASE, p, pr.h_out, self.sigma_base, rows)

    def base_weight(self, p: int) -> np.ndarray:
        """Dense W [h_in][h_out] ~ N(0, sigma_w); only meant for small instances."""
        pr = self.projs[p]
        W = _rng(self.seed, _P_W, p).standard_normal((pr.h_in, pr.h_out), dtype=np.float32) * np.float32(self.sigma_w)
        return self._q(W)


# ---------------------------------------------------------------------------
# distributions
# ---------------------------------------------------------------------------
def _zipf_choice(rng: np.random.Generator, n_items: int, alpha: float, size: int) -> np.ndarray:
    k = np.arange(1, n_items + 1, dtype=np.float64)
    p = k ** (-alpha)
    p /= p.sum()
    return rng.choice(n_items, size=size, p=p)


def _prompt_lengths(rng: np.random.Generator, n: int, mu: float = 6.0, sigma: float = 0.8, lo: int = 32, hi: int = 2048) -> np.ndarray:
    ln = np.exp(rng.normal(mu, sigma, size=n))
    return np.clip(np.rint(ln), lo, hi).astype(np.int32)


def _llama_projs(hidden: int, inter: int) -> List[Projection]:
    return [
        Projection("q", hidden, hidden, 0),
        Projection("k", hidden, hidden, 0),
        Projection("v", hidden, hidden, 0),
        Projection("o", hidden, hidden, 1),
        Projection("gate", hidden, inter, 2),
        Projection("up", hidden, inter, 2),
        Projection("down", inter, hidden, 3),
    ]


def make_instance(
    name: str,
    *,
    dtype: str,
    seed: int,
    projs: List[Projection],
    n_adapters: int,
    rank_choices: Sequence[int],
    n_decode: int,
    prompt_lens: Sequence[int],
    zipf_alpha: Optional[float],
    distinct_prefill_adapters: bool = False,
    prefill_rank_choices: Optional[Sequence[int]] = None,
    scale: float = 2.0,
    n_layers: int = 1,
    miss_fraction: float = 0.0,
    n_base_only: int = 0,
    note: str = "",
    popularity_within_rank: bool = False,
) -> Instance:
    """Mixed prefill/decode batch: one segment per request, requests in seeded order.

    popularity_within_rank: the paper's own law (section 5.1) -- every rank has the same number of
    adapters, a request draws its rank uniformly and then an adapter of that rank by a power law
    (exponent zipf_alpha; the paper does not state it).  Otherwise ranks are drawn per adapter and
    one power law runs over the whole pool."""
    n_pre = len(prompt_lens)
    n_req = n_decode + n_pre + n_base_only
    prng = _rng(seed, _P_POP, 1)
    perm = _rng(seed, _P_POP, 0).permutation(n_adapters)  # popularity rank -> pool index
    if popularity_within_rank:
        n_ranks = len(rank_choices)
        assert n_adapters % n_ranks == 0 and zipf_alpha is not None
        per_rank = n_adapters // n_ranks
        ranks = np.empty(n_adapters, np.int32)
        ranks[perm] = np.repeat(np.asarray(rank_choices, np.int32), per_rank)  # perm[c * per_rank + k]: k-th most popular of rank c
        cls = prng.integers(0, n_ranks, size=n_req)
        pick = perm[cls * per_rank + _zipf_choice(prng, per_rank, zipf_alpha, n_req)]
    else:
        ranks = _rng(seed, _P_RANK).choice(np.asarray(rank_choices, np.int32), size=n_adapters).astype(np.int32)
        if zipf_alpha is None:
            pick = prng.integers(0, n_adapters, size=n_req)
        else:
            pick = perm[_zipf_choice(prng, n_adapters, zipf_alpha, n_req)]
    pick = pick.astype(np.int32)
    lens = np.concatenate([np.ones(n_decode, np.int32), np.asarray(prompt_lens, np.int32), np.ones(n_base_only, np.int32)])
    if distinct_prefill_adapters and n_pre:
        # every prompt gets its own adapter; its rank is redrawn from prefill_rank_choices
        chosen = perm[:n_pre].astype(np.int32)
        if prefill_rank_choices is not None:
            ranks[chosen] = _rng(seed, _P_RANK, 1).choice(np.asarray(prefill_rank_choices, np.int32), size=n_pre)
        pick[n_decode : n_decode + n_pre] = chosen
    if n_base_only:
        pick[n_decode + n_pre :] = -1
    order = _rng(seed, _P_ORDER).permutation(n_req)
    lens, pick = lens[order], pick[order]
    seg_offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    inst = Instance(
        name=name,
        dtype=dtype,
        seed=seed,
        projs=projs,
        ranks=ranks,
        adapter_ids=(np.arange(n_adapters, dtype=np.int64) * 7919 + 100003),
        alpha=np.ones(n_adapters, np.float32),
        scale=float(scale),
        seg_offsets=seg_offsets,
        seg_adapter=pick,
        n_layers=n_layers,
        note=note,
    )
    if miss_fraction > 0:
        used_req = np.flatnonzero(pick >= 0)
        n_miss = int(np.ceil(miss_fraction * len(used_req)))
        miss_req = _rng(seed, _P_MISS).choice(used_req, size=n_miss, replace=False)
        inst.miss_adapters = np.unique(pick[miss_req]).astype(np.int32)
    return inst


# ---------------------------------------------------------------------------
# the five configurations, plus a small all-paths one for fast parity runs
# ---------------------------------------------------------------------------
def tiny(seed: int = 0) -> Instance:
    """One 256->256 fp32 projection, ranks {4,8,8,16}, 16 tokens in segments {1,3,5,7}."""
    return Instance(
        name="tiny",
        dtype="f32",
        seed=seed,
        projs=[Projection("p", 256, 256, 0)],
        ranks=np.asarray([4, 8, 8, 16], np.int32),
        adapter_ids=np.asarray([11, 22, 33, 44], np.int64),
        alpha=np.ones(4, np.float32),
        scale=2.0,
        seg_offsets=np.asarray([0, 1, 4, 9, 16], np.int32),
        seg_adapter=np.asarray([0, 1, 2, 3], np.int32),
        note="base_out is x.W with W from base_weight(0)",
    )


def decode(seed: int = 0, n_layers: int = 1) -> Instance:
    """64 decode tokens, 4096->4096 bf16, pool of 100, Zipf(1.0)."""
    return make_instance(
        "decode", dtype="bf16", seed=seed, projs=[Projection("q", 4096, 4096, 0)], n_adapters=100,
        rank_choices=[8, 16, 32, 64, 128], n_decode=64, prompt_lens=[], zipf_alpha=1.0, n_layers=n_layers,
    )


def decode_heavy(seed: int = 0, n_layers: int = 1) -> Instance:
    """Not one of the task's configurations: the decode configuration at the size of a loaded
    server -- 1024 decode tokens, 4096->4096 bf16, pool of 500, Zipf(1.0) -- where one launch moves
    enough bytes for the bandwidth roof, not launch latency, to be what binds."""
    return make_instance(
        "decode_heavy", dtype="bf16", seed=seed, projs=[Projection("q", 4096, 4096, 0)], n_adapters=500,
        rank_choices=[8, 16, 32, 64, 128], n_decode=1024, prompt_lens=[], zipf_alpha=1.0, n_layers=n_layers,
    )


def decode_qkv(seed: int = 0, n_layers: int = 1, n_decode: int = 64) -> Instance:
    """Not one of the task's configurations: the decode configuration's batch and pool on the three
    projections q, k, v of the layer, which read the same activations (section 3.1: the adapter
    work of a layer is that of all its adapted projections) -- what a serving iteration hands to the
    library as one group."""
    return make_instance(
        "decode_qkv", dtype="bf16", seed=seed, projs=[Projection(n, 4096, 4096, 0) for n in ("q", "k", "v")], n_adapters=100,
        rank_choices=[8, 16, 32, 64, 128], n_decode=n_decode, prompt_lens=[], zipf_alpha=1.0, n_layers=n_layers,
    )


def decode_paper(seed: int = 0, n_layers: int = 1, n_adapters: int = 100, n_decode: int = 64) -> Instance:
    """Not one of the task's configurations: the decode configuration with the paper's own adapter
    population (section 5.1: N_a adapters, N_a / 5 of each of the five ranks, rank drawn uniformly,
    power law within the rank) -- for the sweep over N_a = 10 .. 200 of the paper's sensitivity study."""
    return make_instance(
        f"decode_paper_{n_adapters}", dtype="bf16", seed=seed, projs=[Projection("q", 4096, 4096, 0)], n_adapters=n_adapters,
        rank_choices=[8, 16, 32, 64, 128], n_decode=n_decode, prompt_lens=[], zipf_alpha=1.0, n_layers=n_layers,
        popularity_within_rank=True,
    )


def prefill(seed: int = 0, n_layers: int = 1) -> Instance:
    """8 prompts, lognormal(6, 0.8) lengths in [32, 2048], distinct adapters of rank {16,64,128}."""
    lens = _prompt_lengths(_rng(seed, _P_LEN), 8)
    return make_instance(
        "prefill", dtype="bf16", seed=seed, projs=[Projection("q", 4096, 4096, 0)], n_adapters=100,
        rank_choices=[8, 16, 32, 64, 128], n_decode=0, prompt_lens=lens, zipf_alpha=None,
        distinct_prefill_adapters=True, prefill_rank_choices=[16, 64, 128], n_layers=n_layers,
    )


def mixed(seed: int = 0, n_layers: int = 1) -> Instance:
    """Full 7B-shaped layer (7 projections), 224 decode + 32 prompts, pool of 500, Zipf(1.2)."""
    lens = _prompt_lengths(_rng(seed, _P_LEN), 32)
    return make_instance(
        "mixed", dtype="bf16", seed=seed, projs=_llama_projs(4096, 11008), n_adapters=500,
        rank_choices=[8, 16, 32, 64, 128], n_decode=224, prompt_lens=lens, zipf_alpha=1.2, n_layers=n_layers,
    )


def stress(seed: int = 0, n_layers: int = 4) -> Instance:
    """13B-shaped layer, pool of 1000 in 4 layer copies (~39 GB), 512 decode + 4x512 prompt tokens, 10 % misses."""
    return make_instance(
        "stress", dtype="bf16", seed=seed, projs=_llama_projs(5120, 13824), n_adapters=1000,
        rank_choices=[8, 16, 32, 64, 128], n_decode=512, prompt_lens=[512] * 4, zipf_alpha=1.2,
        n_layers=n_layers, miss_fraction=0.10,
    )


def small_mixed(seed: int = 0, dtype: str = "bf16") -> Instance:
    """Small instance that still reaches every code path: decode tokens, short and long
    prompts with ragged tails, a hot adapter shared by many decode tokens, base-only
    requests, and two projection shapes.  Sized for the oracle to finish in seconds."""
    lens = [3, 17, 64, 100, 7, 129]
    projs = [Projection("a", 512, 384, 0), Projection("b", 384, 512, 1)]
    return make_instance(
        "small_mixed", dtype=dtype, seed=seed, projs=projs, n_adapters=12,
        rank_choices=[8, 16, 32, 64, 128], n_decode=40, prompt_lens=lens, zipf_alpha=1.5, n_base_only=3,
    )


CONFIGS = {
    "tiny": tiny,
    "decode": decode,
    "prefill": prefill,
    "mixed": mixed,
    "stress": stress,
    "small_mixed": small_mixed,
    "decode_heavy": decode_heavy,
    "decode_paper": decode_paper,
    "decode_qkv": decode_qkv,
}
