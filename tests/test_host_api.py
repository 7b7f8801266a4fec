"""CPU-only checks of the C ABI: the library loads and exports what the header declares, the
indexer equals the oracle's indexer bit for bit, byte accounting, slot-table state machine,
argument validation.  No kernel is launched here."""
import os
import re

import numpy as np
import pytest

import oracle
import workloads as wl
from paper_2411_17741_amd import binding as B

INCLUDE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")


def _declared_functions():
    names = set()
    for header in sorted(os.listdir(INCLUDE)):
        if header.endswith(".h"):
            src = open(os.path.join(INCLUDE, header)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names |= set(re.findall(r"\b(lora_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(B._lib, n), f"{n} declared in include/ but not exported"
    assert sorted(B.EXPORTS) == names


# ---------------------------------------------------------------------------------------
def _index_both(T, off, slot, rank, m0):
    rc, got = B.lora_index(T, off, slot, rank, m0)
    assert rc == B.LORA_OK
    want = oracle.index(T, off, slot, rank, m0)
    for k in ("tok_list", "tiles", "groups"):
        assert got[k] == [tuple(v) if not isinstance(v, int) else v for v in want[k]], k


@pytest.mark.parametrize("name", ["tiny", "decode", "prefill", "small_mixed", "stress", "mixed"])
@pytest.mark.parametrize("m0", [0, 16])
def test_indexer_matches_oracle_on_configs(name, m0):
    inst = wl.CONFIGS[name]()
    slot = np.where(inst.seg_adapter >= 0, inst.seg_adapter * 3 + 1, -1)
    _index_both(inst.T, inst.seg_offsets, slot, inst.seg_rank, m0)


def test_indexer_matches_oracle_on_random_batches():
    rng = np.random.default_rng(0)
    for trial in range(200):
        n_seg = int(rng.integers(0, 40))
        lens = rng.choice([0, 1, 1, 1, 2, 5, 15, 16, 17, 63, 64, 65, 130], size=n_seg)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        n_slots = int(rng.integers(1, 12))
        slot_rank = rng.choice([1, 4, 8, 12, 16, 24, 32, 40, 64, 100, 128], size=n_slots)
        slot = rng.integers(-1, n_slots, size=n_seg).astype(np.int32)
        rank = np.where(slot >= 0, slot_rank[np.maximum(slot, 0)], 0).astype(np.int32)
        m0 = int(rng.choice([0, 1, 8, 16, 64]))
        _index_both(int(off[-1]), off, slot, rank, m0)


# ---------------------------------------------------------------------------------------
# The lists the kernels read (lora_plan_dump of a host-only cache: the staged copy of the plan), checked
# against the oracle's token map through coverage properties -- no kernel item shape is restated here.
def _host_plan_check(T, off, slot_of_seg, rank, projs, dtype=B.LORA_BF16, m0=0, seed=0):
    from plan_checks import check_plan_units

    slot_of_seg = np.asarray(slot_of_seg, np.int32)
    rank = np.asarray(rank, np.int32)
    # one slot per distinct name, in a pool of one class per distinct storage size; alpha differs per slot
    names = sorted({int(s) for s in slot_of_seg if s >= 0})
    name_rank = {int(s): int(r) for s, r in zip(slot_of_seg, rank) if s >= 0}
    class_rank = [8, 16, 32, 64, 128]
    cls_of = lambda r: next(i for i, c in enumerate(class_rank) if c >= r)
    class_slots = [0] * 5
    for n in names:
        class_slots[cls_of(name_rank[n])] += 1
    class_slots = [c + 1 for c in class_slots]  # a spare slot per class, left empty
    first = np.concatenate([[0], np.cumsum(class_slots)[:-1]])
    nxt = list(first)
    real = {}
    for n in names:
        k = cls_of(name_rank[n])
        real[n] = int(nxt[k])
        nxt[k] += 1
    cfg = B.make_config(projs, 1, class_rank, class_slots, dtype, max(1, T), max(1, len(slot_of_seg)), mfma_min_tokens=m0,
                        flags=B.LORA_CACHE_HOST_ONLY)
    rc, h = B.lora_cache_create(cfg, 0, 0)
    assert rc == B.LORA_OK
    alpha = {}
    for n in names:
        alpha[real[n]] = 0.5 + 0.25 * (real[n] % 7)
        for p in range(len(projs)):
            assert B.lora_cache_fill_slot(h, real[n], 1000 + n, name_rank[n], alpha[real[n]], 0, p, 0, 0) == B.LORA_OK
    seg_slot = np.array([real[int(s)] if s >= 0 else -1 for s in slot_of_seg], np.int32)
    rc, plan = B.lora_plan_create(h, T, off, seg_slot, rank)
    assert rc == B.LORA_OK
    counts = check_plan_units(h, plan, T, off, seg_slot, rank, projs, alpha, bf16=dtype == B.LORA_BF16)
    assert B.lora_plan_destroy(h, plan) == B.LORA_OK
    assert B.lora_cache_destroy(h) == B.LORA_OK
    return counts


@pytest.mark.parametrize("name", ["tiny", "decode", "prefill", "small_mixed", "stress", "mixed"])
def test_plan_work_units_cover_every_token_row_and_column_once(name):
    inst = wl.CONFIGS[name]()
    projs = [(p.h_in, p.h_out) for p in inst.projs]
    dtype = B.LORA_BF16 if inst.dtype == "bf16" else B.LORA_F32
    for m0 in (0, 16):  # the library's own choice of the threshold, and a fixed one
        counts = _host_plan_check(inst.T, inst.seg_offsets, inst.seg_adapter, inst.seg_rank, projs, dtype, m0)
        assert counts[0]["gemv_shrink"] + counts[0]["tiles"] > 0


def test_plan_work_units_on_random_batches():
    rng = np.random.default_rng(1)
    for trial in range(60):
        n_seg = int(rng.integers(0, 40))
        lens = rng.choice([0, 1, 1, 1, 2, 3, 5, 9, 15, 16, 17, 63, 64, 65, 130], size=n_seg)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        n_names = int(rng.integers(1, 12))
        name_rank = rng.choice([1, 3, 4, 8, 12, 16, 24, 32, 40, 64, 100, 128], size=n_names)
        slot = rng.integers(-1, n_names, size=n_seg).astype(np.int32)
        rank = np.where(slot >= 0, name_rank[np.maximum(slot, 0)], 0).astype(np.int32)
        projs = [(64 * int(rng.integers(1, 5)), 64 * int(rng.choice([1, 2, 15, 16, 17, 33]))) for _ in range(int(rng.integers(1, 4)))]
        _host_plan_check(int(off[-1]), off, slot, rank, projs, B.LORA_BF16, int(rng.choice([0, 1, 8, 16, 64])))


def test_plan_tile_shrink_pieces_on_random_prompt_batches():
    """Wide inputs and long segments: tiles are worked on in pieces, with cuts inside tiles (checked by check_plan_units)."""
    rng = np.random.default_rng(7)
    in_pieces = 0
    for trial in range(12):
        n_seg = int(rng.integers(1, 14))
        lens = rng.choice([1, 3, 40, 64, 65, 128, 200, 513, 1000], size=n_seg)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        n_names = int(rng.integers(1, 6))
        name_rank = rng.choice([8, 16, 32, 64, 100, 128], size=n_names)
        slot = rng.integers(-1, n_names, size=n_seg).astype(np.int32)
        rank = np.where(slot >= 0, name_rank[np.maximum(slot, 0)], 0).astype(np.int32)
        widths = [int(w) for w in rng.choice([1024, 1536, 2048, 4096, 5120], size=int(rng.integers(1, 3)))]
        projs = [(w, 64 * int(rng.choice([1, 16, 17]))) for w in widths]
        counts = _host_plan_check(int(off[-1]), off, slot, rank, projs, B.LORA_BF16, int(rng.choice([0, 16])))
        in_pieces += counts[0]["tile_partial_sums"] > 0
    assert in_pieces >= 6


def test_slot_state_call():
    h = _host_cache()
    assert B.lora_cache_slot_state(h, 2) == (B.LORA_OK, B.LORA_SLOT_EMPTY)
    assert B.lora_cache_fill_slot(h, 2, 77, 16, 0.5, 0, 0, 0, 0) == B.LORA_OK
    assert B.lora_cache_slot_state(h, 2) == (B.LORA_OK, B.LORA_SLOT_FILLING)
    for l, p in [(0, 1), (1, 0), (1, 1)]:
        assert B.lora_cache_fill_slot(h, 2, 77, 16, 0.5, l, p, 0, 0) == B.LORA_OK
    assert B.lora_cache_slot_state(h, 2) == (B.LORA_OK, B.LORA_SLOT_READY)
    assert B.lora_cache_release_slot(h, 2) == B.LORA_OK
    assert B.lora_cache_slot_state(h, 2) == (B.LORA_OK, B.LORA_SLOT_EMPTY)
    assert B.lora_cache_slot_state(h, 9)[0] == B.LORA_E_INVAL
    assert B.lora_cache_destroy(h) == B.LORA_OK


def test_indexer_rejects_malformed_batches():
    ok = dict(T=4, off=[0, 2, 4], slot=[0, 1], rank=[8, 16])
    assert B.lora_index(ok["T"], ok["off"], ok["slot"], ok["rank"], 16)[0] == B.LORA_OK
    bad = [
        (4, [1, 2, 4], [0, 1], [8, 16]),      # does not start at 0
        (4, [0, 2, 3], [0, 1], [8, 16]),      # does not end at T
        (4, [0, 3, 2, 4], [0, 1, 0], [8, 16, 8]),  # decreasing
        (4, [0, 2, 4], [0, 1], [8, 0]),       # rank 0 on an active segment
        (4, [0, 2, 4], [0, 1], [8, 129]),     # rank above the maximum
        (4, [0, 2, 4], [0, 0], [8, 16]),      # one slot, two ranks
    ]
    for T, off, slot, rank in bad:
        assert B.lora_index(T, off, slot, rank, 16)[0] == B.LORA_E_INVAL
    # empty batch and batch without adapters are fine
    rc, w = B.lora_index(0, [0], [], [], 16)
    assert rc == B.LORA_OK and w["tok_list"] == []
    rc, w = B.lora_index(3, [0, 3], [-1], [0], 16)
    assert rc == B.LORA_OK and w["tok_list"] == [] and w["tiles"] == [] and w["groups"] == []


# ---------------------------------------------------------------------------------------
def test_adapter_bytes_match_the_papers_footprint():
    """Section 3.2: a rank-32 adapter of Llama-7B (q,k,v,o x 32 layers, 16 bit) takes 64 MB;
    the Llama-70B one (k,v are 8192->1024) about 256 MB."""
    per_proj = B.lora_adapter_bytes(4096, 4096, 32, B.LORA_BF16)
    assert per_proj * 4 * 32 == 64 * 1024 * 1024
    b70 = (2 * B.lora_adapter_bytes(8192, 8192, 32, B.LORA_BF16) + 2 * B.lora_adapter_bytes(8192, 1024, 32, B.LORA_BF16)) * 80
    assert abs(b70 / 2**20 - 250) < 1
    assert B.lora_adapter_bytes(4096, 4096, 0, B.LORA_BF16) == 0
    assert B.lora_adapter_bytes(4096, 4096, 8, 7) == 0


def test_pool_bytes_account_for_every_slab():
    proj = [(4096, 4096)] * 4
    cfg = B.make_config(proj, 32, [8, 16, 32, 64, 128], [0, 0, 1, 0, 0], B.LORA_BF16, 64, 64)
    cfg0 = B.make_config(proj, 32, [8, 16, 32, 64, 128], [0, 0, 2, 0, 0], B.LORA_BF16, 64, 64)
    one, two = B.lora_cache_bytes_required(cfg), B.lora_cache_bytes_required(cfg0)
    # adding one rank-32 slot to a 7B-shaped q,k,v,o pool of 32 layers adds exactly the 64 MiB of section 3.2
    # (plus 8 bytes per projection in the offset table, rounded to the 256-byte granule)
    assert 0 <= (two - one) - 64 * 1024 * 1024 <= 256
    assert B.lora_cache_bytes_required(B.make_config(proj, 0, [8], [1], B.LORA_BF16, 64, 64)) == 0
    assert B.lora_cache_bytes_required(B.make_config([(100, 64)], 1, [8], [1], B.LORA_BF16, 64, 64)) == 0  # h_in % 64
    assert B.lora_cache_bytes_required(B.make_config(proj, 1, [16, 8], [1, 1], B.LORA_BF16, 64, 64)) == 0  # not increasing
    assert B.lora_cache_bytes_required(B.make_config(proj, 1, [256], [1], B.LORA_BF16, 64, 64)) == 0  # above LORA_MAX_RANK


def _host_cache(n_layers=2, n_proj=2, class_slots=(2, 1)):
    cfg = B.make_config([(64, 128)] * n_proj, n_layers, [8, 32], list(class_slots), B.LORA_BF16, 64, 16, flags=B.LORA_CACHE_HOST_ONLY)
    rc, h = B.lora_cache_create(cfg, 0, 0)
    assert rc == B.LORA_OK
    return h


def test_slot_table_state_machine():
    """Cache-entry life cycle of section 4.2: load a missing adapter, look it up, count
    references, never evict or overwrite an entry that running requests use."""
    h = _host_cache()
    st = lambda s: B.lora_cache_slot_info(h, s)[1]
    assert st(0).state == B.LORA_SLOT_EMPTY
    assert B.lora_cache_lookup(h, 77)[0] == B.LORA_E_NOTFOUND
    # rank must fit the class of the slot (slots 0,1: class 8; slot 2: class 32)
    assert B.lora_cache_fill_slot(h, 0, 77, 16, 1.0, 0, 0, 0, 0) == B.LORA_E_INVAL
    assert B.lora_cache_find_free_slot(h, 16) == (B.LORA_OK, 2)
    assert B.lora_cache_find_free_slot(h, 4) == (B.LORA_OK, 0)
    assert B.lora_cache_find_free_slot(h, 33)[0] == B.LORA_E_NOMEM
    # four parts (2 layers x 2 projections): FILLING until the last one
    for i, (l, p) in enumerate([(0, 0), (0, 1), (1, 0), (1, 1)]):
        assert B.lora_cache_fill_slot(h, 2, 77, 16, 0.5, l, p, 0, 0) == B.LORA_OK
        info = st(2)
        assert info.parts_filled == i + 1
        assert info.state == (B.LORA_SLOT_READY if i == 3 else B.LORA_SLOT_FILLING)
    info = st(2)
    assert (info.adapter_id, info.rank, info.class_rank, info.alpha) == (77, 16, 32, 0.5)
    assert B.lora_cache_lookup(h, 77) == (B.LORA_OK, 2, 16)
    # the same adapter cannot be cached twice; a bound slot cannot take another adapter
    assert B.lora_cache_fill_slot(h, 0, 77, 8, 0.5, 0, 0, 0, 0) == B.LORA_E_STATE
    assert B.lora_cache_fill_slot(h, 2, 78, 16, 0.5, 0, 0, 0, 0) == B.LORA_E_STATE
    # reference counting: referenced entries can be neither evicted nor overwritten
    assert B.lora_cache_slot_ref(h, 2, +1) == B.LORA_OK
    assert B.lora_cache_release_slot(h, 2) == B.LORA_E_STATE
    assert B.lora_cache_fill_slot(h, 2, 77, 16, 0.5, 0, 0, 0, 0) == B.LORA_E_STATE
    assert B.lora_cache_slot_ref(h, 2, -1) == B.LORA_OK
    assert B.lora_cache_slot_ref(h, 2, -1) == B.LORA_E_STATE
    assert B.lora_cache_slot_ref(h, 0, +1) == B.LORA_E_STATE  # empty slot
    assert B.lora_cache_fill_slot(h, 2, 77, 16, 0.5, 0, 0, 0, 0) == B.LORA_OK  # unreferenced refill is allowed
    # eviction discards (no write-back), the id is forgotten, the slot can be rebound
    assert B.lora_cache_release_slot(h, 2) == B.LORA_OK
    assert st(2).state == B.LORA_SLOT_EMPTY
    assert B.lora_cache_lookup(h, 77)[0] == B.LORA_E_NOTFOUND
    assert B.lora_cache_fill_slot(h, 2, 78, 32, 1.0, 0, 0, 0, 0) == B.LORA_OK
    rc, stats = B.lora_cache_stats(h)
    assert (stats.hits, stats.misses, stats.evictions, stats.fills) == (1, 2, 1, 6)
    # out-of-range arguments
    assert B.lora_cache_fill_slot(h, 3, 1, 8, 1.0, 0, 0, 0, 0) == B.LORA_E_INVAL
    assert B.lora_cache_fill_slot(h, 0, 1, 8, 1.0, 2, 0, 0, 0) == B.LORA_E_INVAL
    assert B.lora_cache_fill_slot(h, 0, 1, 8, 1.0, 0, 2, 0, 0) == B.LORA_E_INVAL
    assert B.lora_cache_release_slot(h, -1) == B.LORA_E_INVAL
    assert B.lora_cache_slot_info(h, 9)[0] == B.LORA_E_INVAL
    # no device work on a host-only cache
    assert B.lora_apply(h, 0, 0, 0, 0, 0, [0], [], [], 1.0) == B.LORA_E_INVAL
    assert B.lora_cache_destroy(h) == B.LORA_OK


def test_fill_of_several_parts_in_one_call():
    """lora_cache_fill_slot_parts: the slot table moves as if the parts had come one by one; a call with a
    bad part changes nothing."""
    h = _host_cache()
    st = lambda s: B.lora_cache_slot_info(h, s)[1]
    parts = B.make_fill_parts([(0, 0, 0, 0), (0, 1, 0, 0), (1, 0, 0, 0)])
    assert B.lora_cache_fill_slot_parts(h, 2, 77, 16, 0.5, parts) == B.LORA_OK
    assert (st(2).parts_filled, st(2).state, st(2).adapter_id, st(2).rank) == (3, B.LORA_SLOT_FILLING, 77, 16)
    assert B.lora_cache_fill_slot_parts(h, 2, 77, 16, 0.5, B.make_fill_parts([(1, 1, 0, 0)])) == B.LORA_OK
    assert st(2).state == B.LORA_SLOT_READY
    assert B.lora_cache_lookup(h, 77) == (B.LORA_OK, 2, 16)
    # errors leave the slot as it was
    assert B.lora_cache_fill_slot_parts(h, 0, 5, 8, 1.0, B.make_fill_parts([(0, 0, 0, 0), (2, 0, 0, 0)])) == B.LORA_E_INVAL  # layer
    assert B.lora_cache_fill_slot_parts(h, 0, 5, 8, 1.0, B.make_fill_parts([(0, 0, 0, 0), (0, 2, 0, 0)])) == B.LORA_E_INVAL  # projection
    assert st(0).state == B.LORA_SLOT_EMPTY and B.lora_cache_lookup(h, 5)[0] == B.LORA_E_NOTFOUND
    assert B.lora_cache_fill_slot_parts(h, 0, 5, 16, 1.0, parts) == B.LORA_E_INVAL       # rank above the slot's class
    assert B.lora_cache_fill_slot_parts(h, 0, 77, 8, 0.5, parts) == B.LORA_E_STATE      # cached elsewhere
    assert B.lora_cache_fill_slot_parts(h, 2, 78, 16, 0.5, parts) == B.LORA_E_STATE     # bound to another adapter
    assert B.lora_cache_slot_ref(h, 2, +1) == B.LORA_OK
    assert B.lora_cache_fill_slot_parts(h, 2, 77, 16, 0.5, parts) == B.LORA_E_STATE     # in use and complete
    assert B.lora_cache_slot_ref(h, 2, -1) == B.LORA_OK
    assert B.lora_cache_fill_slot_parts(h, 2, 77, 16, 0.5, parts) == B.LORA_OK
    assert B.lora_cache_fill_slot_parts(h, 0, 5, 8, 1.0, B.make_fill_parts([])) == B.LORA_OK and st(0).state == B.LORA_SLOT_EMPTY
    rc, stats = B.lora_cache_stats(h)
    assert stats.fills == 7
    assert B.lora_cache_destroy(h) == B.LORA_OK


def test_plan_validation_against_slot_table():
    h = _host_cache(n_layers=1, n_proj=1)
    assert B.lora_cache_fill_slot(h, 0, 5, 8, 1.0, 0, 0, 0, 0) == B.LORA_OK
    mk = lambda T, off, slot, rank: B.lora_plan_create(h, T, off, slot, rank)[0]
    assert mk(3, [0, 3], [0], [8]) == B.LORA_OK
    assert mk(3, [0, 3], [0], [4]) == B.LORA_E_INVAL    # rank differs from the cached adapter's
    assert mk(3, [0, 3], [1], [8]) == B.LORA_E_STATE    # empty slot
    assert mk(3, [0, 3], [3], [8]) == B.LORA_E_INVAL    # no such slot
    assert mk(65, [0, 65], [0], [8]) == B.LORA_E_INVAL  # more tokens than max_tokens
    assert mk(3, [0, 2], [0], [8]) == B.LORA_E_INVAL
    assert mk(3, [0, 3], [0], [8]) == B.LORA_OK
    assert mk(3, [0, 3], [0], [8]) == B.LORA_E_NOMEM    # both user plans taken
    assert B.lora_cache_destroy(h) == B.LORA_OK


def test_create_rejects_bad_arguments():
    cfg = B.make_config([(64, 64)], 1, [8], [1], B.LORA_BF16, 16, 4)
    assert B.lora_cache_create(cfg, 0, 0)[0] == B.LORA_E_INVAL         # device pool required
    assert B.lora_cache_create(cfg, 0x1001, 1 << 30)[0] == B.LORA_E_INVAL  # misaligned
    assert B.lora_cache_create(cfg, 0x1000, 16)[0] == B.LORA_E_NOMEM   # too small
    assert B.lora_strerror(B.LORA_E_STATE) != B.lora_strerror(B.LORA_E_INVAL)
