"""Pins for the oracle's indexer: a hand-worked batch and properties that hold for any batch."""
import numpy as np

import oracle
import workloads as wl


def test_handworked_index():
    # 5 requests: 2 decode tokens on slot 7 (rank 8), a 3-token prompt on slot 2 (rank 16),
    # a base-only token, an empty segment, and a 5-token prompt on slot 7.  M0 = 4, tiles of 4.
    off = [0, 1, 4, 5, 5, 6, 11]
    slot = [7, 2, -1, 3, 7, 7]
    rank = [8, 16, 0, 32, 8, 8]
    w = oracle.index(11, off, slot, rank, mfma_min_tokens=4, tile_tokens=4)
    # long segment: tokens 6..10 on slot 7 -> tiles (6,7,8,9) and (10); pooled: slot 2 -> 1,2,3; slot 7 -> 0,5
    assert w["tok_list"] == [6, 7, 8, 9, 10, 1, 2, 3, 0, 5]
    assert w["tiles"] == [(0, 4, 7, 8, 0, 0), (4, 1, 7, 8, 1, 0)]
    assert w["groups"] == [(5, 3, 2, 16, 0, 0), (8, 2, 7, 8, 0, 0)]
    # six decode tokens of one slot stay one group below the threshold and become a gathered tile at it
    w = oracle.index(6, [0, 1, 2, 3, 4, 5, 6], [9] * 6, [8] * 6, mfma_min_tokens=16)
    assert w["groups"] == [(0, 6, 9, 8, 0, 0)] and w["tiles"] == []
    w = oracle.index(6, [0, 1, 2, 3, 4, 5, 6], [9, 4, 9, 9, 4, 9], [8, 32, 8, 8, 32, 8], mfma_min_tokens=4)
    assert w["tiles"] == [(0, 4, 9, 8, 0, 0)] and w["groups"] == [(4, 2, 4, 32, 0, 0)] and w["tok_list"] == [0, 2, 3, 5, 1, 4]
    ts, tr = oracle.token_map(11, off, slot, rank)
    assert ts == [7, 2, 2, 2, -1, 7, 7, 7, 7, 7, 7]
    assert tr == [8, 16, 16, 16, 0, 8, 8, 8, 8, 8, 8]


def _check_cover(inst, m0):
    slot = np.where(inst.seg_adapter >= 0, inst.seg_adapter + 100, -1)  # any injective slot naming
    w = oracle.index(inst.T, inst.seg_offsets, slot, inst.seg_rank, m0)
    ts, tr = oracle.token_map(inst.T, inst.seg_offsets, slot, inst.seg_rank)
    seen = np.zeros(inst.T, np.int32)
    for (o, n, s, r, _, _) in w["tiles"] + w["groups"]:
        assert 1 <= n and (n <= 64 or (o, n, s, r, 0, 0) in w["groups"])
        for t in w["tok_list"][o : o + n]:
            seen[t] += 1
            assert ts[t] == s and tr[t] == r
    active = np.array(ts) >= 0
    assert np.array_equal(seen, active.astype(np.int32))
    assert sorted(w["tok_list"]) == list(np.flatnonzero(active))
    for (o, n, s, r, _, _) in w["groups"]:
        assert m0 == 0 or n < m0
    for (o, n, s, r, k, _) in w["tiles"]:
        assert m0 > 0 and 1 <= n <= 64
    return w


def test_every_active_token_exactly_once():
    for name in ("tiny", "decode", "prefill", "small_mixed", "stress"):
        inst = wl.CONFIGS[name]()
        for m0 in (0, 16):
            w = _check_cover(inst, m0)
            if m0 == 0:
                assert w["tiles"] == []


def test_decode_batch_groups_tokens_by_slot():
    inst = wl.decode()
    w = _check_cover(inst, 16)
    assert len(w["groups"]) + len({s for (_, _, s, _, _, _) in w["tiles"]}) == len(inst.used_adapters())
    slots = [s for (_, _, s, _, _, _) in w["groups"]]
    assert slots == sorted(slots) and len(set(slots)) == len(slots)
