"""Shared by CPU and GPU tests: properties the work units of a plan must have, whatever shape the
kernels give their work items.

`lora_plan_dump` returns the units decoded from the buffer the kernels read.  The slot/segment
indexing is right exactly when these units, taken together, say for every token what the
oracle's `token_map` says (which slot, which rank) and cover the work once:

* tile units: the tokens, slot and rank of the oracle's tiles, tile by tile (the tile/group
  partition under the plan's threshold is part of the library's contract);
* GEMV units: their tokens are the tokens of the oracle's groups; per token the shrink units cover
  rank rows [0, rank) exactly once (rows of the zero padding up to the next multiple of 8 at most
  once) and, per projection, the expand units cover columns [0, h_out) exactly once;
* row units of the fused linear path: every token of the batch exactly once.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2411_17741_amd import binding as B


def check_plan_units(cache, plan, T, seg_offsets, seg_slot, seg_rank, projs, alpha_of_slot, bf16=True):
    """projs: [(h_in, h_out)]; alpha_of_slot: dict slot -> alpha.  Returns a dict of counts."""
    rc, info = B.lora_plan_info(plan)
    assert rc == B.LORA_OK
    tm_slot, tm_rank = (np.asarray(v, np.int64) for v in oracle.token_map(T, seg_offsets, seg_slot, seg_rank))
    want = oracle.index(T, seg_offsets, seg_slot, seg_rank, info.mfma_min_tokens)
    want_tile_toks = [want["tok_list"][o : o + n] for (o, n, *_r) in want["tiles"]]
    want_gemv = sorted(t for (o, n, *_r) in want["groups"] for t in want["tok_list"][o : o + n])
    gemv_pos = {t: i for i, t in enumerate(want_gemv)}
    counts = {}
    for p, (h_in, h_out) in enumerate(projs):
        rc, units, toks = B.lora_plan_dump(cache, plan, p)
        assert rc == B.LORA_OK
        assert (units["tok_off"] >= 0).all() and (units["tok_off"] + units["n_tok"] <= len(toks)).all()
        assert ((toks >= 0) & (toks < T)).all()
        toks_of = lambda u: toks[u["tok_off"] : u["tok_off"] + u["n_tok"]]

        def same_entry(u):
            tk = toks_of(u)
            assert u["n_tok"] >= 1
            assert (tm_slot[tk] == u["slot"]).all() and (tm_rank[tk] == u["rank"]).all(), (u, tk)
            assert u["alpha"] == np.float32(alpha_of_slot[int(u["slot"])])

        # --- tiles: the oracle's, in order
        tiles = units[units["kind"] == B.LORA_UNIT_TILE]
        assert len(tiles) == len(want["tiles"]) == info.n_tiles
        for u, wt, (_, _, slot, rank, _, _) in zip(tiles, want_tile_toks, want["tiles"]):
            assert list(toks_of(u)) == wt and (u["slot"], u["rank"]) == (slot, rank)
            assert 1 <= u["n_tok"] <= B.LORA_TILE_TOKENS
            same_entry(u)

        # --- tile shrink: under every run table the pieces of a tile cover its input columns [0, h_in) once, in pieces
        # of whole 128-column stages; runs are walked in order, each at most a tail, whole tiles and a head; pieces that
        # are not whole tiles leave partial sums in slots of their own, and the reduce adds up exactly those
        pieces = units[units["kind"] == B.LORA_UNIT_TILE_SHRINK]
        sums = units[units["kind"] == B.LORA_UNIT_TILE_SUM]
        tile_of_off = {int(u["tok_off"]): i for i, u in enumerate(tiles)}
        for table in range(5):
            pc = pieces[(pieces["where"] >> 20) == table]
            sm = sums[(sums["where"] >> 20) == table]
            if len(tiles) == 0 or (table == 4 and T > B.LORA_STATIC_MAX_TOKENS):  # (no table for what the call refuses)
                assert len(pc) == 0 and len(sm) == 0
                continue
            runs = pc["where"] & 0xFFFFF
            assert (np.diff(runs) >= 0).all() and runs.max() < 512 // (1 if table == 4 else table + 1)
            if table == 4:
                assert runs.max() < 128
            cover = np.zeros((len(tiles), h_in), np.int8)
            slots_of_tile = [[] for _ in tiles]
            order = []
            for u in pc:
                i = tile_of_off[int(u["tok_off"])]
                assert (u["n_tok"], u["slot"], u["rank"]) == (tiles[i]["n_tok"], tiles[i]["slot"], tiles[i]["rank"])
                assert 0 <= u["lo"] < u["hi"] <= h_in and u["lo"] % 128 == 0 and (u["hi"] % 128 == 0 or u["hi"] == h_in)
                cover[i, u["lo"] : u["hi"]] += 1
                whole = u["lo"] == 0 and u["hi"] == h_in
                assert (u["alpha"] == -1) == whole
                if not whole:
                    assert u["hi"] - u["lo"] >= min(256, h_in // 2), u  # no slivers
                    slots_of_tile[i].append(int(u["alpha"]))
                order.append((i, int(u["lo"])))
            assert (cover == 1).all()
            assert order == sorted(order)  # the runs walk the tiles' columns in order
            all_slots = [s for l in slots_of_tile for s in l]
            assert len(set(all_slots)) == len(all_slots) and all(0 <= s < 2 * (int(runs.max()) + 1) for s in all_slots)
            for r in np.unique(runs):  # a run leaves at most two partial sums
                assert (pc[runs == r]["alpha"] >= 0).sum() <= 2
            got = [[] for _ in tiles]
            for u in sm:
                i = tile_of_off[int(u["tok_off"])]
                assert u["lo"] == len(got[i]) and u["hi"] == len(slots_of_tile[i])
                got[i].append(int(u["alpha"]))
            assert got == slots_of_tile

        # --- GEMV shrink: every (token, rank row) once
        gs = units[units["kind"] == B.LORA_UNIT_GEMV_SHRINK]
        cover = np.zeros((len(want_gemv), B.LORA_MAX_RANK), np.int32)
        for u in gs:
            same_entry(u)
            assert 0 <= u["lo"] < u["hi"] <= (u["rank"] + 7) // 8 * 8
            idx = [gemv_pos[int(t)] for t in toks_of(u)]  # KeyError: a token that is not on the GEMV path
            assert len(set(idx)) == len(idx)
            cover[idx, u["lo"] : u["hi"]] += 1
        for i, t in enumerate(want_gemv):
            r = tm_rank[t]
            assert (cover[i, :r] == 1).all() and (cover[i, r:] <= 1).all() and (cover[i, (r + 7) // 8 * 8 :] == 0).all(), t
        assert sorted(gs["where"]) == list(range(len(gs)))

        # --- GEMV expand: every (token, output column) once
        ge = units[units["kind"] == B.LORA_UNIT_GEMV_EXPAND]
        cover = np.zeros((len(want_gemv), h_out), np.int8)
        for u in ge:
            same_entry(u)
            assert 0 <= u["lo"] < u["hi"] <= h_out
            idx = [gemv_pos[int(t)] for t in toks_of(u)]
            assert len(set(idx)) == len(idx)
            cover[idx, u["lo"] : u["hi"]] += 1
        assert (cover == 1).all()

        # --- rows of the fused linear path: every token once, adapter tokens where the other lists have them
        lin = units[units["kind"] == B.LORA_UNIT_LINEAR_ROWS]
        if bf16:
            seen = np.zeros(T, np.int32)
            for u in lin:
                np.add.at(seen, toks_of(u), 1)
                assert 1 <= u["n_tok"] <= B.LORA_TILE_TOKENS
            assert (seen == 1).all()
            lt = lin[lin["where"] == 2]
            assert len(lt) == len(tiles)
            for u, v in zip(lt, tiles):
                assert list(toks_of(u)) == list(toks_of(v)) and (u["slot"], u["rank"], u["alpha"]) == (v["slot"], v["rank"], v["alpha"])
            g_rows = sorted(int(t) for u in lin[lin["where"] == 1] for t in toks_of(u))
            assert g_rows == want_gemv
            for u in lin[lin["where"] == 0]:
                assert (tm_slot[toks_of(u)] == -1).all()
        else:
            assert len(lin) == 0
        counts[p] = {"tiles": len(tiles), "gemv_shrink": len(gs), "gemv_expand": len(ge), "linear_rows": len(lin),
                     "tile_partial_sums": int((pieces["alpha"] >= 0).sum())}
    return counts
