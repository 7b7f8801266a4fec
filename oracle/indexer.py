"""CPU ORACLE (test infrastructure, not part of the product): segment/slot indexer.

Restates, with the dumbest loops available, the integer work the GPU library
does before it launches anything: which cache slot and rank every token uses
(`token_map`), and which tokens go to the tile path and which to the GEMV path
under the library's stated threshold rule (`index`).  The GPU library's indexer is
written separately (C++, different algorithm); tests demand exact equality.

The batch structure follows the paper: the scheduler re-forms the batch on
every decode iteration (sections 2 and 4.1), so one batch mixes 1-token decode
requests and whole prompts, each request bringing its own adapter; the engine
receives the batch together with the adapters its requests name (section 2).
One segment = one request of the iteration.

Canonical work lists (the library's contract for `lora_index`):

* A segment is *active* if its slot is >= 0 and it is not empty.
* With `mfma_min_tokens` = M0 > 0, an active segment of at least M0 tokens is
  *long*: it is cut into tiles of `tile_tokens` consecutive tokens (the last
  one ragged), in segment order.
* Tokens of all other active segments are pooled per slot, slots ascending,
  tokens ascending.  A pool of at least M0 tokens (M0 > 0) is cut into tiles
  the same way (a *gathered* tile: its tokens need not be consecutive); a
  smaller pool, or any pool when M0 = 0, is one *group*.
* `tok_list` = tokens of all tiles (long-segment tiles first, then gathered
  tiles), then tokens of all groups.  A tile or group names its tokens as
  (`tok_off`, `n_tok`) into `tok_list`.

How the kernels cut a tile or a group into blocks, wavefronts, rank rows and
column runs is their own business and no part of this contract; the tests check
those work lists through properties (every token, rank row and output column
covered exactly once, with the slot and rank `token_map` gives).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

Item = Tuple[int, int, int, int, int, int]  # tok_off, n_tok, slot, rank, a, b


def token_map(T: int, seg_offsets: Sequence[int], seg_slot: Sequence[int], seg_rank: Sequence[int]):
    """Per-token (slot, rank); -1 / 0 where the token has no adapter."""
    tok_slot = [-1] * T
    tok_rank = [0] * T
    for g in range(len(seg_slot)):
        for t in range(int(seg_offsets[g]), int(seg_offsets[g + 1])):
            if seg_slot[g] >= 0:
                tok_slot[t] = int(seg_slot[g])
                tok_rank[t] = int(seg_rank[g])
    return tok_slot, tok_rank


def index(
    T: int,
    seg_offsets: Sequence[int],
    seg_slot: Sequence[int],
    seg_rank: Sequence[int],
    mfma_min_tokens: int,
    tile_tokens: int = 64,
) -> Dict[str, list]:
    n_seg = len(seg_slot)
    tiles: List[Item] = []
    tile_toks: List[int] = []
    pooled: Dict[int, List[int]] = {}
    pooled_rank: Dict[int, int] = {}

    def cut(tokens: List[int], slot: int, rank: int) -> None:
        i = 0
        while i < len(tokens):
            part = tokens[i : i + tile_tokens]
            tiles.append((len(tile_toks), len(part), slot, rank, i // tile_tokens, 0))
            tile_toks.extend(part)
            i += tile_tokens

    for g in range(n_seg):
        lo, hi = int(seg_offsets[g]), int(seg_offsets[g + 1])
        slot = int(seg_slot[g])
        if slot < 0 or hi == lo:
            continue
        toks = list(range(lo, hi))
        if mfma_min_tokens > 0 and len(toks) >= mfma_min_tokens:
            cut(toks, slot, int(seg_rank[g]))
        else:
            pooled.setdefault(slot, []).extend(toks)
            pooled_rank[slot] = int(seg_rank[g])

    group_sets: List[Tuple[List[int], int, int]] = []
    for slot in sorted(pooled):
        toks = sorted(pooled[slot])
        if mfma_min_tokens > 0 and len(toks) >= mfma_min_tokens:
            cut(toks, slot, pooled_rank[slot])
        else:
            group_sets.append((toks, slot, pooled_rank[slot]))

    tok_list = list(tile_toks)
    groups: List[Item] = []
    for toks, slot, rank in group_sets:
        groups.append((len(tok_list), len(toks), slot, rank, 0, 0))
        tok_list.extend(toks)

    return {
        "tok_list": tok_list,
        "tiles": tiles,
        "groups": groups,
    }
