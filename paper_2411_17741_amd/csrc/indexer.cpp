// Segment/slot indexer: the integer work between the scheduler's batch (one segment per
// request of the iteration, each naming the cache slot of its adapter; paper sections 2
// and 4.1) and the kernels' work lists.  Pure host code; the contract is in lora_cache.h.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <unordered_map>
#include <vector>

#include "lora_internal.h"

namespace {

struct ShortSeg {
    int32_t slot, seg;
};

template <typename T> T *dup(const std::vector<T> &v)
{
    T *p = static_cast<T *>(std::malloc(sizeof(T) * (v.empty() ? 1 : v.size())));
    if (p && !v.empty()) std::memcpy(p, v.data(), sizeof(T) * v.size());
    return p;
}

lora_item_t make_item(int32_t off, int32_t n, int32_t slot, int32_t rank, int32_t a, int32_t b)
{
    lora_item_t it;
    it.tok_off = off; it.n_tok = n; it.slot = slot; it.rank = rank; it.a = a; it.b = b; it.c = 0; it.d = 0;
    return it;
}

}  // namespace

extern "C" int lora_index(int32_t T, const int32_t *seg_offsets, const int32_t *seg_slot, const int32_t *seg_rank,
                          int32_t n_seg, int32_t mfma_min_tokens, lora_worklists_t *out)
{
    if (!out) return LORA_E_INVAL;
    std::memset(out, 0, sizeof(*out));
    if (T < 0 || n_seg < 0 || mfma_min_tokens < 0 || !seg_offsets) return LORA_E_INVAL;
    if (n_seg > 0 && (!seg_slot || !seg_rank)) return LORA_E_INVAL;
    if (seg_offsets[0] != 0 || seg_offsets[n_seg] != T) return LORA_E_INVAL;

    std::unordered_map<int32_t, int32_t> rank_of;
    for (int32_t g = 0; g < n_seg; ++g) {
        if (seg_offsets[g + 1] < seg_offsets[g]) return LORA_E_INVAL;
        if (seg_slot[g] < 0) continue;
        if (seg_rank[g] < 1 || seg_rank[g] > LORA_MAX_RANK) return LORA_E_INVAL;
        auto ins = rank_of.emplace(seg_slot[g], seg_rank[g]);
        if (!ins.second && ins.first->second != seg_rank[g]) return LORA_E_INVAL;
    }

    const int32_t TM = LORA_TILE_TOKENS;
    std::vector<int32_t> tile_tok, group_tok;
    std::vector<lora_item_t> tiles, groups;
    std::vector<ShortSeg> shorts;

    // long segments become runs of tiles straight away; the rest is bucketed by slot
    for (int32_t g = 0; g < n_seg; ++g) {
        const int32_t lo = seg_offsets[g], n = seg_offsets[g + 1] - lo;
        if (seg_slot[g] < 0 || n == 0) continue;
        if (mfma_min_tokens > 0 && n >= mfma_min_tokens) {
            for (int32_t s = 0, k = 0; s < n; s += TM, ++k) {
                const int32_t cnt = std::min(TM, n - s);
                tiles.push_back(make_item((int32_t)tile_tok.size(), cnt, seg_slot[g], seg_rank[g], k, 0));
                for (int32_t t = 0; t < cnt; ++t) tile_tok.push_back(lo + s + t);
            }
        } else {
            shorts.push_back({seg_slot[g], g});
        }
    }
    std::stable_sort(shorts.begin(), shorts.end(), [](const ShortSeg &a, const ShortSeg &b) { return a.slot < b.slot; });

    for (size_t i = 0; i < shorts.size();) {
        size_t e = i;
        int32_t total = 0;
        while (e < shorts.size() && shorts[e].slot == shorts[i].slot) {
            total += seg_offsets[shorts[e].seg + 1] - seg_offsets[shorts[e].seg];
            ++e;
        }
        const int32_t slot = shorts[i].slot, rank = seg_rank[shorts[i].seg];
        const bool as_tiles = mfma_min_tokens > 0 && total >= mfma_min_tokens;
        std::vector<int32_t> &dst = as_tiles ? tile_tok : group_tok;
        const int32_t first = (int32_t)dst.size();
        for (size_t q = i; q < e; ++q)  // segments of one slot are already in ascending token order
            for (int32_t t = seg_offsets[shorts[q].seg]; t < seg_offsets[shorts[q].seg + 1]; ++t) dst.push_back(t);
        if (as_tiles) {
            for (int32_t s = 0, k = 0; s < total; s += TM, ++k)
                tiles.push_back(make_item(first + s, std::min(TM, total - s), slot, rank, k, 0));
        } else {
            groups.push_back(make_item(first, total, slot, rank, 0, 0));  // tok_off fixed up below
        }
        i = e;
    }

    const int32_t n_tile_tok = (int32_t)tile_tok.size();
    for (auto &gr : groups) gr.tok_off += n_tile_tok;
    tile_tok.insert(tile_tok.end(), group_tok.begin(), group_tok.end());

    out->n_tok_list = (int32_t)tile_tok.size();
    out->n_tiles = (int32_t)tiles.size();
    out->n_groups = (int32_t)groups.size();
    out->tok_list = dup(tile_tok);
    out->tiles = dup(tiles);
    out->groups = dup(groups);
    if (!out->tok_list || !out->tiles || !out->groups) {
        lora_worklists_free(out);
        return LORA_E_NOMEM;
    }
    return LORA_OK;
}

extern "C" void lora_worklists_free(lora_worklists_t *w)
{
    if (!w) return;
    std::free(w->tok_list);
    std::free(w->tiles);
    std::free(w->groups);
    std::memset(w, 0, sizeof(*w));
}
