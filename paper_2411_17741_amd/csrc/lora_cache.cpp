// Host side of liblora_cache: pool layout, slot table (the adapter cache's entries and their
// metadata, paper section 4.2), fills from host memory, plans and the apply launches.
#include <algorithm>
#include <limits>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

#include "lora_internal.h"

namespace {

thread_local int g_last_hip = 0;

#define HIP_TRY(expr)                          \
    do {                                       \
        hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) {                \
            g_last_hip = (int)e_;              \
            return LORA_E_HIP;                 \
        }                                      \
    } while (0)

constexpr int N_INTERNAL_PLANS = 4;
constexpr int N_STAGES = 2;
constexpr int N_APPLY_EVENTS = 64;
constexpr size_t ALIGN = 256;
// Tile shrink: at most this many runs per launch (two resident blocks per compute unit of a 256-unit part), and
// the variants of the run tables a plan carries: one per number of projections served by one launch, and one with
// few runs for the small fixed scratch.
constexpr int SHRINK_MAX_RUNS = 512;
constexpr int SHRINK_VARIANTS = lora::MAX_SHRINK_PROJS + 1;
constexpr int SHRINK_VARIANT_SMALL = lora::MAX_SHRINK_PROJS;
constexpr int N_LINEAR_FLAGS = 1024;  // split-off parts of lora_linear_plan's last round of tiles: fewer than CUs x 3
constexpr double TILE_PATH_FIXED_US = 25.0;          // what the three launches of the tile path cost beside their work
constexpr double TILE_PATH_L2_BYTES_PER_US = 10e6;  // rate at which repeated passes over a slab come out of L2
constexpr int N_VSETS = lora::MAX_SHRINK_PROJS;  // applies that share their input run shrink-first, each with its own intermediate

size_t align_up(size_t v, size_t a = ALIGN) { return (v + a - 1) / a * a; }

// Device memory an apply needs beside its inputs and outputs: the shrink results (one set per
// projection of a group), the partial sums that the runs of the tile shrink leave, and the tagged words through
// which the one-launch GEMV form hands its intermediate over.
struct Scratch {
    char *v;
    size_t v_set_bytes;
    int n_sets;
    char *vpart;
    int64_t vpart_rows;        // rows of the partial-sum scratch, shared by the projections of a group
    bool small;                // the scratch holds the partial sums of the small run table only
    char *vtag;                // hand-over words of the GEMV phases, one set per projection of a group
    size_t vtag_set_bytes;
    uint32_t *epoch;           // host counter of the one-launch GEMV launches that have used vtag
    // the latest one-launch GEMV enqueued under stream capture with this scratch: capture, plan and sets
    // (a replayed launch finds its own number in the words it wrote the last time, unless another launch
    // of the graph has written them since)
    unsigned long long *cap_id;
    uint64_t *cap_plan;
    int *cap_sets;
};

// The same scratch as a fixed array in the library's image, for lora_apply_plan_static: one set,
// sized for LORA_STATIC_MAX_TOKENS tokens.  Every device the library runs on holds its own copy
// at its own address (found once per device with hipGetSymbolAddress; the array's name itself is
// no device address in host code).
constexpr size_t STATIC_V_BYTES = sizeof(float) * (size_t)LORA_STATIC_MAX_TOKENS * LORA_MAX_RANK;
constexpr int STATIC_SHRINK_RUNS = 128;
constexpr int64_t STATIC_VPART_ROWS = 2 * (int64_t)lora::SHRINK_SLOT_ROWS * STATIC_SHRINK_RUNS;  // = 4 x LORA_STATIC_MAX_TOKENS
constexpr size_t STATIC_VPART_BYTES = sizeof(float) * (size_t)STATIC_VPART_ROWS * LORA_MAX_RANK;
constexpr size_t STATIC_VTAG_BYTES = sizeof(uint64_t) * (size_t)LORA_STATIC_MAX_TOKENS * LORA_MAX_RANK;  // fp32 words; bf16 takes half
constexpr size_t STATIC_SCRATCH_BYTES = STATIC_V_BYTES + STATIC_VPART_BYTES + STATIC_VTAG_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
struct StaticScratch {
    char *ptr = nullptr;   // this device's copy of `scratch`
    uint32_t epoch = 0;    // one-launch GEMV launches that have used its hand-over words, over all caches of the process
    unsigned long long cap_id = 0;
    uint64_t cap_plan = 0;
    int cap_sets = 0;
};
StaticScratch g_static[MAX_DEVICES];

// Once per device, with that device current: the address of its copy, and tagged words that carry no
// launch number yet.
int static_scratch_setup(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return LORA_E_INVAL;
    StaticScratch &ss = g_static[device];
    if (ss.ptr) return LORA_OK;
    char *ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)));
    if (!ptr) return LORA_E_HIP;
    HIP_TRY(hipMemset(ptr + STATIC_V_BYTES + STATIC_VPART_BYTES, 0, STATIC_VTAG_BYTES));
    ss.ptr = ptr;
    return LORA_OK;
}
int esize_of(int dtype) { return dtype == LORA_BF16 ? 2 : 4; }

struct Slot {
    int32_t cls = 0;
    bool bound = false;
    int64_t adapter_id = 0;
    int32_t rank = 0;
    float alpha = 1.f;
    int32_t refcount = 0;
    int64_t use_count = 0, last_used = 0;
    double req_freq = 0;   // requests that used the entry, halved every policy.freq_window requests
    int64_t req_last = 0;  // number of the last such request
    uint32_t generation = 0;  // bumped whenever the slot is bound to another adapter or evicted
    std::vector<uint8_t> part;  // [n_layers * n_proj] 1 = data enqueued
    int32_t parts_filled = 0;
    hipEvent_t fill_ev = nullptr;
    bool fill_pending = false;
};

struct Stage {
    char *dev = nullptr;
    hipEvent_t ev = nullptr;  // the repack that read this buffer is done: it may be overwritten
    bool pending = false;
};

}  // namespace

struct lora_plan {
    bool in_use = false;
    bool internal = false;
    char *dev = nullptr;
    char *pinned = nullptr;
    hipEvent_t ev_upload = nullptr, ev_last_use = nullptr;
    bool upload_pending = false, use_pending = false;
    int32_t T = 0;
    int32_t n_tok_list = 0, n_tiles = 0, n_gs = 0, n_ge = 0;
    int32_t n_tile_tok = 0;  // tokens of all tiles = leading entries of tok_list
    // the tile shrink's run tables (cuts, then the tiles' piece records), per variant
    int32_t shrink_quanta = 1;
    int32_t shrink_runs[SHRINK_VARIANTS] = {0};
    bool shrink_pieces[SHRINK_VARIANTS] = {false};
    size_t off_cuts[SHRINK_VARIANTS] = {0}, off_sums[SHRINK_VARIANTS] = {0};
    int32_t mfma_min_used = 0;  // the threshold the work lists were made with
    uint64_t build_seq = 0;     // changes whenever the plan's lists are rebuilt
    size_t off_tiles = 0, off_gs = 0, off_ge = 0, bytes = 0;
    // for lora_linear_plan: every token of the batch in row tiles -- the tiles above, then runs of up
    // to 64 of the other tokens (rank 0) -- over a token list of its own
    size_t off_lin_tok = 0, off_lin_tiles = 0;
    int32_t n_lin_tiles = 0;
    std::vector<int32_t> slots;        // distinct slots the batch names
    std::vector<uint32_t> generations;  // their generation at plan time
};

struct lora_cache {
    std::vector<lora_proj_t> proj;
    std::vector<int32_t> class_rank, class_slots, class_first;
    int32_t n_layers = 0, n_slots = 0, dtype = 0, esize = 0;
    int32_t max_tokens = 0, max_segments = 0, n_user_plans = 0, mfma_min = 0, flags = 0;
    bool mfma_min_auto = false;  // the configuration left the threshold to the library
    int32_t v_stride = 0;
    bool host_only = false;

    char *pool = nullptr;
    size_t pool_bytes = 0;
    size_t layer_stride = 0;
    std::vector<int32_t> slot_row;  // [n_slots] first storage row of the slot (same in every projection)
    std::vector<size_t> proj_off;   // [n_proj] byte offset of the projection's slabs inside a layer
    std::vector<size_t> row_bytes;  // [n_proj] (h_in + h_out) * element size
    int64_t total_rows = 0;
    size_t off_fault = 0, off_vpart = 0, off_vtag = 0, v_set_bytes = 0, vtag_set_bytes = 0;
    uint32_t tag_epoch = 0;  // one-launch GEMV launches so far; the number the words of the latest one carry
    unsigned long long cap_id = 0;
    uint64_t cap_plan = 0;  // build number of the plan
    int cap_sets = 0;
    int64_t vpart_rows = 0;  // rows of the tile shrink's partial-sum scratch
    size_t vpart_bytes = 0;
    int fused_gemv = 0;  // 0 never, 1 by size, 2 always
    size_t off_v = 0, off_plans = 0, off_stage = 0, plan_cap = 0, stage_cap = 0, total = 0;

    std::vector<Slot> slots;
    std::unordered_map<int64_t, int32_t> id2slot;
    std::vector<lora_plan> plans;  // user plans first, then the internal ring
    uint64_t internal_next = 0, plan_builds = 0;
    Stage stage[N_STAGES];
    bool direct_fill = false;
    uint64_t stage_next = 0;

    // Within a group the GEMV launch (decode tokens) and the tile kernels (prompts) touch different tokens and
    // different scratch: they run side by side, the GEMV launch on a stream of the cache's own between a fork
    // and a join event (default priority, like every stream here)
    hipStream_t side_stream = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int device = 0;  // the device that was current at lora_cache_create
    int n_cu = 256;  // its compute units
    bool fencing = true;
    int64_t apply_seq = 0;
    hipEvent_t apply_ev[N_APPLY_EVENTS] = {};
    int64_t apply_ev_seq[N_APPLY_EVENTS] = {};
    std::unordered_map<hipStream_t, hipEvent_t> stream_fence;  // per stream that ran applies: an event of its own, recorded with every fence
    // raised by a kernel that gave up a bounded wait: one word of pinned host memory that the kernels
    // write through its device address, so the host sees it without a synchronisation
    int32_t *fault_host = nullptr, *fault_dev = nullptr;

    lora_cache_stats_t stats = {};
    lora_policy_t policy = {0.45, 0.10, 0.45, 0};  // section 4.2's F, R, S
    int64_t req_seq = 0;                           // requests seen by lora_cache_acquire

    // benchmark aid: event pairs around kernels
    bool timing = false;
    struct Timed {
        int kind;
        hipEvent_t start, stop;
    };
    std::vector<Timed> timed;
    std::vector<hipEvent_t> free_events;
};

namespace {

bool config_ok(const lora_cache_config_t *cfg)
{
    if (!cfg || cfg->n_proj < 1 || !cfg->proj || cfg->n_layers < 1 || cfg->n_classes < 1 || !cfg->class_rank ||
        !cfg->class_slots)
        return false;
    if (cfg->dtype != LORA_F32 && cfg->dtype != LORA_BF16) return false;
    if (cfg->max_tokens < 1 || cfg->max_segments < 1 || cfg->n_plans < 0 || cfg->mfma_min_tokens < 0) return false;
    for (int p = 0; p < cfg->n_proj; ++p)
        if (cfg->proj[p].h_in < 64 || cfg->proj[p].h_out < 64 || cfg->proj[p].h_in % 64 || cfg->proj[p].h_out % 64)
            return false;
    int64_t total_slots = 0;
    for (int c = 0; c < cfg->n_classes; ++c) {
        if (cfg->class_rank[c] < 1 || cfg->class_rank[c] > LORA_MAX_RANK || cfg->class_slots[c] < 0) return false;
        if (c && cfg->class_rank[c] <= cfg->class_rank[c - 1]) return false;
        total_slots += cfg->class_slots[c];
    }
    return total_slots >= 1 && total_slots * (int64_t)LORA_MAX_RANK < (int64_t)1 << 31;
}

// Fills every layout field of `c` from the config; used by bytes_required and create alike.
void compute_layout(lora_cache &c, const lora_cache_config_t *cfg)
{
    c.proj.assign(cfg->proj, cfg->proj + cfg->n_proj);
    c.class_rank.assign(cfg->class_rank, cfg->class_rank + cfg->n_classes);
    c.class_slots.assign(cfg->class_slots, cfg->class_slots + cfg->n_classes);
    c.n_layers = cfg->n_layers;
    c.dtype = cfg->dtype;
    c.esize = esize_of(cfg->dtype);
    c.max_tokens = cfg->max_tokens;
    c.max_segments = cfg->max_segments;
    c.n_user_plans = cfg->n_plans;
    c.mfma_min = cfg->dtype == LORA_BF16 ? (cfg->mfma_min_tokens ? cfg->mfma_min_tokens : LORA_MFMA_MIN_TOKENS) : 0;
    c.mfma_min_auto = cfg->dtype == LORA_BF16 && cfg->mfma_min_tokens == 0;
    c.flags = cfg->flags;
    c.host_only = (cfg->flags & LORA_CACHE_HOST_ONLY) != 0;
    c.direct_fill = (cfg->flags & LORA_CACHE_DIRECT_FILL) != 0;
    c.fused_gemv = (cfg->flags & LORA_CACHE_SPLIT_GEMV) ? 0 : ((cfg->flags & LORA_CACHE_FUSED_GEMV) ? 2 : 1);

    const int n_proj = cfg->n_proj, n_cls = cfg->n_classes;
    c.class_first.resize(n_cls);
    c.n_slots = 0;
    for (int k = 0; k < n_cls; ++k) {
        c.class_first[k] = c.n_slots;
        c.n_slots += c.class_slots[k];
    }
    c.slot_row.assign(c.n_slots, 0);
    c.total_rows = 0;
    for (int k = 0; k < n_cls; ++k)
        for (int s = 0; s < c.class_slots[k]; ++s) {
            c.slot_row[c.class_first[k] + s] = (int32_t)c.total_rows;
            c.total_rows += lora::rank_storage(c.class_rank[k]);
        }
    c.proj_off.assign(n_proj, 0);
    c.row_bytes.assign(n_proj, 0);
    size_t off = 0, max_part = 0;
    for (int p = 0; p < n_proj; ++p) {
        const size_t width = (size_t)c.proj[p].h_in + (size_t)c.proj[p].h_out;
        c.proj_off[p] = off;
        c.row_bytes[p] = width * c.esize;  // a multiple of 256 bytes: h_in, h_out are multiples of 64
        off += (size_t)c.total_rows * c.row_bytes[p];
        max_part = std::max(max_part, (size_t)c.class_rank[n_cls - 1] * width * c.esize);
    }
    c.layer_stride = off;
    c.v_stride = LORA_MAX_RANK;  // the GEMV expand reads whole rows of 128 entries (masked past the rank)

    const size_t max_tiles = (size_t)c.max_tokens / LORA_TILE_TOKENS + 2 * (size_t)c.max_segments + 2;
    // GEMV items: per token batch up to 32 shrink + 16 expand items; batches <= groups + tokens/4
    const size_t max_batches = (size_t)c.max_segments + (size_t)c.max_tokens / lora::GEMV_BATCH + 1;
    const size_t max_items = max_tiles + max_batches * (LORA_MAX_RANK / 4 + 16);
    c.plan_cap = align_up(sizeof(int32_t) * (size_t)c.max_tokens) + align_up(sizeof(lora_item_t) * max_items) +
                 align_up(sizeof(int32_t) * max_batches) + 4 * ALIGN +
                 align_up(sizeof(int32_t) * (size_t)c.max_tokens) +
                 align_up(sizeof(lora_item_t) * (max_tiles + (size_t)c.max_tokens / LORA_TILE_TOKENS + 2)) +
                 SHRINK_VARIANTS * (align_up(sizeof(lora::ShrinkCut) * (SHRINK_MAX_RUNS + 1)) + align_up(sizeof(lora::ShrinkSum) * max_tiles));
    c.stage_cap = align_up(max_part) + ALIGN;

    size_t cur = align_up(c.layer_stride * (size_t)c.n_layers);
    c.off_fault = cur;  // (once the fault word; now the flags of the fused linear kernel's split tiles)
    cur += align_up(sizeof(uint32_t) * N_LINEAR_FLAGS);
    c.off_v = cur;
    c.v_set_bytes = align_up(sizeof(float) * (size_t)c.max_tokens * c.v_stride);
    cur += c.v_set_bytes * N_VSETS;
    // partial sums of the tile shrink: two slots per run and projection of a group; a launch has at most
    // SHRINK_MAX_RUNS blocks whatever the group's size, and a batch of few tiles has few runs (a piece is at least
    // two of the parts a tile's k range is cut into)
    {
        const int64_t tiles = std::max<int64_t>(1, ((int64_t)c.max_tokens + LORA_TILE_TOKENS - 1) / LORA_TILE_TOKENS);
        const int64_t runs = std::min<int64_t>(SHRINK_MAX_RUNS, 16 * N_VSETS * tiles);
        c.vpart_rows = c.dtype == LORA_BF16 ? 2 * lora::SHRINK_SLOT_ROWS * runs : 0;
    }
    c.off_vpart = cur;
    c.vpart_bytes = align_up(sizeof(float) * (size_t)c.vpart_rows * c.v_stride);
    // (the fused linear kernel parks the partial sums of its split tiles in the same region: at most 48 MB,
    // less for caches of small batches)
    if (c.dtype == LORA_BF16)
        c.vpart_bytes = std::max(c.vpart_bytes, std::min<size_t>((size_t)48 << 20, align_up(sizeof(float) * (size_t)c.v_stride * 8 * (size_t)c.max_tokens)));
    cur += c.vpart_bytes;
    // the GEMV phases hand their intermediate over as 64-bit words, one row per token and projection of a group
    c.off_vtag = cur;
    c.vtag_set_bytes = align_up(lora::gemv_handover_bytes(c.dtype, c.max_tokens));
    cur += c.vtag_set_bytes * N_VSETS;
    c.off_plans = cur;
    cur += c.plan_cap * (size_t)(c.n_user_plans + N_INTERNAL_PLANS);
    c.off_stage = cur;
    cur += c.stage_cap * N_STAGES;
    c.total = cur;
}

char *slab_ptr(const lora_cache &c, int32_t layer, int32_t proj, int32_t slot)
{
    return c.pool + (size_t)layer * c.layer_stride + c.proj_off[proj] + (size_t)c.slot_row[slot] * c.row_bytes[proj];
}

int class_of_slot(const lora_cache &c, int32_t slot)
{
    int k = (int)c.class_first.size() - 1;
    while (k > 0 && slot < c.class_first[k]) --k;
    return k;
}

void unbind(lora_cache &c, Slot &s)
{
    if (s.bound) {
        auto it = c.id2slot.find(s.adapter_id);
        if (it != c.id2slot.end() && &c.slots[it->second] == &s) c.id2slot.erase(it);
    }
    s.bound = false;
    s.adapter_id = 0;
    s.rank = 0;
    s.alpha = 1.f;
    s.use_count = 0;
    s.req_freq = 0;
    s.req_last = 0;
    s.refcount = 0;
    s.parts_filled = 0;
    std::fill(s.part.begin(), s.part.end(), 0);
    ++s.generation;
}

// Section 4.2's eviction score of every cached entry: F * frequency + R * recency + S * size.
// The paper gives no units: each term is scaled to [0, 1] over the cached entries (frequency and
// rank by the largest cached, recency as 1 - age / largest age, age counted in requests), so that
// the coefficients weigh comparable quantities.  Entries that are not cached get +inf.
std::vector<double> eviction_scores(const lora_cache &c)
{
    double max_f = 0, max_age = 0, max_rank = 0;
    for (const Slot &s : c.slots) {
        if (!s.bound) continue;
        max_f = std::max(max_f, s.req_freq);
        max_age = std::max(max_age, (double)(c.req_seq - s.req_last));
        max_rank = std::max(max_rank, (double)s.rank);
    }
    std::vector<double> score(c.slots.size(), std::numeric_limits<double>::infinity());
    for (size_t i = 0; i < c.slots.size(); ++i) {
        const Slot &s = c.slots[i];
        if (!s.bound) continue;
        const double f = max_f > 0 ? s.req_freq / max_f : 0.0;
        const double r = max_age > 0 ? 1.0 - (double)(c.req_seq - s.req_last) / max_age : 1.0;
        const double z = (double)s.rank / max_rank;
        score[i] = c.policy.w_freq * f + c.policy.w_recency * r + c.policy.w_size * z;
    }
    return score;
}

bool is_queued(const int64_t *ids, int32_t n, int64_t id)
{
    for (int32_t i = 0; i < n; ++i)
        if (ids[i] == id) return true;
    return false;
}

// The entry to evict for an adapter of `rank` (any rank if 0): lowest score among the entries
// no running request uses and whose slot is large enough; entries of queued requests only if
// there is no other (section 4.2).  Ties go to the lower slot.  -1 if every candidate is in use.
int32_t choose_victim(const lora_cache &c, int32_t rank, const int64_t *queued, int32_t n_queued)
{
    const std::vector<double> score = eviction_scores(c);
    for (int pass = 0; pass < 2; ++pass) {
        int32_t best = -1;
        for (int32_t i = 0; i < c.n_slots; ++i) {
            const Slot &s = c.slots[i];
            if (!s.bound || s.refcount > 0 || c.class_rank[s.cls] < rank) continue;
            if (pass == 0 && is_queued(queued, n_queued, s.adapter_id)) continue;
            if (best < 0 || score[i] < score[best]) best = i;
        }
        if (best >= 0) return best;
    }
    return -1;
}

// bytes of pool memory the entry of a slot holds: its rank's storage rows in every layer and projection
size_t entry_bytes(const lora_cache &c, const Slot &s)
{
    size_t per_row = 0;
    for (size_t p = 0; p < c.proj.size(); ++p) per_row += c.row_bytes[p];
    return (size_t)lora::rank_storage(s.rank) * per_row * (size_t)c.n_layers;
}

int slot_state(lora_cache &c, Slot &s)
{
    if (!s.bound) return LORA_SLOT_EMPTY;
    if (s.parts_filled < (int32_t)s.part.size()) return LORA_SLOT_FILLING;
    if (s.fill_pending && !c.host_only) {
        if (hipEventQuery(s.fill_ev) == hipSuccess) s.fill_pending = false;
        else return LORA_SLOT_FILLING;
    }
    return LORA_SLOT_READY;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

bool is_capturing(hipStream_t st)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs != hipStreamCaptureStatusNone;
}

// The tile shrink's run table for `max_runs` runs (header of ShrinkCut in lora_internal.h): cuts[0 .. n_runs] and one
// piece record per tile.  A tile's cost per part of its k range: its x rows (absent rows are still loaded) plus its
// stored At rows (measured: a rank-128 tile takes 1.8 times as long as a rank-16 one).
struct ShrinkRuns {
    std::vector<lora::ShrinkCut> cuts;
    std::vector<lora::ShrinkSum> sums;
    int n_runs = 0;
    bool any_pieces = false;
};
bool shrink_pieces_of(const lora::DevItem *tiles, int n_tiles, int quanta, ShrinkRuns &out)
{
    out.sums.assign((size_t)n_tiles, lora::ShrinkSum{0, 0});
    out.any_pieces = false;
    for (int r = 0; r < out.n_runs; ++r) {
        const lora::ShrinkCut from = out.cuts[r], to = out.cuts[r + 1];
        const int last_tile = std::min(to.part > 0 ? to.tile : to.tile - 1, n_tiles - 1);
        for (int t = from.tile; t <= last_tile; ++t) {
            const int lo = t == from.tile ? from.part : 0, hi = t == to.tile ? to.part : quanta;
            if (lo >= hi) continue;
            lora::ShrinkSum &sm = out.sums[t];
            const int32_t slot = lora::shrink_slot(r, from.tile, t);
            if (sm.n_pieces == 0) sm.first_slot = (lo == 0 && hi == quanta) ? 0 : slot;
            else if (slot != 2 * (sm.first_slot / 2 + sm.n_pieces)) return false;  // (cannot happen: later pieces start their runs)
            ++sm.n_pieces;
            if (sm.n_pieces > 1) out.any_pieces = true;
        }
    }
    for (int t = 0; t < n_tiles; ++t)
        if (out.sums[t].n_pieces < 1) return false;
    (void)tiles;
    return true;
}
// Runs of about equal cost, at most max_runs of them (a multiple of 8).  A piece costs its parts times its tile's
// weight, plus a fixed amount.  Measured with every block of a launch resident from the start (two per compute unit):
// a block spends about 6.5 us beside its k loop (the item, the first three stages of loads that every block requests at
// once, the write of the result); a stage of 128 k takes it 1.4 us at rank 16, 1.6 us at rank 32, 1.9 us at rank 64 and
// 2.6 us at rank 128 when the launch is long (x arrives at the rate the memory gives, the higher ranks add their At
// loads).  The result is flat around these weights: a fixed amount of 3 to 6 stages and a stage offset of 30 to 60
// gave the same launch times to within 1 %.  For a cost limit the sequence is walked once, every run taking pieces until
// the limit is reached; the smallest limit that needs no more than max_runs runs is found by bisection.
void build_shrink_runs(const lora::DevItem *tiles, int n_tiles, int quanta, int max_runs, ShrinkRuns &out)
{
    constexpr int64_t MINP = lora::SHRINK_MIN_PARTS, PIECE = 6 * (44 + LORA_TILE_TOKENS + 16);  // six stages at rank 16
    std::vector<int64_t> weight((size_t)n_tiles);
    int64_t total = 0, w_max = 1;
    for (int t = 0; t < n_tiles; ++t) {
        weight[t] = 44 + (int64_t)tiles[t].n_tok + lora::rank_storage(tiles[t].rank);  // rank 128 : rank 16 = 1.9
        total += weight[t] * quanta + PIECE;
        w_max = std::max(w_max, weight[t]);
    }
    // one walk: the number of runs; their starts go to `cuts` when given
    auto walk = [&](int64_t limit, std::vector<lora::ShrinkCut> *cuts) -> int64_t {
        int t = 0, q = 0;
        int64_t runs = 0;
        while (t < n_tiles) {
            if (cuts) cuts->push_back(lora::ShrinkCut{t, q});
            ++runs;
            int64_t cost = 0;
            bool first = true;
            while (t < n_tiles) {
                const int64_t w = weight[t], rem = quanta - q;
                if (cost + w * rem + PIECE <= limit) {  // the rest of the tile
                    cost += w * rem + PIECE;
                    ++t, q = 0, first = false;
                    continue;
                }
                int64_t parts = (limit - cost - PIECE) / w;  // what still fits (rounded towards zero: never negative parts >= MINP)
                if (parts < MINP) {
                    if (!first) break;  // the run ends on the tile boundary
                    parts = MINP;       // a run takes something
                }
                if (rem - parts < MINP) ++t, q = 0;  // no slivers: the rest of the tile
                else q += (int)parts;
                break;
            }
        }
        return runs;
    };
    int64_t lo = w_max * std::min<int64_t>(MINP, quanta) + PIECE, hi = std::max(total, lo);  // hi: one run takes everything
    while (hi - lo > hi / 128) {  // to within 1 % of the smallest limit
        const int64_t mid = lo + (hi - lo) / 2;
        if (walk(mid, nullptr) <= max_runs) hi = mid;
        else lo = mid + 1;
    }
    for (int attempt = 0; attempt < 2; ++attempt) {
        out.cuts.clear();
        // second attempt (never needed as far as the walk goes): whole tiles only, as many per run as it takes
        int64_t used;
        if (attempt == 0) used = walk(hi, &out.cuts);
        else {
            const int per_run = (n_tiles + max_runs - 1) / max_runs;
            for (int t = 0; t < n_tiles; t += per_run) out.cuts.push_back(lora::ShrinkCut{t, 0});
            used = (int64_t)out.cuts.size();
        }
        out.n_runs = (int)((used + 7) / 8 * 8);
        out.cuts.resize((size_t)out.n_runs + 1, lora::ShrinkCut{n_tiles, 0});
        if (used <= max_runs && shrink_pieces_of(tiles, n_tiles, quanta, out)) return;
    }
}

// Validates a batch against the slot table and writes its work lists into plan `p`
// (pinned copy + upload on `st`).
int build_plan(lora_cache &c, lora_plan &p, int32_t T, const int32_t *seg_offsets, const int32_t *seg_slot,
               const int32_t *seg_rank, int32_t n_seg, hipStream_t st)
{
    if (T < 0 || T > c.max_tokens || n_seg < 0 || n_seg > c.max_segments) return LORA_E_INVAL;
    lora_worklists_t w;
    int rc = lora_index(T, seg_offsets, seg_slot, seg_rank, n_seg, c.mfma_min, &w);
    if (rc != LORA_OK) return rc;
    p.mfma_min_used = c.mfma_min;
    // With the threshold left to the library: the tile path costs three more launches per apply
    // (about 25 us), which a batch with only a few hundred tile tokens (the pooled tokens of a few
    // hot adapters in a decode batch) does not earn back -- as GEMV groups those tokens cost one
    // more pass over their slab per 4 tokens, out of L2.  So: estimate that cost; below the fixed
    // cost of the tile launches everything stays GEMV; else the batch pays for the tile launches
    // anyway and smaller pools of tokens become tiles too.
    if (c.mfma_min_auto && w.n_tiles > 0) {
        double mean_width = 0;
        for (const auto &pr : c.proj) mean_width += (double)pr.h_in + pr.h_out;
        mean_width /= (double)c.proj.size();
        std::unordered_map<int32_t, std::pair<int64_t, int32_t>> of_slot;  // slot -> (tile tokens, rank)
        for (int i = 0; i < w.n_tiles; ++i) {
            auto &e = of_slot[w.tiles[i].slot];
            e.first += w.tiles[i].n_tok;
            e.second = w.tiles[i].rank;
        }
        double extra_bytes = 0;
        for (const auto &kv : of_slot)
            extra_bytes += (double)((kv.second.first + lora::GEMV_BATCH - 1) / lora::GEMV_BATCH) * kv.second.second * mean_width * c.esize;
        const double gemv_us = extra_bytes / TILE_PATH_L2_BYTES_PER_US;
        lora_worklists_free(&w);
        p.mfma_min_used = gemv_us < TILE_PATH_FIXED_US ? 0 : LORA_MFMA_MIN_TOKENS_MIXED;
        rc = lora_index(T, seg_offsets, seg_slot, seg_rank, n_seg, p.mfma_min_used, &w);
        if (rc != LORA_OK) return rc;
    }

    p.slots.clear();
    p.generations.clear();
    auto check = [&](const lora_item_t &it) -> int {
        if (it.slot >= c.n_slots) return LORA_E_INVAL;
        const Slot &s = c.slots[it.slot];
        if (!s.bound) return LORA_E_STATE;
        if (s.rank != it.rank) return LORA_E_INVAL;
        if (p.slots.empty() || p.slots.back() != it.slot) {
            p.slots.push_back(it.slot);
        }
        return LORA_OK;
    };
    for (int i = 0; i < w.n_tiles && rc == LORA_OK; ++i) rc = check(w.tiles[i]);
    for (int i = 0; i < w.n_groups && rc == LORA_OK; ++i) rc = check(w.groups[i]);
    if (rc != LORA_OK) {
        lora_worklists_free(&w);
        return rc;
    }
    std::sort(p.slots.begin(), p.slots.end());
    p.slots.erase(std::unique(p.slots.begin(), p.slots.end()), p.slots.end());
    for (int32_t s : p.slots) p.generations.push_back(c.slots[s].generation);

    // resolve slots: the device copy of an item carries the slot's first storage row, the
    // entry's alpha and the item's first token
    auto stamp = [&](lora_item_t *items, int n) {
        for (int i = 0; i < n; ++i) {
            const Slot &s = c.slots[items[i].slot];
            lora::DevItem d;
            d.tok_off = items[i].tok_off;
            d.n_tok = items[i].n_tok;
            d.row = c.slot_row[items[i].slot];
            d.rank = items[i].rank;
            d.a = items[i].a;
            d.consecutive = 1;
            for (int t = 1; t < items[i].n_tok; ++t)
                if (w.tok_list[items[i].tok_off + t] != w.tok_list[items[i].tok_off] + t) d.consecutive = 0;
            d.alpha = s.alpha;
            d.tok0 = w.tok_list[items[i].tok_off];
            std::memcpy(&items[i], &d, sizeof(d));
        }
    };
    p.n_tile_tok = 0;
    for (int i = 0; i < w.n_tiles; ++i) p.n_tile_tok += w.tiles[i].n_tok;
    // GEMV work items.  A group is worked on in token batches (runs of up to GEMV_BATCH entries of its
    // part of tok_list), every batch with items of its own so that batches run side by side: per batch
    // one shrink item per GEMV_SHRINK_ROWS stored rank rows, and one expand item per run of
    // gemv_expand_width(rank) columns of a super-chunk (the launch repeats it for every super-chunk of
    // the projection).
    // Groups in order of rising rank, whatever the caller's slot numbering (measured on the decode configuration:
    // 10.0 us per layer, 10.5 us with the order reversed).
    std::vector<lora::GemvItem> gs, ge;
    std::vector<int> group_order((size_t)w.n_groups);
    for (int i = 0; i < w.n_groups; ++i) group_order[i] = i;
    std::stable_sort(group_order.begin(), group_order.end(),
                     [&](int x, int y) { return lora::rank_storage(w.groups[x].rank) < lora::rank_storage(w.groups[y].rank); });
    for (int gi = 0; gi < w.n_groups; ++gi) {
        const lora_item_t &gr = w.groups[group_order[gi]];
        lora::GemvItem d;
        d.row = c.slot_row[gr.slot];
        d.rank = gr.rank;
        d.alpha = c.slots[gr.slot].alpha;
        const int32_t nc = lora::gemv_expand_width(gr.rank);
        for (int pass = 0; pass < 2; ++pass)
            for (int32_t b0 = 0; b0 < gr.n_tok; b0 += lora::GEMV_BATCH) {
                for (int t = 0; t < lora::GEMV_BATCH; ++t) d.tok[t] = b0 + t < gr.n_tok ? w.tok_list[gr.tok_off + b0 + t] : -1;
                if (pass == 0) {
                    for (int32_t j0 = 0; j0 < lora::rank_storage(gr.rank); j0 += lora::GEMV_SHRINK_ROWS) {
                        d.a = lora::gemv_pack_shrink(j0);
                        gs.push_back(d);
                    }
                } else {
                    for (int32_t col = 0; col < lora::GEMV_SUPER_COLS; col += nc) {
                        d.a = lora::gemv_pack_expand(col);
                        ge.push_back(d);
                    }
                }
            }
    }
    stamp(w.tiles, w.n_tiles);
    // the tile shrink's run tables
    ShrinkRuns shrink_runs[SHRINK_VARIANTS];
    {
        int32_t quanta = INT32_MAX;
        for (const auto &pr : c.proj) quanta = std::min(quanta, (pr.h_in + lora::SHRINK_STAGE_K - 1) / lora::SHRINK_STAGE_K);
        p.shrink_quanta = std::max(1, std::min(quanta, 1 << 14));
        const int64_t slots = std::min<int64_t>(SHRINK_MAX_RUNS, 2 * (int64_t)c.n_cu);
        const lora::DevItem *dev_tiles = reinterpret_cast<const lora::DevItem *>(w.tiles);  // stamped above
        for (int v = 0; v < SHRINK_VARIANTS && w.n_tiles > 0 && c.vpart_rows > 0; ++v) {
            if (v == SHRINK_VARIANT_SMALL && T > LORA_STATIC_MAX_TOKENS) continue;  // lora_apply_plan_static refuses such a batch
            const int n = v == SHRINK_VARIANT_SMALL ? 1 : v + 1;
            int64_t max_runs = slots / 8 / n * 8;
            max_runs = std::min(max_runs, (v == SHRINK_VARIANT_SMALL ? STATIC_VPART_ROWS : c.vpart_rows) / (2 * lora::SHRINK_SLOT_ROWS) / n / 8 * 8);
            build_shrink_runs(dev_tiles, w.n_tiles, p.shrink_quanta, (int)std::max<int64_t>(8, max_runs), shrink_runs[v]);
        }
    }

    p.T = T;
    p.n_tok_list = w.n_tok_list;
    p.n_tiles = w.n_tiles;
    p.n_gs = (int32_t)gs.size();
    p.n_ge = (int32_t)ge.size();
    p.off_tiles = align_up(sizeof(int32_t) * (size_t)w.n_tok_list);
    p.off_gs = p.off_tiles + align_up(sizeof(lora_item_t) * (size_t)w.n_tiles);
    p.off_ge = p.off_gs + align_up(sizeof(lora::GemvItem) * gs.size());
    // row tiles of the whole batch (bf16 caches: lora_linear_plan): the tiles; then runs of up to 64
    // of the tokens of the GEMV groups (marked a = 1: their output rows carry the adapter term when
    // the base product is added); then runs of the tokens that name no adapter.  The token list is
    // tok_list followed by the latter.
    std::vector<int32_t> lin_tok;
    std::vector<lora::DevItem> lin_tiles;
    if (c.dtype == LORA_BF16) {
        std::vector<uint8_t> named((size_t)T, 0);
        lin_tok.assign(w.tok_list, w.tok_list + w.n_tok_list);
        for (int32_t t : lin_tok) named[t] = 1;
        for (int32_t t = 0; t < T; ++t)
            if (!named[t]) lin_tok.push_back(t);
        lin_tiles.resize(w.n_tiles);
        std::memcpy(lin_tiles.data(), w.tiles, sizeof(lora::DevItem) * (size_t)w.n_tiles);  // stamped above
        auto plain_runs = [&](int32_t from, int32_t to, int32_t mark) {
            for (int32_t o = from; o < to; o += LORA_TILE_TOKENS) {
                lora::DevItem d{};
                d.tok_off = o;
                d.n_tok = std::min<int32_t>(LORA_TILE_TOKENS, to - o);
                d.a = mark;
                d.tok0 = lin_tok[o];
                d.consecutive = 1;
                for (int32_t i = 1; i < d.n_tok; ++i)
                    if (lin_tok[o + i] != d.tok0 + i) d.consecutive = 0;
                lin_tiles.push_back(d);
            }
        };
        plain_runs(p.n_tile_tok, w.n_tok_list, 1);
        plain_runs(w.n_tok_list, (int32_t)lin_tok.size(), 0);
    }
    p.n_lin_tiles = (int32_t)lin_tiles.size();
    p.off_lin_tok = p.off_ge + align_up(sizeof(lora::GemvItem) * ge.size());
    p.off_lin_tiles = p.off_lin_tok + align_up(sizeof(int32_t) * lin_tok.size());
    size_t bytes = p.off_lin_tiles + align_up(sizeof(lora::DevItem) * lin_tiles.size());
    for (int v = 0; v < SHRINK_VARIANTS; ++v) {
        p.shrink_runs[v] = shrink_runs[v].n_runs;
        p.shrink_pieces[v] = shrink_runs[v].any_pieces;
        p.off_cuts[v] = bytes;
        bytes += align_up(sizeof(lora::ShrinkCut) * shrink_runs[v].cuts.size());
        p.off_sums[v] = bytes;
        bytes += align_up(sizeof(lora::ShrinkSum) * shrink_runs[v].sums.size());
    }
    if (bytes > c.plan_cap) {
        lora_worklists_free(&w);
        return LORA_E_NOMEM;
    }
    // A captured upload would re-read the staged copy on every replay; plans are made outside of captures.
    if (!c.host_only && is_capturing(st)) {
        lora_worklists_free(&w);
        return LORA_E_STATE;
    }
    // the staged copy may still be the source of an earlier upload; the device copy may still be read
    // by earlier applies
    if (p.upload_pending) {
        const hipError_t e = hipEventSynchronize(p.ev_upload);
        if (e != hipSuccess) {
            lora_worklists_free(&w);
            g_last_hip = (int)e;
            return LORA_E_HIP;
        }
        p.upload_pending = false;
    }
    std::memcpy(p.pinned, w.tok_list, sizeof(int32_t) * (size_t)w.n_tok_list);
    std::memcpy(p.pinned + p.off_tiles, w.tiles, sizeof(lora_item_t) * (size_t)w.n_tiles);
    lora_worklists_free(&w);
    if (!gs.empty()) std::memcpy(p.pinned + p.off_gs, gs.data(), sizeof(lora::GemvItem) * gs.size());
    if (!ge.empty()) std::memcpy(p.pinned + p.off_ge, ge.data(), sizeof(lora::GemvItem) * ge.size());
    if (!lin_tok.empty()) std::memcpy(p.pinned + p.off_lin_tok, lin_tok.data(), sizeof(int32_t) * lin_tok.size());
    if (!lin_tiles.empty()) std::memcpy(p.pinned + p.off_lin_tiles, lin_tiles.data(), sizeof(lora::DevItem) * lin_tiles.size());
    for (int v = 0; v < SHRINK_VARIANTS; ++v) {
        if (!shrink_runs[v].cuts.empty()) std::memcpy(p.pinned + p.off_cuts[v], shrink_runs[v].cuts.data(), sizeof(lora::ShrinkCut) * shrink_runs[v].cuts.size());
        if (!shrink_runs[v].sums.empty()) std::memcpy(p.pinned + p.off_sums[v], shrink_runs[v].sums.data(), sizeof(lora::ShrinkSum) * shrink_runs[v].sums.size());
    }
    p.bytes = bytes;
    p.build_seq = ++c.plan_builds;
    if (!c.host_only && bytes) {
        if (p.use_pending) {
            HIP_TRY(hipStreamWaitEvent(st, p.ev_last_use, 0));
            p.use_pending = false;
        }
        HIP_TRY(hipMemcpyAsync(p.dev, p.pinned, bytes, hipMemcpyHostToDevice, st));
        HIP_TRY(hipEventRecord(p.ev_upload, st));
        p.upload_pending = true;
    }
    return LORA_OK;
}

// Makes `st` wait for every apply enqueued so far that named the slot.  The fence of the call that
// used it last sits in a ring; once that entry has been taken over by a later call, the latest fence
// of every stream that ever ran applies stands in (stream order covers the older ones).
int wait_for_applies(lora_cache &c, const Slot &s, hipStream_t st)
{
    if (!c.fencing || s.last_used <= 0) return LORA_OK;
    const int e = (int)(s.last_used % N_APPLY_EVENTS);
    if (c.apply_ev_seq[e] == s.last_used) {
        HIP_TRY(hipStreamWaitEvent(st, c.apply_ev[e], 0));
    } else {
        for (const auto &kv : c.stream_fence) HIP_TRY(hipStreamWaitEvent(st, kv.second, 0));
    }
    return LORA_OK;
}

hipEvent_t take_event(lora_cache &c)
{
    if (!c.free_events.empty()) {
        hipEvent_t e = c.free_events.back();
        c.free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// KernelTimer callback: two events from the pool, remembered with the kernel kind.
void timer_pair(void *ctx, int kind, hipEvent_t *start, hipEvent_t *stop)
{
    lora_cache &c = *static_cast<lora_cache *>(ctx);
    lora_cache::Timed t{kind, take_event(c), take_event(c)};
    if (!t.start || !t.stop) return;  // the launch then goes untimed
    c.timed.push_back(t);
    *start = t.start;
    *stop = t.stop;
}

}  // namespace

// ------------------------------------------------------------------------------------------
extern "C" {

const char *lora_strerror(int status)
{
    switch (status) {
        case LORA_OK: return "ok";
        case LORA_E_INVAL: return "invalid argument";
        case LORA_E_STATE: return "cache slot in the wrong state";
        case LORA_E_NOMEM: return "out of pool / plan / host memory";
        case LORA_E_HIP: return "HIP call failed";
        case LORA_E_NOTFOUND: return "adapter not cached";
        case LORA_E_FAULT: return "a kernel of an earlier apply gave up a bounded wait";
        default: return "unknown status";
    }
}

int lora_last_hip_error(void) { return g_last_hip; }

size_t lora_adapter_bytes(int32_t h_in, int32_t h_out, int32_t rank, int32_t dtype)
{
    if (h_in < 1 || h_out < 1 || rank < 1 || (dtype != LORA_F32 && dtype != LORA_BF16)) return 0;
    return (size_t)rank * ((size_t)h_in + (size_t)h_out) * esize_of(dtype);
}

size_t lora_cache_bytes_required(const lora_cache_config_t *cfg)
{
    if (!config_ok(cfg)) return 0;
    lora_cache tmp;
    compute_layout(tmp, cfg);
    return tmp.total;
}

int lora_cache_create(const lora_cache_config_t *cfg, void *dev_pool, size_t dev_pool_bytes, lora_cache_t **out)
{
    if (!out) return LORA_E_INVAL;
    *out = nullptr;
    if (!config_ok(cfg)) return LORA_E_INVAL;
    lora_cache *c = new (std::nothrow) lora_cache;
    if (!c) return LORA_E_NOMEM;
    compute_layout(*c, cfg);
    c->slots.resize(c->n_slots);
    for (int32_t s = 0; s < c->n_slots; ++s) {
        c->slots[s].cls = class_of_slot(*c, s);
        c->slots[s].part.assign((size_t)c->n_layers * c->proj.size(), 0);
    }
    c->plans.resize(c->n_user_plans + N_INTERNAL_PLANS);
    for (size_t i = 0; i < c->plans.size(); ++i) c->plans[i].internal = (int)i >= c->n_user_plans;
    if (c->host_only) {
        // plans are still built (and can be inspected with lora_plan_dump), only never uploaded
        for (auto &p : c->plans) {
            p.pinned = static_cast<char *>(std::malloc(c->plan_cap));
            if (!p.pinned) {
                lora_cache_destroy(c);
                return LORA_E_NOMEM;
            }
        }
        *out = c;
        return LORA_OK;
    }
    if (!dev_pool || (reinterpret_cast<uintptr_t>(dev_pool) & (ALIGN - 1))) {
        delete c;
        return LORA_E_INVAL;
    }
    if (dev_pool_bytes < c->total) {
        delete c;
        return LORA_E_NOMEM;
    }
    c->pool = static_cast<char *>(dev_pool);
    c->pool_bytes = dev_pool_bytes;
    if (hipGetDevice(&c->device) != hipSuccess) {
        g_last_hip = (int)hipGetLastError();
        delete c;
        return LORA_E_HIP;
    }
    {
        int n_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && n_cu > 0) c->n_cu = n_cu;
        else (void)hipGetLastError();
    }
    if (const int rc_s = static_scratch_setup(c->device)) {
        delete c;
        return rc_s;
    }

    int rc = LORA_OK;
    // the tagged words must not carry a future launch number by accident: numbers start at 1
    if (hipHostMalloc(reinterpret_cast<void **>(&c->fault_host), 64, hipHostMallocMapped) != hipSuccess ||
        hipHostGetDevicePointer(reinterpret_cast<void **>(&c->fault_dev), c->fault_host, 0) != hipSuccess ||
        (*c->fault_host = 0, false) ||
        hipMemset(c->pool + c->off_vtag, 0, c->vtag_set_bytes * N_VSETS) != hipSuccess ||
        hipMemset(c->pool + c->off_fault, 0, sizeof(uint32_t) * N_LINEAR_FLAGS) != hipSuccess) {
        g_last_hip = (int)hipGetLastError();
        delete c;
        return LORA_E_HIP;
    }
    auto fail = [&](hipError_t e) {
        if (e != hipSuccess && rc == LORA_OK) {
            g_last_hip = (int)e;
            rc = LORA_E_HIP;
        }
    };
    for (size_t i = 0; i < c->plans.size() && rc == LORA_OK; ++i) {
        lora_plan &p = c->plans[i];
        p.dev = c->pool + c->off_plans + c->plan_cap * i;
        fail(hipHostMalloc(reinterpret_cast<void **>(&p.pinned), c->plan_cap, hipHostMallocDefault));
        fail(hipEventCreateWithFlags(&p.ev_upload, hipEventDisableTiming));
        fail(hipEventCreateWithFlags(&p.ev_last_use, hipEventDisableTiming));
    }
    for (int i = 0; i < N_STAGES && rc == LORA_OK; ++i) {
        c->stage[i].dev = c->pool + c->off_stage + c->stage_cap * i;
        fail(hipEventCreateWithFlags(&c->stage[i].ev, hipEventDisableTiming));
    }
    for (int i = 0; i < N_APPLY_EVENTS && rc == LORA_OK; ++i) fail(hipEventCreateWithFlags(&c->apply_ev[i], hipEventDisableTiming));
    if (rc == LORA_OK && !(c->flags & LORA_CACHE_NO_OVERLAP)) {
        fail(hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking));
        fail(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
        fail(hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming));
    }
    if (rc != LORA_OK) {
        lora_cache_destroy(c);
        return rc;
    }
    *out = c;
    return LORA_OK;
}

int lora_cache_destroy(lora_cache_t *c)
{
    if (!c) return LORA_E_INVAL;
    if (c->host_only) {
        for (auto &p : c->plans) std::free(p.pinned);
    } else {
        for (auto &p : c->plans) {
            if (p.pinned) (void)hipHostFree(p.pinned);
            if (p.ev_upload) (void)hipEventDestroy(p.ev_upload);
            if (p.ev_last_use) (void)hipEventDestroy(p.ev_last_use);
        }
        for (auto &s : c->stage)
            if (s.ev) (void)hipEventDestroy(s.ev);
        for (auto &e : c->apply_ev)
            if (e) (void)hipEventDestroy(e);
        for (auto &kv : c->stream_fence)
            if (kv.second) (void)hipEventDestroy(kv.second);
        if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
        if (c->ev_join) (void)hipEventDestroy(c->ev_join);
        if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
        if (c->fault_host) (void)hipHostFree(c->fault_host);
        for (auto &s : c->slots)
            if (s.fill_ev) (void)hipEventDestroy(s.fill_ev);
        for (auto &t : c->timed) {
            (void)hipEventDestroy(t.start);
            (void)hipEventDestroy(t.stop);
        }
        for (auto &e : c->free_events) (void)hipEventDestroy(e);
    }
    delete c;
    return LORA_OK;
}

// The address under which the device sees pinned (page-locked, mapped) host memory, or null for
// any other kind of pointer.
static const void *device_view_of_pinned(const void *host)
{
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, host) != hipSuccess) {
        (void)hipGetLastError();  // pageable memory is reported as an error by some runtimes
        return nullptr;
    }
    return at.type == hipMemoryTypeHost ? at.devicePointer : nullptr;
}

int lora_cache_fill_slot(lora_cache_t *c, int32_t slot, int64_t adapter_id, int32_t rank, float alpha, int32_t layer,
                         int32_t proj, const void *host_A, const void *host_B, void *fill_stream)
{
    if (!c || slot < 0 || slot >= c->n_slots || layer < 0 || layer >= c->n_layers || proj < 0 ||
        proj >= (int32_t)c->proj.size() || rank < 1)
        return LORA_E_INVAL;
    Slot &s = c->slots[slot];
    if (rank > c->class_rank[s.cls]) return LORA_E_INVAL;
    if (!c->host_only && (!host_A || !host_B)) return LORA_E_INVAL;
    const size_t part = (size_t)layer * c->proj.size() + proj;

    const bool was_bound = s.bound;
    if (s.bound) {
        if (s.adapter_id != adapter_id || s.rank != rank || s.alpha != alpha) return LORA_E_STATE;
        if (s.part[part] && s.refcount > 0) return LORA_E_STATE;  // would overwrite data in use
    } else {
        auto other = c->id2slot.find(adapter_id);
        if (other != c->id2slot.end()) return LORA_E_STATE;  // the adapter is already cached elsewhere
        s.bound = true;
        s.adapter_id = adapter_id;
        s.rank = rank;
        s.alpha = alpha;
        s.use_count = 0;
        ++s.generation;
        c->id2slot[adapter_id] = slot;
    }

    const int32_t h_in = c->proj[proj].h_in, h_out = c->proj[proj].h_out;
    const size_t bytes_a = (size_t)rank * h_in * c->esize, bytes_b = (size_t)rank * h_out * c->esize;
    if (!c->host_only) {
        hipStream_t st = static_cast<hipStream_t>(fill_stream);
        // a HIP failure below must not leave a bound, empty entry behind
        struct Rollback {
            lora_cache *c;
            Slot *s;
            bool armed;
            ~Rollback()
            {
                if (armed) unbind(*c, *s);
            }
        } rollback{c, &s, !was_bound};
        // applies enqueued earlier may still read this slab; an earlier fill of the slot (of the entry it
        // held before, or of the same part) may still be writing it on another stream
        if (int rc = wait_for_applies(*c, s, st)) return rc;
        if (s.fill_pending) HIP_TRY(hipStreamWaitEvent(st, s.fill_ev, 0));
        char *slab = slab_ptr(*c, layer, proj, slot);
        const void *dev_A = c->direct_fill ? device_view_of_pinned(host_A) : nullptr;
        const void *dev_B = c->direct_fill ? device_view_of_pinned(host_B) : nullptr;
        if (dev_A && dev_B && ((reinterpret_cast<uintptr_t>(dev_A) | reinterpret_cast<uintptr_t>(dev_B)) & 15) == 0) {
            // pinned host memory is mapped into the device's address space: the repack kernel reads
            // it over PCIe itself (fastest for a fill that has the device to itself; kernels that
            // wait on PCIe reads slow concurrent applies down far more than copy engines do)
            HIP_TRY(lora::launch_repack(c->dtype, dev_A, dev_B, slab, h_in, h_out, rank, true, st));
        } else {
            // copy engine -> staging buffer -> repack, all on the caller's stream.  (Copies on a
            // stream of the cache's own, to overlap them with the repack of the part before, made
            // every call block on the host for ~300 us with this runtime.)
            Stage &sg = c->stage[c->stage_next++ % N_STAGES];
            if (sg.pending) HIP_TRY(hipStreamWaitEvent(st, sg.ev, 0));
            char *stage_b = sg.dev + align_up(bytes_a);
            HIP_TRY(hipMemcpyAsync(sg.dev, host_A, bytes_a, hipMemcpyHostToDevice, st));
            HIP_TRY(hipMemcpyAsync(stage_b, host_B, bytes_b, hipMemcpyHostToDevice, st));
            HIP_TRY(lora::launch_repack(c->dtype, sg.dev, stage_b, slab, h_in, h_out, rank, false, st));
            HIP_TRY(hipEventRecord(sg.ev, st));
            sg.pending = true;
        }
        if (!s.fill_ev) HIP_TRY(hipEventCreateWithFlags(&s.fill_ev, hipEventDisableTiming));
        HIP_TRY(hipEventRecord(s.fill_ev, st));
        s.fill_pending = true;
        rollback.armed = false;
    }
    if (!s.part[part]) {
        s.part[part] = 1;
        ++s.parts_filled;
    }
    ++c->stats.fills;
    c->stats.bytes_filled += (int64_t)(bytes_a + bytes_b);
    return LORA_OK;
}

int lora_cache_fill_slot_parts(lora_cache_t *c, int32_t slot, int64_t adapter_id, int32_t rank, float alpha,
                               const lora_fill_part_t *parts, int32_t n_parts, void *fill_stream)
{
    if (!c || slot < 0 || slot >= c->n_slots || rank < 1 || n_parts < 0 || (n_parts > 0 && !parts)) return LORA_E_INVAL;
    Slot &s = c->slots[slot];
    if (rank > c->class_rank[s.cls]) return LORA_E_INVAL;
    bool direct = c->direct_fill && !c->host_only;
    for (int32_t i = 0; i < n_parts; ++i) {
        const lora_fill_part_t &q = parts[i];
        if (q.layer < 0 || q.layer >= c->n_layers || q.proj < 0 || q.proj >= (int32_t)c->proj.size()) return LORA_E_INVAL;
        if (!c->host_only && (!q.host_A || !q.host_B)) return LORA_E_INVAL;
        if (s.bound && s.part[(size_t)q.layer * c->proj.size() + q.proj] && s.refcount > 0) return LORA_E_STATE;
    }
    if (s.bound) {
        if (s.adapter_id != adapter_id || s.rank != rank || s.alpha != alpha) return LORA_E_STATE;
    } else if (c->id2slot.find(adapter_id) != c->id2slot.end()) {
        return LORA_E_STATE;
    }
    if (n_parts == 0) return LORA_OK;
    // pinned host arrays as the device sees them (all parts, or the call takes the staged way)
    std::vector<const void *> dev_view;
    if (direct) {
        dev_view.resize(2 * (size_t)n_parts);
        for (int32_t i = 0; i < n_parts && direct; ++i) {
            dev_view[2 * i] = device_view_of_pinned(parts[i].host_A);
            dev_view[2 * i + 1] = device_view_of_pinned(parts[i].host_B);
            if (!dev_view[2 * i] || !dev_view[2 * i + 1] ||
                ((reinterpret_cast<uintptr_t>(dev_view[2 * i]) | reinterpret_cast<uintptr_t>(dev_view[2 * i + 1])) & 15))
                direct = false;
        }
    }
    if (!direct) {
        for (int32_t i = 0; i < n_parts; ++i) {
            const int rc = lora_cache_fill_slot(c, slot, adapter_id, rank, alpha, parts[i].layer, parts[i].proj, parts[i].host_A,
                                                parts[i].host_B, fill_stream);
            if (rc != LORA_OK) return rc;
        }
        return LORA_OK;
    }
    const bool was_bound = s.bound;
    if (!s.bound) {
        s.bound = true;
        s.adapter_id = adapter_id;
        s.rank = rank;
        s.alpha = alpha;
        s.use_count = 0;
        ++s.generation;
        c->id2slot[adapter_id] = slot;
    }
    hipStream_t st = static_cast<hipStream_t>(fill_stream);
    struct Rollback {
        lora_cache *c;
        Slot *s;
        bool armed;
        ~Rollback()
        {
            if (armed) unbind(*c, *s);
        }
    } rollback{c, &s, !was_bound};
    if (int rc = wait_for_applies(*c, s, st)) return rc;
    if (s.fill_pending) HIP_TRY(hipStreamWaitEvent(st, s.fill_ev, 0));
    for (int32_t i0 = 0; i0 < n_parts; i0 += lora::REPACK_MAX_PARTS) {
        lora::RepackTable t;
        t.n = std::min<int32_t>(lora::REPACK_MAX_PARTS, n_parts - i0);
        for (int32_t i = 0; i < t.n; ++i) {
            const lora_fill_part_t &q = parts[i0 + i];
            t.p[i].A = dev_view[2 * (size_t)(i0 + i)];
            t.p[i].B = dev_view[2 * (size_t)(i0 + i) + 1];
            t.p[i].slab = slab_ptr(*c, q.layer, q.proj, slot);
            t.p[i].h_in = c->proj[q.proj].h_in;
            t.p[i].h_out = c->proj[q.proj].h_out;
        }
        HIP_TRY(lora::launch_repack_parts(c->dtype, t, rank, true, st));
    }
    if (!s.fill_ev) HIP_TRY(hipEventCreateWithFlags(&s.fill_ev, hipEventDisableTiming));
    HIP_TRY(hipEventRecord(s.fill_ev, st));
    s.fill_pending = true;
    rollback.armed = false;
    for (int32_t i = 0; i < n_parts; ++i) {
        const lora_fill_part_t &q = parts[i];
        const size_t part = (size_t)q.layer * c->proj.size() + q.proj;
        if (!s.part[part]) {
            s.part[part] = 1;
            ++s.parts_filled;
        }
        ++c->stats.fills;
        c->stats.bytes_filled += (int64_t)rank * (c->proj[q.proj].h_in + c->proj[q.proj].h_out) * c->esize;
    }
    return LORA_OK;
}

int lora_cache_release_slot(lora_cache_t *c, int32_t slot)
{
    if (!c || slot < 0 || slot >= c->n_slots) return LORA_E_INVAL;
    Slot &s = c->slots[slot];
    if (s.refcount > 0) return LORA_E_STATE;
    if (s.bound) ++c->stats.evictions;
    unbind(*c, s);
    return LORA_OK;
}

int lora_cache_slot_ref(lora_cache_t *c, int32_t slot, int32_t delta)
{
    if (!c || slot < 0 || slot >= c->n_slots) return LORA_E_INVAL;
    Slot &s = c->slots[slot];
    if (!s.bound) return LORA_E_STATE;
    if (s.refcount + delta < 0) return LORA_E_STATE;
    s.refcount += delta;
    return LORA_OK;
}

int lora_cache_lookup(lora_cache_t *c, int64_t adapter_id, int32_t *slot, int32_t *rank)
{
    if (!c) return LORA_E_INVAL;
    auto it = c->id2slot.find(adapter_id);
    if (it == c->id2slot.end()) {
        ++c->stats.misses;
        return LORA_E_NOTFOUND;
    }
    ++c->stats.hits;
    if (slot) *slot = it->second;
    if (rank) *rank = c->slots[it->second].rank;
    return LORA_OK;
}

int lora_cache_slot_info(lora_cache_t *c, int32_t slot, lora_slot_info_t *out)
{
    if (!c || !out || slot < 0 || slot >= c->n_slots) return LORA_E_INVAL;
    Slot &s = c->slots[slot];
    out->adapter_id = s.adapter_id;
    out->rank = s.rank;
    out->class_rank = c->class_rank[s.cls];
    out->state = slot_state(*c, s);
    out->refcount = s.refcount;
    out->use_count = s.use_count;
    out->last_used = s.last_used;
    out->alpha = s.alpha;
    out->parts_filled = s.parts_filled;
    return LORA_OK;
}

int lora_cache_slot_state(lora_cache_t *c, int32_t slot, int32_t *state)
{
    if (!c || !state || slot < 0 || slot >= c->n_slots) return LORA_E_INVAL;
    *state = slot_state(*c, c->slots[slot]);
    return LORA_OK;
}

int lora_cache_find_free_slot(lora_cache_t *c, int32_t rank, int32_t *slot)
{
    if (!c || !slot || rank < 1) return LORA_E_INVAL;
    for (size_t k = 0; k < c->class_rank.size(); ++k) {
        if (c->class_rank[k] < rank) continue;
        for (int32_t s = c->class_first[k]; s < c->class_first[k] + c->class_slots[k]; ++s)
            if (!c->slots[s].bound) {
                *slot = s;
                return LORA_OK;
            }
    }
    return LORA_E_NOMEM;
}

int lora_cache_set_policy(lora_cache_t *c, const lora_policy_t *p)
{
    if (!c || !p || !(p->w_freq >= 0) || !(p->w_recency >= 0) || !(p->w_size >= 0) || p->freq_window < 0) return LORA_E_INVAL;
    c->policy = *p;
    return LORA_OK;
}

int lora_cache_get_policy(const lora_cache_t *c, lora_policy_t *p)
{
    if (!c || !p) return LORA_E_INVAL;
    *p = c->policy;
    return LORA_OK;
}

int lora_cache_score(lora_cache_t *c, int32_t slot, double *score)
{
    if (!c || !score || slot < 0 || slot >= c->n_slots) return LORA_E_INVAL;
    if (!c->slots[slot].bound) return LORA_E_STATE;
    *score = eviction_scores(*c)[slot];
    return LORA_OK;
}

int lora_cache_choose_victim(lora_cache_t *c, int32_t rank, const int64_t *queued_ids, int32_t n_queued, int32_t *slot)
{
    if (!c || !slot || rank < 0 || n_queued < 0 || (n_queued > 0 && !queued_ids)) return LORA_E_INVAL;
    const int32_t v = choose_victim(*c, rank, queued_ids, n_queued);
    if (v < 0) return LORA_E_NOMEM;
    *slot = v;
    return LORA_OK;
}

int lora_cache_acquire(lora_cache_t *c, int64_t adapter_id, int32_t rank, float alpha, int32_t pin,
                       const int64_t *queued_ids, int32_t n_queued, int32_t *slot, int32_t *hit)
{
    if (!c || !slot || !hit || rank < 1 || n_queued < 0 || (n_queued > 0 && !queued_ids)) return LORA_E_INVAL;
    if (rank > c->class_rank.back()) return LORA_E_INVAL;
    auto touch = [&](Slot &s) {
        ++c->req_seq;
        if (c->policy.freq_window > 0 && c->req_seq % c->policy.freq_window == 0)
            for (Slot &o : c->slots) o.req_freq *= 0.5;
        s.req_freq += 1.0;
        s.req_last = c->req_seq;
        if (pin) ++s.refcount;
    };
    auto it = c->id2slot.find(adapter_id);
    if (it != c->id2slot.end()) {
        Slot &s = c->slots[it->second];
        if (s.rank != rank) return LORA_E_INVAL;
        ++c->stats.hits;
        touch(s);
        *slot = it->second;
        *hit = 1;
        return LORA_OK;
    }
    int32_t where = -1;
    if (lora_cache_find_free_slot(c, rank, &where) != LORA_OK) {
        where = choose_victim(*c, rank, queued_ids, n_queued);
        if (where < 0) return LORA_E_NOMEM;  // every large-enough entry is used by a running request
        ++c->stats.evictions;
        unbind(*c, c->slots[where]);
    }
    ++c->stats.misses;
    Slot &s = c->slots[where];
    s.bound = true;
    s.adapter_id = adapter_id;
    s.rank = rank;
    s.alpha = alpha;
    s.use_count = 0;
    ++s.generation;
    c->id2slot[adapter_id] = where;
    touch(s);
    *slot = where;
    *hit = 0;
    return LORA_OK;
}

int lora_cache_resident_bytes(const lora_cache_t *c, size_t *bytes)
{
    if (!c || !bytes) return LORA_E_INVAL;
    size_t sum = 0;
    for (const Slot &s : c->slots)
        if (s.bound) sum += entry_bytes(*c, s);
    *bytes = sum;
    return LORA_OK;
}

int lora_cache_trim(lora_cache_t *c, size_t max_bytes, const int64_t *queued_ids, int32_t n_queued, int32_t *n_evicted)
{
    if (!c || n_queued < 0 || (n_queued > 0 && !queued_ids)) return LORA_E_INVAL;
    size_t held = 0;
    lora_cache_resident_bytes(c, &held);
    int32_t n = 0;
    int rc = LORA_OK;
    while (held > max_bytes) {
        const int32_t v = choose_victim(*c, 0, queued_ids, n_queued);
        if (v < 0) {
            rc = LORA_E_NOMEM;  // what is left is in use
            break;
        }
        held -= entry_bytes(*c, c->slots[v]);
        ++c->stats.evictions;
        unbind(*c, c->slots[v]);
        ++n;
    }
    if (n_evicted) *n_evicted = n;
    return rc;
}

int lora_cache_stats(const lora_cache_t *c, lora_cache_stats_t *out)
{
    if (!c || !out) return LORA_E_INVAL;
    *out = c->stats;
    return LORA_OK;
}

int lora_cache_slab(const lora_cache_t *c, int32_t layer, int32_t proj, int32_t slot, void **dev_ptr, size_t *bytes)
{
    if (!c || layer < 0 || layer >= c->n_layers || proj < 0 || proj >= (int32_t)c->proj.size() || slot < 0 ||
        slot >= c->n_slots)
        return LORA_E_INVAL;
    if (dev_ptr)
        *dev_ptr = c->pool ? slab_ptr(*c, layer, proj, slot) : nullptr;
    if (bytes) *bytes = (size_t)lora::rank_storage(c->class_rank[c->slots[slot].cls]) * c->row_bytes[proj];
    return LORA_OK;
}

int lora_cache_set_fencing(lora_cache_t *c, int32_t on)
{
    if (!c) return LORA_E_INVAL;
    c->fencing = on != 0;
    return LORA_OK;
}

int lora_cache_check_fault(lora_cache_t *c, void *stream, int32_t *fault)
{
    if (!c || !fault || c->host_only) return LORA_E_INVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(hipStreamSynchronize(st));
    const int32_t v = __atomic_exchange_n(c->fault_host, 0, __ATOMIC_ACQ_REL);
    *fault = v ? 1 : 0;
    return LORA_OK;
}

int lora_cache_set_timing(lora_cache_t *c, int32_t on)
{
    if (!c || c->host_only) return LORA_E_INVAL;
    c->timing = on != 0;
    return LORA_OK;
}

int lora_cache_read_timing(lora_cache_t *c, double ms[LORA_K_COUNT], int64_t launches[LORA_K_COUNT])
{
    if (!c || !ms || !launches) return LORA_E_INVAL;
    for (int k = 0; k < LORA_K_COUNT; ++k) {
        ms[k] = 0.0;
        launches[k] = 0;
    }
    int rc = LORA_OK;
    for (auto &t : c->timed) {
        float el = 0.f;
        hipError_t e = hipEventSynchronize(t.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&el, t.start, t.stop);
        if (e == hipSuccess) {
            ms[t.kind] += el;
            ++launches[t.kind];
        } else {
            g_last_hip = (int)e;
            rc = LORA_E_HIP;
        }
        c->free_events.push_back(t.start);
        c->free_events.push_back(t.stop);
    }
    c->timed.clear();
    return rc;
}

int lora_plan_create(lora_cache_t *c, int32_t T, const int32_t *seg_offsets, const int32_t *seg_slot,
                     const int32_t *seg_rank, int32_t n_seg, void *stream, lora_plan_t **out)
{
    if (!c || !out) return LORA_E_INVAL;
    *out = nullptr;
    lora_plan *p = nullptr;
    for (int i = 0; i < c->n_user_plans; ++i)
        if (!c->plans[i].in_use) {
            p = &c->plans[i];
            break;
        }
    if (!p) return LORA_E_NOMEM;
    const int rc = build_plan(*c, *p, T, seg_offsets, seg_slot, seg_rank, n_seg, static_cast<hipStream_t>(stream));
    if (rc != LORA_OK) return rc;
    p->in_use = true;
    *out = p;
    return LORA_OK;
}

int lora_plan_destroy(lora_cache_t *c, lora_plan_t *p)
{
    if (!c || !p || p->internal || !p->in_use) return LORA_E_INVAL;
    if (p < c->plans.data() || p >= c->plans.data() + c->n_user_plans) return LORA_E_INVAL;
    p->in_use = false;
    return LORA_OK;
}

int lora_plan_info(const lora_plan_t *p, lora_plan_info_t *out)
{
    if (!p || !out || !p->in_use) return LORA_E_INVAL;
    out->T = p->T;
    out->mfma_min_tokens = p->mfma_min_used;
    out->n_tiles = p->n_tiles;
    out->n_tile_tokens = p->n_tile_tok;
    out->n_gemv_shrink_items = p->n_gs;
    out->n_gemv_expand_items = p->n_ge;
    return LORA_OK;
}

int lora_plan_dump(lora_cache_t *c, const lora_plan_t *p, int32_t proj, lora_plan_unit_t *units, int32_t cap_units,
                   int32_t *n_units, int32_t *toks, int32_t cap_toks, int32_t *n_toks)
{
    if (!c || !p || !p->in_use || !n_units || !n_toks || proj < 0 || proj >= (int32_t)c->proj.size() || cap_units < 0 ||
        cap_toks < 0 || (cap_units > 0 && !units) || (cap_toks > 0 && !toks))
        return LORA_E_INVAL;
    // the bytes the kernels read
    std::vector<char> copy;
    const char *buf = p->pinned;
    if (!c->host_only) {
        copy.resize(p->bytes);
        if (p->upload_pending) HIP_TRY(hipEventSynchronize(p->ev_upload));
        if (p->bytes) HIP_TRY(hipMemcpy(copy.data(), p->dev, p->bytes, hipMemcpyDeviceToHost));
        buf = copy.data();
    }
    const int32_t *tok_list = reinterpret_cast<const int32_t *>(buf);
    const lora::DevItem *tiles = reinterpret_cast<const lora::DevItem *>(buf + p->off_tiles);
    const lora::GemvItem *gs = reinterpret_cast<const lora::GemvItem *>(buf + p->off_gs);
    const lora::GemvItem *ge = reinterpret_cast<const lora::GemvItem *>(buf + p->off_ge);
    const int32_t *lin_tok = reinterpret_cast<const int32_t *>(buf + p->off_lin_tok);
    const lora::DevItem *lin_tiles = reinterpret_cast<const lora::DevItem *>(buf + p->off_lin_tiles);

    int32_t nu = 0, nt = 0;
    auto slot_of_row = [&](int32_t row) -> int32_t {
        auto it = std::upper_bound(c->slot_row.begin(), c->slot_row.end(), row);
        return (int32_t)(it - c->slot_row.begin()) - 1;
    };
    auto put_tok = [&](int32_t t) {
        if (nt < cap_toks) toks[nt] = t;
        ++nt;
    };
    auto put_unit = [&](int32_t kind, int32_t tok_off, int32_t n_tok, int32_t row, int32_t rank, int32_t lo, int32_t hi,
                        int32_t where, float alpha) {
        if (nu < cap_units) units[nu] = lora_plan_unit_t{kind, tok_off, n_tok, row >= 0 ? slot_of_row(row) : -1, rank, lo, hi, where, alpha};
        ++nu;
    };
    // tokens of a tile as the tile kernels find them: a run from tok0, or through the token list
    auto tile_tokens = [&](const lora::DevItem &it, const int32_t *list) {
        for (int32_t i = 0; i < it.n_tok; ++i) put_tok(lora::tile_token_of(list, it, i));
    };
    std::vector<int32_t> tile_off((size_t)p->n_tiles, 0);
    for (int32_t i = 0; i < p->n_tiles; ++i) {
        tile_off[i] = nt;
        tile_tokens(tiles[i], tok_list);
        put_unit(LORA_UNIT_TILE, tile_off[i], tiles[i].n_tok, tiles[i].row, tiles[i].rank, 0, 0, 0, tiles[i].alpha);
    }
    // the tile shrink's pieces for this projection's h_in, per run table, walked as the kernel walks them; and the
    // scratch slots the reduce adds up per tile
    for (int v = 0; v < SHRINK_VARIANTS && p->n_tiles > 0; ++v) {
        if (p->shrink_runs[v] == 0) continue;  // (no such table: the batch is too large for the call it serves)
        const lora::ShrinkCut *cuts = reinterpret_cast<const lora::ShrinkCut *>(buf + p->off_cuts[v]);
        const lora::ShrinkSum *sums = reinterpret_cast<const lora::ShrinkSum *>(buf + p->off_sums[v]);
        const int32_t quanta = p->shrink_quanta, h_in = c->proj[proj].h_in, SK = lora::SHRINK_STAGE_K;
        for (int32_t r = 0; r < p->shrink_runs[v]; ++r) {
            const lora::ShrinkCut from = cuts[r], to = cuts[r + 1];
            const int32_t last_tile = std::min(to.part > 0 ? to.tile : to.tile - 1, p->n_tiles - 1);
            for (int32_t t = from.tile; t <= last_tile; ++t) {
                const int32_t lo = t == from.tile ? from.part : 0, hi = t == to.tile ? to.part : quanta;
                if (lo >= hi) continue;
                const int32_t k_begin = lora::shrink_part_stage(lo, quanta, h_in, SK) * SK;
                const int32_t k_end = std::min(h_in, lora::shrink_part_stage(hi, quanta, h_in, SK) * SK);
                const bool whole = lo == 0 && hi == quanta;
                put_unit(LORA_UNIT_TILE_SHRINK, tile_off[t], tiles[t].n_tok, tiles[t].row, tiles[t].rank, k_begin, k_end,
                         (v << 20) | r, whole ? -1.f : (float)lora::shrink_slot(r, from.tile, t));
            }
        }
        for (int32_t t = 0; t < p->n_tiles; ++t)
            for (int32_t j = 0; j < sums[t].n_pieces && sums[t].n_pieces > 1; ++j)
                put_unit(LORA_UNIT_TILE_SUM, tile_off[t], tiles[t].n_tok, tiles[t].row, tiles[t].rank, j, sums[t].n_pieces, v << 20,
                         (float)(j == 0 ? sums[t].first_slot : 2 * (sums[t].first_slot / 2 + j)));
    }
    auto gemv_tokens = [&](const lora::GemvItem &it) -> int32_t {
        int32_t n = 0;
        for (int t = 0; t < lora::GEMV_BATCH; ++t)
            if (it.tok[t] >= 0) {
                put_tok(it.tok[t]);
                ++n;
            }
        return n;
    };
    // the GEMV launch of this projection alone: blocks and units mapped to items as the kernel maps them
    for (uint32_t b = 0; b < (uint32_t)p->n_gs; ++b) {
        uint32_t item, pj;
        lora::gemv_shrink_block(b, (uint32_t)p->n_gs, 1u, item, pj);
        int32_t j0, n;
        lora::gemv_shrink_rows(gs[item], j0, n);
        const int32_t off = nt, cnt = gemv_tokens(gs[item]);
        put_unit(LORA_UNIT_GEMV_SHRINK, off, cnt, gs[item].row, gs[item].rank, j0, j0 + n, (int32_t)b, gs[item].alpha);
    }
    lora::GemvMap gm{};
    const int32_t h_out = c->proj[proj].h_out, n_super = (h_out + lora::GEMV_SUPER_COLS - 1) / lora::GEMV_SUPER_COLS;
    for (int i = 0; i < lora::GEMV_MAX_PROJS; ++i) {
        gm.unit_end[i] = p->n_ge * n_super;
        gm.n_super_packed |= (uint32_t)n_super << (8 * i);
        gm.super_magic[i] = lora::gemv_magic((uint32_t)n_super);
    }
    for (uint32_t u = 0; u < (uint32_t)gm.unit_end[0]; ++u) {
        uint32_t pj, item, sc;
        lora::gemv_expand_unit(u, gm, pj, item, sc);
        int32_t c0, c1;
        lora::gemv_expand_cols(ge[item], (int32_t)sc, h_out, c0, c1);
        if (c0 >= c1) continue;  // the wavefront returns at once
        const int32_t off = nt, cnt = gemv_tokens(ge[item]);
        put_unit(LORA_UNIT_GEMV_EXPAND, off, cnt, ge[item].row, ge[item].rank, c0, c1, 0, ge[item].alpha);
    }
    for (int32_t i = 0; i < p->n_lin_tiles; ++i) {
        const int32_t off = nt;
        tile_tokens(lin_tiles[i], lin_tok);
        const bool tile = i < p->n_tiles;
        put_unit(LORA_UNIT_LINEAR_ROWS, off, lin_tiles[i].n_tok, tile ? lin_tiles[i].row : -1, tile ? lin_tiles[i].rank : 0, 0, 0,
                 tile ? 2 : lin_tiles[i].a, tile ? lin_tiles[i].alpha : 0.f);
    }
    *n_units = nu;
    *n_toks = nt;
    return LORA_OK;
}

static int validate_apply(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x, void *base_out)
{
    if (c->fault_host && __atomic_load_n(c->fault_host, __ATOMIC_ACQUIRE)) return LORA_E_FAULT;
    if (layer < 0 || layer >= c->n_layers || proj < 0 || proj >= (int32_t)c->proj.size()) return LORA_E_INVAL;
    if (p->T > 0 && (!x || !base_out || !aligned16(x) || !aligned16(base_out))) return LORA_E_INVAL;
    const size_t part = (size_t)layer * c->proj.size() + proj;
    for (size_t i = 0; i < p->slots.size(); ++i) {
        const Slot &s = c->slots[p->slots[i]];
        if (!s.bound || s.generation != p->generations[i] || !s.part[part]) return LORA_E_STATE;
    }
    return LORA_OK;
}

// shrink items up to which the one-launch GEMV form is chosen: measured faster than two launches up to
// 7726 items (2048 one-token requests over 300 adapters: 83 against 86 us); not measured beyond
constexpr int FUSED_GEMV_MAX_ITEMS = 8192;

// Applies descs[0 .. n), n <= N_VSETS: one projection, or several that read the same x and do not
// write to it.  Those run shrink-first, each with its own copy of the intermediate buffers: one
// tile-shrink launch for all of them (x is then fetched from memory once), their GEMV launches,
// then their expands.
static Scratch pool_scratch(lora_cache_t *c)
{
    return Scratch{c->pool + c->off_v, c->v_set_bytes, N_VSETS, c->pool + c->off_vpart, c->vpart_rows, false,
                   c->pool + c->off_vtag, c->vtag_set_bytes, &c->tag_epoch, &c->cap_id, &c->cap_plan, &c->cap_sets};
}

// The run table of a tile-shrink launch for n projections, and where their partial sums go in `vpart`.
static int shrink_setup(const lora_cache_t *c, const lora_plan_t *p, int n, char *vpart, int64_t vpart_rows, bool small, lora::ShrinkProjs &ps)
{
    const int v = small ? SHRINK_VARIANT_SMALL : n - 1;
    if (n < 1 || n > lora::MAX_SHRINK_PROJS || (small && n != 1)) return LORA_E_INVAL;
    ps.n = n;
    ps.n_runs = p->shrink_runs[v];
    if (p->n_tiles > 0 && ps.n_runs == 0) return LORA_E_STATE;  // the plan carries no such table
    ps.quanta = p->shrink_quanta;
    ps.any_pieces = p->shrink_pieces[v] ? 1 : 0;
    ps.cuts = reinterpret_cast<const lora::ShrinkCut *>(p->dev + p->off_cuts[v]);
    ps.sums = reinterpret_cast<const lora::ShrinkSum *>(p->dev + p->off_sums[v]);
    const int64_t rows_per_proj = 2 * (int64_t)lora::SHRINK_SLOT_ROWS * ps.n_runs;
    if (rows_per_proj * n > vpart_rows) return LORA_E_NOMEM;
    for (int i = 0; i < lora::MAX_SHRINK_PROJS; ++i)
        ps.part[i] = i < n ? reinterpret_cast<float *>(vpart) + (size_t)i * rows_per_proj * c->v_stride : nullptr;
    return LORA_OK;
}

// The GEMV part of a group of n projections that read the same x: one launch with the in-kernel
// hand-over when the part is small (the launch in between then costs more than the hand-over), else a
// shrink and an expand launch.  y32[i], when set, receives projection i's update as fp32 instead of y.
static int enqueue_gemv(lora_cache_t *c, lora_plan_t *p, const lora::ApplyArgs *a, float *const *y32, int n, bool allow_one_launch,
                        hipStream_t st, const Scratch &sc, const lora::KernelTimer *tm)
{
    if (p->n_gs <= 0) return LORA_OK;
    lora::GemvArgs ga{};
    lora::GemvMap gm{};
    ga.x = a[0].x;
    gm.gs = reinterpret_cast<const lora::GemvItem *>(p->dev + p->off_gs);
    gm.ge = reinterpret_cast<const lora::GemvItem *>(p->dev + p->off_ge);
    gm.n_gs = (uint32_t)p->n_gs;
    gm.n_proj_phase = (uint32_t)n;
    ga.fault = c->fault_dev;
    ga.h_in = a[0].h_in;
    ga.n_ge = p->n_ge;
    ga.scale = a[0].scale;
    int64_t units = 0;
    for (int i = 0; i < lora::GEMV_MAX_PROJS; ++i) {
        const int k = std::min(i, n - 1);  // entries past the group repeat its last
        lora::GemvProj &q = ga.p[i];
        q.proj_base = a[k].proj_base;
        q.row_bytes = a[k].row_bytes;
        q.y = a[k].y;
        q.y32 = y32 ? y32[k] : nullptr;
        q.vw = reinterpret_cast<unsigned long long *>(sc.vtag + (size_t)k * sc.vtag_set_bytes);
        q.h_out = a[k].h_out;
        const int32_t n_super = (a[k].h_out + lora::GEMV_SUPER_COLS - 1) / lora::GEMV_SUPER_COLS;
        if (n_super > 255) return LORA_E_INVAL;  // beyond the kernels' unit arithmetic
        gm.n_super_packed |= (uint32_t)n_super << (8 * i);
        gm.super_magic[i] = lora::gemv_magic((uint32_t)n_super);
        if (i < n) units += (int64_t)p->n_ge * n_super;
        gm.unit_end[i] = (int32_t)std::min<int64_t>(units, INT32_MAX);
    }
    if (units >= (1 << 24) || (int64_t)p->n_gs * n >= (1 << 24)) return LORA_E_INVAL;  // beyond the kernels' unit arithmetic
    // (after 2^32 - 1 one-launch applies the numbers would repeat: two launches from then on)
    const bool one = allow_one_launch && *sc.epoch < UINT32_MAX - 1 &&
                     (c->fused_gemv == 2 || (c->fused_gemv == 1 && (int64_t)p->n_gs * n <= FUSED_GEMV_MAX_ITEMS));
    if (one) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        unsigned long long cap = 0;
        if (hipStreamGetCaptureInfo(st, &cs, &cap) != hipSuccess) {
            (void)hipGetLastError();
            cs = hipStreamCaptureStatusNone;
        }
        if (cs != hipStreamCaptureStatusNone) {
            // A graph freezes the launch number, so a replay could take the words its own launch wrote in the
            // replay before for fresh ones.  Not when another launch of the same graph has written the same
            // words in between (its number differs): that holds for every launch after the first of a capture
            // that works on the same plan with at least as many projections.  Otherwise the words are cleared
            // first, by a small kernel that becomes part of the graph.
            const bool covered = cap == *sc.cap_id && p->build_seq == *sc.cap_plan && n <= *sc.cap_sets;
            if (!covered) {
                const int32_t *toks = reinterpret_cast<const int32_t *>(p->dev) + p->n_tile_tok;
                for (int i = 0; i < n; ++i) HIP_TRY(lora::launch_gemv_clear(c->dtype, ga.p[i].vw, toks, p->n_tok_list - p->n_tile_tok, st));
            }
            *sc.cap_id = cap;
            *sc.cap_plan = p->build_seq;
            *sc.cap_sets = n;
        }
        ga.epoch = ++*sc.epoch;
    }
    HIP_TRY(lora::launch_gemv(c->dtype, gm, ga, st, tm));
    return LORA_OK;
}

static int enqueue_group(lora_cache_t *c, lora_plan_t *p, const lora_apply_desc_t *descs, int n, float scale, hipStream_t st,
                         const Scratch &sc)
{
    // the work lists may have been uploaded on another stream
    if (p->upload_pending) {
        if (is_capturing(st)) {  // a wait on an event from outside the capture would not become part of the graph
            HIP_TRY(hipEventSynchronize(p->ev_upload));
            p->upload_pending = false;
        } else if (hipEventQuery(p->ev_upload) == hipSuccess) {
            p->upload_pending = false;
        } else {
            HIP_TRY(hipStreamWaitEvent(st, p->ev_upload, 0));
        }
    }
    for (int32_t sl : p->slots) {
        Slot &s = c->slots[sl];
        if (s.fill_pending) {
            if (hipEventQuery(s.fill_ev) == hipSuccess) s.fill_pending = false;
            else HIP_TRY(hipStreamWaitEvent(st, s.fill_ev, 0));
        }
    }
    const lora::KernelTimer timer{c, timer_pair};
    const lora::KernelTimer *tm = c->timing && !is_capturing(st) ? &timer : nullptr;
    const lora::DevItem *tiles = reinterpret_cast<const lora::DevItem *>(p->dev + p->off_tiles);

    lora::ApplyArgs a[N_VSETS];
    lora::ShrinkProjs ps;
    if (const int rc_s = shrink_setup(c, p, n, sc.vpart, sc.vpart_rows, sc.small, ps)) return rc_s;
    for (int i = 0; i < n; ++i) {
        const int32_t proj = descs[i].proj;
        a[i].proj_base = c->pool + (size_t)descs[i].layer * c->layer_stride + c->proj_off[proj];
        a[i].row_bytes = (int64_t)c->row_bytes[proj];
        a[i].tok_list = reinterpret_cast<const int32_t *>(p->dev);
        a[i].x = descs[i].x;
        a[i].y = descs[i].base_out;
        a[i].v = reinterpret_cast<float *>(sc.v + (size_t)i * sc.v_set_bytes);
        a[i].h_in = c->proj[proj].h_in;
        a[i].h_out = c->proj[proj].h_out;
        a[i].v_stride = c->v_stride;
        a[i].scale = scale;
        ps.proj_base[i] = a[i].proj_base;
        ps.row_bytes[i] = a[i].row_bytes;
        ps.v[i] = a[i].v;
    }
    for (int i = n; i < N_VSETS; ++i) {
        ps.proj_base[i] = nullptr;
        ps.row_bytes[i] = 0;
        ps.v[i] = nullptr;
    }
    // The GEMV launch and the tile kernels of a group work on different tokens (rows of base_out) with different
    // scratch: when a batch has both, the GEMV launch goes to the cache's side stream, forked off here and
    // joined again behind the tile expands (also under stream capture, where fork and join become edges of the graph).
    // Not while kernels are being timed: a kernel's duration is then its own, not that of two kernels sharing the memory.
    const bool fork = p->n_tiles > 0 && p->n_gs > 0 && c->side_stream != nullptr && c->side_stream != st && tm == nullptr;
    hipStream_t gemv_st = st;
    if (fork) {
        HIP_TRY(hipEventRecord(c->ev_fork, st));
        HIP_TRY(hipStreamWaitEvent(c->side_stream, c->ev_fork, 0));
        gemv_st = c->side_stream;
    }
    // everything that reads x
    if (p->n_tiles > 0) {
        HIP_TRY(lora::launch_mfma_shrink(a[0], ps, tiles, p->n_tiles, st, tm));
    }
    // joined behind the tile expands, whatever happens in between: a captured fork must not stay open
    struct Join {
        lora_cache_t *c;
        hipStream_t st;
        bool armed;
        hipError_t now()
        {
            if (!armed) return hipSuccess;
            armed = false;
            const hipError_t e = hipEventRecord(c->ev_join, c->side_stream);
            return e == hipSuccess ? hipStreamWaitEvent(st, c->ev_join, 0) : e;
        }
        ~Join() { (void)now(); }
    } join{c, st, fork};
    if (const int rc_g = enqueue_gemv(c, p, a, nullptr, n, true, gemv_st, sc, tm)) return rc_g;
    // the updates of base_out
    for (int i = 0; i < n; ++i) {
        HIP_TRY(lora::launch_mfma_expand(a[i], tiles, p->n_tiles, st, tm));
        const int64_t seq = ++c->apply_seq;
        ++c->stats.applies;
        for (int32_t sl : p->slots) {
            c->slots[sl].last_used = seq;
            ++c->slots[sl].use_count;
        }
    }
    HIP_TRY(join.now());
    return LORA_OK;
}

static int enqueue_apply(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x, void *base_out,
                         float scale, hipStream_t st)
{
    const lora_apply_desc_t d{layer, proj, x, base_out};
    return enqueue_group(c, p, &d, 1, scale, st, pool_scratch(c));
}

// One event pair per call (not per apply): fills that come later wait for it.
static int fence_applies(lora_cache_t *c, lora_plan_t *p, hipStream_t st)
{
    if (!c->fencing || is_capturing(st)) return LORA_OK;
    const int64_t seq = c->apply_seq;
    HIP_TRY(hipEventRecord(c->apply_ev[seq % N_APPLY_EVENTS], st));
    c->apply_ev_seq[seq % N_APPLY_EVENTS] = seq;
    hipEvent_t &own = c->stream_fence[st];
    if (!own) HIP_TRY(hipEventCreateWithFlags(&own, hipEventDisableTiming));
    HIP_TRY(hipEventRecord(own, st));
    HIP_TRY(hipEventRecord(p->ev_last_use, st));
    p->use_pending = true;
    return LORA_OK;
}

int lora_apply_plan(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x, void *base_out,
                    float scale, void *stream)
{
    if (!c || !p || !p->in_use || c->host_only) return LORA_E_INVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = validate_apply(c, p, layer, proj, x, base_out);
    if (rc != LORA_OK) return rc;
    rc = enqueue_apply(c, p, layer, proj, x, base_out, scale, st);
    if (rc != LORA_OK) return rc;
    return fence_applies(c, p, st);
}

int lora_apply_plan_static(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x, void *base_out,
                           float scale, void *stream)
{
    if (!c || !p || !p->in_use || c->host_only) return LORA_E_INVAL;
    if (p->T > LORA_STATIC_MAX_TOKENS) return LORA_E_NOMEM;  // the fixed scratch does not hold this batch
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = validate_apply(c, p, layer, proj, x, base_out);
    if (rc != LORA_OK) return rc;
    StaticScratch &ss = g_static[c->device];  // set up by lora_cache_create on this device
    if (!ss.ptr) return LORA_E_STATE;
    const Scratch sc{ss.ptr, STATIC_V_BYTES, 1, ss.ptr + STATIC_V_BYTES, STATIC_VPART_ROWS, true,
                     ss.ptr + STATIC_V_BYTES + STATIC_VPART_BYTES, STATIC_VTAG_BYTES, &ss.epoch, &ss.cap_id, &ss.cap_plan, &ss.cap_sets};
    const lora_apply_desc_t d{layer, proj, x, base_out};
    const bool timing = c->timing;
    c->timing = false;  // timed launches take events from a pool that may have to grow
    rc = enqueue_group(c, p, &d, 1, scale, st, sc);
    c->timing = timing;
    if (rc != LORA_OK) return rc;
    return fence_applies(c, p, st);
}

int lora_linear_workspace_bytes(const lora_cache_t *c, const lora_plan_t *p, int32_t proj, size_t *bytes)
{
    if (!c || !p || !p->in_use || !bytes || proj < 0 || proj >= (int32_t)c->proj.size()) return LORA_E_INVAL;
    *bytes = p->n_tok_list > p->n_tile_tok ? (size_t)p->T * c->proj[proj].h_out * sizeof(float) : 0;
    return LORA_OK;
}

int lora_linear_plan(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x, const void *Wt, void *y,
                     float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!c || !p || !p->in_use || c->host_only || c->dtype != LORA_BF16) return LORA_E_INVAL;
    if (workspace) {
        size_t need = 0;
        if (lora_linear_workspace_bytes(c, p, proj, &need) != LORA_OK || !aligned16(workspace) || workspace_bytes < need) return LORA_E_INVAL;
    }
    int rc = validate_apply(c, p, layer, proj, x, y);
    if (rc != LORA_OK) return rc;
    if (p->T > 0 && (!Wt || !aligned16(Wt))) return LORA_E_INVAL;
    if (p->T == 0) return LORA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (p->upload_pending) HIP_TRY(hipStreamWaitEvent(st, p->ev_upload, 0));
    for (int32_t sl : p->slots) {
        Slot &s = c->slots[sl];
        if (s.fill_pending) {
            if (hipEventQuery(s.fill_ev) == hipSuccess) s.fill_pending = false;
            else HIP_TRY(hipStreamWaitEvent(st, s.fill_ev, 0));
        }
    }
    const lora::KernelTimer timer{c, timer_pair};
    const lora::KernelTimer *tm = c->timing && !is_capturing(st) ? &timer : nullptr;
    const lora::DevItem *tiles = reinterpret_cast<const lora::DevItem *>(p->dev + p->off_tiles);
    lora::ApplyArgs a;
    a.proj_base = c->pool + (size_t)layer * c->layer_stride + c->proj_off[proj];
    a.row_bytes = (int64_t)c->row_bytes[proj];
    a.tok_list = reinterpret_cast<const int32_t *>(p->dev);
    a.x = x;
    a.y = y;
    a.v = reinterpret_cast<float *>(c->pool + c->off_v);
    a.h_in = c->proj[proj].h_in;
    a.h_out = c->proj[proj].h_out;
    a.v_stride = c->v_stride;
    a.scale = scale;
    // shrink of the tiles and of the GEMV groups (x is read, v written)
    if (p->n_tiles > 0) {
        lora::ShrinkProjs ps;
        if (const int rc_s = shrink_setup(c, p, 1, c->pool + c->off_vpart, c->vpart_rows, false, ps)) return rc_s;
        for (int i = 0; i < lora::MAX_SHRINK_PROJS; ++i) {
            ps.proj_base[i] = i ? nullptr : a.proj_base;
            ps.row_bytes[i] = i ? 0 : a.row_bytes;
            ps.v[i] = i ? nullptr : a.v;
        }
        HIP_TRY(lora::launch_mfma_shrink(a, ps, tiles, p->n_tiles, st, tm));
    }
    // the adapter term of the GEMV tokens: as fp32 into the caller's workspace (row = token), or, without
    // one, into their zeroed output rows (rounded to the output type on the way)
    if (p->n_tok_list > p->n_tile_tok) {
        a.y32 = static_cast<float *>(workspace);
        if (!a.y32) HIP_TRY(lora::launch_zero_rows(y, a.tok_list + p->n_tile_tok, p->n_tok_list - p->n_tile_tok, a.h_out, st));
        float *const y32 = a.y32;
        if (const int rc_g = enqueue_gemv(c, p, &a, &y32, 1, false, st, pool_scratch(c), tm)) return rc_g;
    }
    // base product of every token + adapter product of the tiles (+ the term just computed for the others)
    lora::ApplyArgs lin = a;
    lin.tok_list = reinterpret_cast<const int32_t *>(p->dev + p->off_lin_tok);
    // (the partial sums of split tiles go where the tile shrink's partial sums went: that kernel is done)
    HIP_TRY(lora::launch_linear_tiles(lin, Wt, reinterpret_cast<const lora::DevItem *>(p->dev + p->off_lin_tiles), p->n_lin_tiles,
                                      c->pool + c->off_vpart, c->vpart_bytes, reinterpret_cast<uint32_t *>(c->pool + c->off_fault),
                                      N_LINEAR_FLAGS, c->fault_dev, c->n_cu, st, tm));
    const int64_t seq = ++c->apply_seq;
    ++c->stats.applies;
    for (int32_t sl : p->slots) {
        c->slots[sl].last_used = seq;
        ++c->slots[sl].use_count;
    }
    return fence_applies(c, p, st);
}

int lora_apply_plan_multi(lora_cache_t *c, lora_plan_t *p, const lora_apply_desc_t *descs, int32_t n, float scale,
                          void *stream)
{
    if (!c || !p || !p->in_use || c->host_only || n < 0 || (n > 0 && !descs)) return LORA_E_INVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int32_t i = 0; i < n; ++i) {
        const int rc = validate_apply(c, p, descs[i].layer, descs[i].proj, descs[i].x, descs[i].base_out);
        if (rc != LORA_OK) return rc;
    }
    // runs of applies that read the same x (q, k, v; gate, up) and do not write to it go as a group
    const size_t e = c->esize;
    for (int32_t i = 0; i < n;) {
        int32_t g = 1;
        const char *x0 = static_cast<const char *>(descs[i].x);
        const size_t x_bytes = (size_t)p->T * c->proj[descs[i].proj].h_in * e;
        auto writes_x = [&](const lora_apply_desc_t &d) {
            const char *y0 = static_cast<const char *>(d.base_out);
            return y0 < x0 + x_bytes && x0 < y0 + (size_t)p->T * c->proj[d.proj].h_out * e;
        };
        if (!writes_x(descs[i])) {
            while (g < N_VSETS && i + g < n && descs[i + g].x == descs[i].x &&
                   c->proj[descs[i + g].proj].h_in == c->proj[descs[i].proj].h_in && !writes_x(descs[i + g]))
                ++g;
        }
        const int rc = enqueue_group(c, p, descs + i, g, scale, st, pool_scratch(c));
        if (rc != LORA_OK) return rc;
        i += g;
    }
    return n > 0 ? fence_applies(c, p, st) : LORA_OK;
}

int lora_apply(lora_cache_t *c, int32_t layer, int32_t proj, const void *x, void *base_out, int32_t T,
               const int32_t *seg_offsets, const int32_t *seg_slot, const int32_t *seg_rank, int32_t n_seg, float scale,
               void *stream)
{
    if (!c || c->host_only) return LORA_E_INVAL;
    lora_plan &p = c->plans[c->n_user_plans + (c->internal_next % N_INTERNAL_PLANS)];
    int rc = build_plan(*c, p, T, seg_offsets, seg_slot, seg_rank, n_seg, static_cast<hipStream_t>(stream));
    if (rc != LORA_OK) return rc;
    ++c->internal_next;
    p.in_use = true;
    rc = lora_apply_plan(c, &p, layer, proj, x, base_out, scale, stream);
    p.in_use = false;
    return rc;
}

}  // extern "C"
