/*
 * lora_cache.h -- C ABI of the MI355X (gfx950) adapter cache pool and the batched
 * heterogeneous-rank LoRA apply.
 *
 * What the library computes.  For one projection (h_in -> h_out) of one layer and a
 * batch of T tokens cut into segments (one segment per request of the iteration:
 * a decode request is one token, a prefill request its whole prompt), every token t
 * of a segment that names cache slot i of rank r_i gets, in place,
 *
 *     base_out[t][:] += scale * alpha_i * (x[t][:] . A_i) . B_i
 *
 * with A_i [h_in][r_i] and B_i [r_i][h_out] read from the adapter cache pool.  This
 * is the per-layer adapter work the paper describes in section 3.1 (two matrix
 * products on top of the base product plus one addition that aggregates the
 * results), for a batch in which requests carry different adapters of different
 * ranks (section 2).  The pool is the paper's adapter cache (section 4.2): adapter
 * weights kept resident in otherwise idle GPU memory, one entry per adapter with its
 * id, rank, last-used stamp, use frequency and reference count; entries are
 * read-only, so eviction discards and nothing is ever written back.
 *
 * Conventions.
 *  - Every function returns LORA_OK (0) or a negative lora_status; nothing aborts or
 *    throws.  lora_strerror() names a status; lora_last_hip_error() returns the HIP
 *    status behind the last LORA_E_HIP on the calling thread.
 *  - "device" pointers are HIP device memory owned by the caller (the Python binding
 *    gets them from PyTorch); "host" pointers are ordinary host memory read during the
 *    call, except the fill sources, which are read asynchronously (see there).
 *  - Streams are hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; none blocks the host except where stated.
 *  - One lora_cache_t must not be used from two host threads at once.  lora_apply /
 *    lora_apply_plan calls that share a cache share its scratch (the T x rank
 *    intermediate), so they must be ordered on the device: issue them on one stream,
 *    or order the streams with events.
 *  - Supported shapes: h_in and h_out multiples of 64; 1 <= rank <= LORA_MAX_RANK.
 */
#ifndef LORA_CACHE_H
#define LORA_CACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LORA_OK = 0,
    LORA_E_INVAL = -1,    /* null / negative / out-of-range argument, malformed segment arrays */
    LORA_E_STATE = -2,    /* slot in the wrong state (apply on an unfilled slot, evict/refill while referenced) */
    LORA_E_NOMEM = -3,    /* caller's pool buffer too small, no free plan, host allocation failed */
    LORA_E_HIP = -4,      /* a HIP call failed; see lora_last_hip_error() */
    LORA_E_NOTFOUND = -5, /* adapter id not cached */
    LORA_E_FAULT = -6     /* a kernel of an earlier apply gave up a bounded wait (its outputs are invalid); every apply
                             returns this until lora_cache_check_fault has been called */
} lora_status;

enum { LORA_F32 = 0, LORA_BF16 = 1 };                               /* element type of x, base_out, A, B */
enum { LORA_SLOT_EMPTY = 0, LORA_SLOT_FILLING = 1, LORA_SLOT_READY = 2 };
enum {
    LORA_CACHE_HOST_ONLY = 1,     /* flags: slot table only, no device work */
    /* GEMV shrink and expand run as one launch with an in-kernel hand-over of the intermediate when
     * the batch's GEMV part is small (the launch in between then costs more than the hand-over),
     * else as two launches.  These two flags take the choice away: */
    LORA_CACHE_FUSED_GEMV = 2,    /* always one launch (except under stream capture, where it is always two) */
    LORA_CACHE_SPLIT_GEMV = 4,    /* always two launches (and no hand-over buffer in the pool) */
    LORA_CACHE_NO_OVERLAP = 16,   /* every kernel of an apply on the caller's stream: by default the GEMV launch of a batch that
                                     also has tiles runs on a stream of the cache's own, forked off the caller's stream and
                                     joined to it again inside the call, side by side with the tile kernels (different tokens) */
    LORA_CACHE_DIRECT_FILL = 8    /* fills read pinned host memory from the repack kernel itself instead of copying it
                                     to a staging buffer first: about twice the fill rate on an idle device, but applies
                                     that run at the same time are slowed down much more (measured 1.6x against 1.1x) */
};

#define LORA_MAX_RANK 128
#define LORA_TILE_TOKENS 64      /* tokens per matrix-core tile */
#define LORA_MFMA_MIN_TOKENS 16  /* default: segments / pooled slots with fewer tokens take the GEMV path ... */
#define LORA_MFMA_MIN_TOKENS_MIXED 8 /* ... and, with the default, this is the threshold once a batch has any tile at 16 */

typedef struct lora_cache lora_cache_t; /* opaque */
typedef struct lora_plan lora_plan_t;   /* opaque: device-resident work lists of one batch */

typedef struct {
    int32_t h_in, h_out;
} lora_proj_t;

typedef struct {
    int32_t n_proj;             /* projections per layer that carry adapters (q,k,v,o in the paper, section 3.2) */
    const lora_proj_t *proj;    /* [n_proj] */
    int32_t n_layers;           /* layer copies the pool holds */
    int32_t n_classes;          /* rank classes; a slot of class c holds any adapter with rank <= class_rank[c] */
    const int32_t *class_rank;  /* [n_classes], strictly increasing, <= LORA_MAX_RANK (paper: 8,16,32,64,128) */
    const int32_t *class_slots; /* [n_classes] slots per class; slot ids run class by class */
    int32_t dtype;              /* LORA_F32 | LORA_BF16 */
    int32_t max_tokens;         /* largest T of any apply */
    int32_t max_segments;       /* largest n_seg of any apply */
    int32_t n_plans;            /* plans that may be alive at once (>= 0; 4 more are kept for lora_apply) */
    int32_t mfma_min_tokens;    /* 0 = default, chosen per batch: no tiles at all if the batch has none at
                                   LORA_MFMA_MIN_TOKENS or too few for the tile launches to pay off, else
                                   LORA_MFMA_MIN_TOKENS_MIXED (see lora_plan_info); ignored (no tile path) for LORA_F32 */
    int32_t flags;
} lora_cache_config_t;

/* ---- sizes (pure host arithmetic) ------------------------------------------------ */

/* Bytes of A and B of one adapter of `rank` for one projection, unpadded:
 * rank * (h_in + h_out) * element size.  (Section 3.2's 64 MB for rank 32 on a 7B
 * model is 4 projections x 32 layers of this at 16 bit.)  0 on bad arguments. */
size_t lora_adapter_bytes(int32_t h_in, int32_t h_out, int32_t rank, int32_t dtype);

/* Bytes the caller must provide to lora_cache_create: slabs of every (layer,
 * projection, slot) + scratch + plan buffers + fill staging.  0 on a bad config. */
size_t lora_cache_bytes_required(const lora_cache_config_t *cfg);

/* ---- pool life cycle ----------------------------------------------------------------- */

/* Carve `dev_pool` (device, >= lora_cache_bytes_required bytes, 256-byte aligned,
 * caller-owned, must outlive the cache) into slabs and scratch, build the slot table.
 * Uploads a small offset table (blocking).  With LORA_CACHE_HOST_ONLY, dev_pool may be
 * NULL and only the slot-table calls work. */
int lora_cache_create(const lora_cache_config_t *cfg, void *dev_pool, size_t dev_pool_bytes, lora_cache_t **out);
int lora_cache_destroy(lora_cache_t *c);

/* ---- cache entries (section 4.2: load a missing adapter, retrieve a cached one, evict) -- */

/* Enqueue, on `fill_stream`, the copy of one (layer, projection) part of an adapter
 * into `slot`: host_A [h_in][rank] and host_B [rank][h_out], row-major, element type =
 * cfg.dtype.  The host buffers are read asynchronously: keep them unchanged until the
 * stream has passed this call.  The part is copied into a staging buffer by the copy engine
 * (pinned host memory makes the copies truly asynchronous) and repacked into the slot by one
 * kernel; with LORA_CACHE_DIRECT_FILL that kernel reads pinned, 16-byte aligned host memory
 * directly.  The
 * first part filled into an EMPTY slot binds (adapter_id, rank, alpha) and moves it to
 * FILLING; later parts must repeat the same three.  The slot reports READY once all
 * n_layers * n_proj parts are enqueued and the last copy has completed.  An apply that
 * names a part still in flight makes its stream wait for it; the fill in turn waits
 * for applies enqueued earlier that read the slot.
 * LORA_E_STATE if the slot is referenced (refcount > 0) and already complete, or bound
 * to another adapter; LORA_E_INVAL if rank exceeds the slot's class. */
int lora_cache_fill_slot(lora_cache_t *c, int32_t slot, int64_t adapter_id, int32_t rank, float alpha,
                         int32_t layer, int32_t proj, const void *host_A, const void *host_B, void *fill_stream);

/* The same for several parts of one adapter in one call (section 4.2: a missing adapter is loaded
 * as a whole before its batch runs): parts[i] names a (layer, projection) and its two host arrays.
 * One wait for earlier applies, one event, and -- with LORA_CACHE_DIRECT_FILL and pinned, 16-byte
 * aligned host arrays -- one kernel per 32 parts instead of one per part: the host side of loading an
 * adapter then costs about as much as one part did.  Otherwise the parts go through the staging
 * buffers one after the other as lora_cache_fill_slot sends them.  Errors as lora_cache_fill_slot;
 * on an error no part of the call is enqueued. */
typedef struct {
    int32_t layer, proj;
    const void *host_A; /* [h_in][rank] */
    const void *host_B; /* [rank][h_out] */
} lora_fill_part_t;
int lora_cache_fill_slot_parts(lora_cache_t *c, int32_t slot, int64_t adapter_id, int32_t rank, float alpha,
                               const lora_fill_part_t *parts, int32_t n_parts, void *fill_stream);

/* Evict: any state -> EMPTY.  No write-back (entries are read-only).  LORA_E_STATE if refcount > 0. */
int lora_cache_release_slot(lora_cache_t *c, int32_t slot);

/* Reference counter of the entry (number of running requests that use it): delta = +1 / -1. */
int lora_cache_slot_ref(lora_cache_t *c, int32_t slot, int32_t delta);

/* adapter id -> slot and rank; LORA_E_NOTFOUND on a miss.  Counts a hit or a miss. */
int lora_cache_lookup(lora_cache_t *c, int64_t adapter_id, int32_t *slot, int32_t *rank);

typedef struct {
    int64_t adapter_id;
    int32_t rank, class_rank, state, refcount;
    int64_t use_count; /* applies that named the slot ("frequency") */
    int64_t last_used; /* sequence number of the last such apply ("last used"), 0 = never */
    float alpha;
    int32_t parts_filled;
} lora_slot_info_t;
int lora_cache_slot_info(lora_cache_t *c, int32_t slot, lora_slot_info_t *out);

/* The state alone (section 4.2: an entry is loaded before the batch that needs it is sent):
 * LORA_SLOT_EMPTY, LORA_SLOT_FILLING (bound, not all parts enqueued or the last copy still in
 * flight) or LORA_SLOT_READY. */
int lora_cache_slot_state(lora_cache_t *c, int32_t slot, int32_t *state);

/* A free slot of the smallest class that fits `rank`, or LORA_E_NOMEM. */
int lora_cache_find_free_slot(lora_cache_t *c, int32_t rank, int32_t *slot);

typedef struct {
    int64_t hits, misses, fills, bytes_filled, applies, evictions;
} lora_cache_stats_t;
int lora_cache_stats(const lora_cache_t *c, lora_cache_stats_t *out);

/* ---- cache manager (section 4.2: cost-aware eviction, reference counters, queued requests,
 *      prefetching, dynamic sizing).  Host-side bookkeeping only: nothing here touches the device. */

/* Eviction score of a cached entry = w_freq * frequency + w_recency * recency + w_size * size; the
 * entry with the LOWEST score goes first.  The paper fixes the coefficients (0.45, 0.10, 0.45: the
 * defaults) but not the units of the three terms; here each is scaled to [0, 1] over the cached
 * entries: frequency = requests that used the entry / the largest such count; recency =
 * 1 - age / largest age, age counted in requests since the entry's last use; size = rank / largest
 * cached rank (a larger adapter costs more to reload, so it is kept longer).  The paper counts uses
 * over a limited period only: here every freq_window requests all frequencies are halved (0 = never).
 * (0, 1, 0) is LRU; equal weights are the paper's FairShare comparison point. */
typedef struct {
    double w_freq, w_recency, w_size;
    int64_t freq_window;
} lora_policy_t;
int lora_cache_set_policy(lora_cache_t *c, const lora_policy_t *p); /* LORA_E_INVAL on negative or NaN values */
int lora_cache_get_policy(const lora_cache_t *c, lora_policy_t *p);

/* A request for an adapter arrives (pin = 1: it is about to run and holds a reference until
 * lora_cache_slot_ref(slot, -1); pin = 0: it waits in a queue and the adapter is only prefetched).
 * Hit: *hit = 1, *slot = its slot (which may still be FILLING).  Miss: *hit = 0 and *slot is bound to
 * (adapter_id, rank, alpha) in state FILLING with no part loaded -- a free slot of the smallest class
 * that fits, else the slot of the entry the policy evicts; the caller then loads the parts with
 * lora_cache_fill_slot.  Never evicted: entries with a reference; entries whose adapter is in
 * queued_ids (host array, adapters of requests that wait; may be NULL with n_queued = 0) are evicted
 * only when no other candidate is left.  Either way the request counts for the entry's frequency
 * and recency.  LORA_E_NOMEM if every entry in a large-enough slot is referenced; LORA_E_INVAL if
 * rank exceeds the largest class or differs from the cached entry's. */
int lora_cache_acquire(lora_cache_t *c, int64_t adapter_id, int32_t rank, float alpha, int32_t pin,
                       const int64_t *queued_ids, int32_t n_queued, int32_t *slot, int32_t *hit);

/* The score of the entry in `slot` (LORA_E_STATE if the slot is empty), and the slot the policy
 * would evict next for an adapter of `rank` (0: any slot) without evicting it; LORA_E_NOMEM if
 * there is none. */
int lora_cache_score(lora_cache_t *c, int32_t slot, double *score);
int lora_cache_choose_victim(lora_cache_t *c, int32_t rank, const int64_t *queued_ids, int32_t n_queued, int32_t *slot);

/* Dynamic sizing: bytes of pool memory held by cached entries (each entry's storage rows in every
 * layer and projection), and eviction in score order until at most max_bytes are held -- what the
 * scheduler asks for when a batch's activations and KV entries need the room.  The pool's memory
 * stays the caller's allocation: a trimmed cache leaves the slabs past the budget empty for the
 * caller to plan with.  LORA_E_NOMEM if entries in use keep it above the budget (what could go has gone). */
int lora_cache_resident_bytes(const lora_cache_t *c, size_t *bytes);
int lora_cache_trim(lora_cache_t *c, size_t max_bytes, const int64_t *queued_ids, int32_t n_queued, int32_t *n_evicted);

/* Device address and byte size of the slab of (layer, proj, slot) -- for tests and tools. */
int lora_cache_slab(const lora_cache_t *c, int32_t layer, int32_t proj, int32_t slot, void **dev_ptr, size_t *bytes);

/* ---- indexing ------------------------------------------------------------------------ */

/* A tile or a group: tokens tok_list[tok_off .. tok_off + n_tok) of one slot.  a = running tile
 * number inside its segment or pool (0 for groups); b, c, d are 0. */
typedef struct {
    int32_t tok_off, n_tok, slot, rank, a, b, c, d;
} lora_item_t;

typedef struct {
    int32_t n_tok_list, n_tiles, n_groups;
    int32_t *tok_list;     /* tokens of all tiles, then of all groups */
    lora_item_t *tiles;    /* <= LORA_TILE_TOKENS tokens of one slot each (matrix-core path) */
    lora_item_t *groups;   /* all remaining tokens of one slot (GEMV path) */
} lora_worklists_t;

/* Pure host: which token goes which way, and with which cache entry (integer work only; section 2:
 * one batch mixes requests of different adapters, section 4.1: the batch is formed anew every
 * iteration, so this runs once per iteration).
 *  - seg_offsets [n_seg+1] non-decreasing, [0] = 0, [n_seg] = T; seg_slot [n_seg], < 0 =
 *    no adapter (tokens keep base_out); seg_rank [n_seg] in 1..LORA_MAX_RANK where slot >= 0.
 *  - A non-empty segment with slot >= 0 and at least mfma_min_tokens tokens is cut into
 *    tiles of LORA_TILE_TOKENS consecutive tokens, in segment order.  Tokens of the other
 *    such segments are pooled per slot (slots ascending, tokens ascending); a pool of at
 *    least mfma_min_tokens tokens is cut into tiles too, any other is one group.
 *    mfma_min_tokens = 0 turns tiles off (everything is pooled into groups).
 * How the kernels cut tiles and groups into blocks and wavefronts is not part of this contract
 * (lora_plan_dump shows it for a plan).
 * All segments that name one slot must carry the same rank (else LORA_E_INVAL).
 * Arrays in *out are malloc'ed; free them with lora_worklists_free. */
int lora_index(int32_t T, const int32_t *seg_offsets, const int32_t *seg_slot, const int32_t *seg_rank,
               int32_t n_seg, int32_t mfma_min_tokens, lora_worklists_t *out);
void lora_worklists_free(lora_worklists_t *w);

/* ---- apply --------------------------------------------------------------------------- */

/* Index a batch once and keep its work lists on the device, so that the same batch can
 * be applied to every projection of every layer of the iteration.  Checks every named
 * slot against the slot table (exists, bound, seg_rank equals its rank).  The upload is
 * enqueued on `stream`; the host arrays may be reused on return. */
int lora_plan_create(lora_cache_t *c, int32_t T, const int32_t *seg_offsets, const int32_t *seg_slot,
                     const int32_t *seg_rank, int32_t n_seg, void *stream, lora_plan_t **out);
int lora_plan_destroy(lora_cache_t *c, lora_plan_t *p);

/* What a plan holds: the threshold its work lists were made with (lora_index with the same
 * arrays and this threshold returns the same lists; 0 = no tiles) and their sizes. */
typedef struct {
    int32_t T, mfma_min_tokens, n_tiles, n_tile_tokens, n_gemv_shrink_items, n_gemv_expand_items;
} lora_plan_info_t;
int lora_plan_info(const lora_plan_t *p, lora_plan_info_t *out);

/* For tests and tools: the units of work the kernels will execute for a plan on projection `proj`,
 * decoded from the very buffer the kernels read (the device copy, fetched back with a blocking
 * copy; the staged host copy for a LORA_CACHE_HOST_ONLY cache) by the routines the kernels
 * themselves decode their work items with.  The slot/segment indexing is correct when:
 * the TILE units and the tokens of the GEMV units partition the batch's tokens that have an
 * adapter; every unit names the slot and rank of its tokens' segments; for every GEMV token the
 * SHRINK units cover rank rows [0, rank) exactly once and the EXPAND units cover output columns
 * [0, h_out) exactly once; the LINEAR_ROWS units (bf16 caches: the row tiles of lora_linear_plan)
 * cover every token of the batch exactly once; for every tile and run table the TILE_SHRINK units
 * (the pieces the tile's input columns are worked on in) cover [0, h_in) exactly once, the pieces
 * that are not whole tiles leave their partial sums in distinct scratch slots, and the TILE_SUM
 * units (the slots the reduce kernel adds up for the tile) name exactly those slots.
 * Writes at most cap_units units and cap_toks tokens; *n_units and *n_toks return the full counts
 * (call with zero capacities to size the arrays). */
enum { LORA_UNIT_TILE = 0, LORA_UNIT_GEMV_SHRINK = 1, LORA_UNIT_GEMV_EXPAND = 2, LORA_UNIT_LINEAR_ROWS = 3, LORA_UNIT_TILE_SHRINK = 4, LORA_UNIT_TILE_SUM = 5 };
typedef struct {
    int32_t kind;
    int32_t tok_off, n_tok; /* the unit's tokens: toks[tok_off .. tok_off + n_tok) */
    int32_t slot, rank;     /* slot found back from the storage row the kernels address; -1, 0: rows without adapter */
    int32_t lo, hi;         /* GEMV_SHRINK: rank rows [lo, hi); GEMV_EXPAND: output columns [lo, hi); TILE_SHRINK: input
                               columns [lo, hi); TILE_SUM: slot number lo of hi; else 0, 0 */
    int32_t where;          /* GEMV_SHRINK: position in launch order; LINEAR_ROWS: 2 = a tile, 1 = rows of GEMV tokens,
                               0 = rows without adapter; TILE_SHRINK, TILE_SUM: run table << 20 | run (run tables 0..3:
                               launches for 1..4 projections; 4: the one of lora_apply_plan_static); TILE: 0 */
    float alpha;            /* the cache entry's own factor as the kernels will apply it; TILE_SHRINK, TILE_SUM: the
                               scratch slot of the partial sum (-1: the piece is the whole tile and leaves none) */
} lora_plan_unit_t;
int lora_plan_dump(lora_cache_t *c, const lora_plan_t *p, int32_t proj, lora_plan_unit_t *units, int32_t cap_units,
                   int32_t *n_units, int32_t *toks, int32_t cap_toks, int32_t *n_toks);

/* base_out[t] += scale*alpha*(x[t].A).B for the planned batch; x [T][h_in] and base_out
 * [T][h_out] are device, row-major, contiguous, element type cfg.dtype.  Asynchronous on
 * `stream`, which need not be the stream the plan was created on (the apply waits for the plan's
 * upload).  LORA_E_STATE if a named slot has no data for (layer, proj).  All checks happen before
 * the first launch.  If the runtime then refuses a launch (LORA_E_HIP), the launches before it stay
 * enqueued and the base_out of this call is unspecified; cache and plan remain usable. */
int lora_apply_plan(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x,
                    void *base_out, float scale, void *stream);

/* lora_apply_plan for callers that cannot allocate device memory or hand any over for scratch: code
 * whose memory is fixed before it starts (a serving loop with a frozen memory plan, a harness that
 * forbids allocation, work recorded for later replay).  Same arguments, same result, same kernels;
 * the intermediate buffers (shrink results, the tile shrink's partial sums, hand-over words) do not come from
 * the cache's pool but from a fixed array of LORA_STATIC_SCRATCH_BYTES (14 MiB) in the library's
 * device image, which every device the library has run on holds until the process ends.  The call
 * allocates nothing and frees nothing, on the device or through the runtime.
 * LORA_E_NOMEM if the plan's batch has more than LORA_STATIC_MAX_TOKENS tokens.
 * All caches of the process share the one array of their device, and it keeps the last call's
 * contents: calls on one device must not overlap -- issue them on one stream or order the streams
 * with events, also across caches (lora_apply_plan and friends use the pool's own scratch and may
 * overlap with it). */
#define LORA_STATIC_MAX_TOKENS 4096
#define LORA_STATIC_SCRATCH_BYTES ((size_t)LORA_STATIC_MAX_TOKENS * LORA_MAX_RANK * (4 + 4 * 4 + 8))
int lora_apply_plan_static(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x,
                           void *base_out, float scale, void *stream);

/* The same for a list of (layer, projection, x, base_out): the result is that of n calls of
 * lora_apply_plan in order on `stream` (one iteration's worth of applies with a single trip
 * through the binding).  Up to 4 consecutive entries that read the same x (q, k, v; gate, up) and
 * do not write into it are run shrink-first -- one pass over x for all of them, then their updates
 * of base_out.  Nothing is enqueued if any entry fails validation. */
typedef struct {
    int32_t layer, proj;
    const void *x;  /* device [T][h_in] */
    void *base_out; /* device [T][h_out], in/out */
} lora_apply_desc_t;
int lora_apply_plan_multi(lora_cache_t *c, lora_plan_t *p, const lora_apply_desc_t *descs, int32_t n, float scale,
                          void *stream);

/* The base projection and the adapter update of a planned batch in one pass (section 3.1 with
 * the separate addition folded away):  y[t] = x[t] . W + s_i * (x[t] . A_i) . B_i  for every token of
 * the batch; tokens without an adapter get x[t] . W.  Wt is the device weight [h_out][h_in], bf16 --
 * W transposed, the layout a linear layer keeps its weight in; y [T][h_out] is written only (it
 * need not hold anything on entry, and must not overlap x).  The shrink runs as in lora_apply_plan;
 * then one matrix-core kernel computes the base product over row tiles of 64 tokens and adds the
 * adapter product of the tiles as one more slab of the contraction.  Tokens on the GEMV path get their
 * adapter term from the GEMV kernels beforehand, and the matrix-core kernel adds it to their rows
 * before the one rounding of the output: as fp32 through `workspace` (device, caller-owned, 16-byte
 * aligned, at least lora_linear_workspace_bytes() bytes: T * h_out floats when the plan has GEMV
 * tokens, else 0; its contents are scratch), or, with workspace = NULL, through the output rows
 * themselves, where the term is rounded to bf16 on the way (its error then adds to the output's).
 * bf16 caches only (LORA_E_INVAL otherwise; also for a workspace that is misaligned or too small);
 * other errors and stream semantics as for lora_apply_plan. */
int lora_linear_workspace_bytes(const lora_cache_t *c, const lora_plan_t *p, int32_t proj, size_t *bytes);
int lora_linear_plan(lora_cache_t *c, lora_plan_t *p, int32_t layer, int32_t proj, const void *x, const void *Wt, void *y,
                     float scale, void *workspace, size_t workspace_bytes, void *stream);

/* One-call form: index + apply (uses one of 4 internal plans in rotation; blocks the
 * host only if the plan used 4 calls ago is still in flight). */
int lora_apply(lora_cache_t *c, int32_t layer, int32_t proj, const void *x, void *base_out, int32_t T,
               const int32_t *seg_offsets, const int32_t *seg_slot, const int32_t *seg_rank, int32_t n_seg,
               float scale, void *stream);

/* When off (0), applies record no last-use event and fills do not wait for earlier
 * applies: the caller then keeps refills away from slots in use (reference counts).
 * Default on (1).  Turn off while capturing applies into a HIP graph. */
int lora_cache_set_fencing(lora_cache_t *c, int32_t on);

/* Per-kernel timing for benchmarks.  While on (1), every kernel an apply launches carries a
 * pair of HIP events that the runtime stamps with the kernel's own start and end.
 * lora_cache_read_timing waits for the recorded events, adds up the elapsed milliseconds and
 * launch counts per kernel kind since the last read, and forgets them. */
enum {
    LORA_K_MFMA_REDUCE = 0, LORA_K_MFMA_SHRINK = 1, LORA_K_GEMV_SHRINK = 2, LORA_K_MFMA_EXPAND = 3, LORA_K_GEMV_EXPAND = 4,
    LORA_K_GEMV_FUSED = 5, LORA_K_LINEAR = 6, LORA_K_COUNT = 7
};
int lora_cache_set_timing(lora_cache_t *c, int32_t on);
int lora_cache_read_timing(lora_cache_t *c, double ms[LORA_K_COUNT], int64_t launches[LORA_K_COUNT]);

/* Blocks until `stream` is idle, then reports whether any kernel of this cache gave up a
 * bounded wait since the last call (*fault = 1; the outputs of that apply are then invalid)
 * and clears the flag.  The fused GEMV launch is the only kernel that waits; with a working
 * device the flag never rises.  The flag lives in pinned host memory that the kernel writes
 * directly, so applies also see it without any synchronisation: once it is up they return
 * LORA_E_FAULT until this call has cleared it. */
int lora_cache_check_fault(lora_cache_t *c, void *stream, int32_t *fault);

const char *lora_strerror(int status);
int lora_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LORA_CACHE_H */
