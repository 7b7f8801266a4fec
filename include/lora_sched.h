/* Request scheduler of the many-adapter serving system (paper section 4.3): request size, size-ranged
 * queues with token quotas, two-phase batch admission, number of queues and boundaries from a
 * clustering of the request sizes, least quota per queue from an M/M/1 model.
 *
 * Host-side only (no device memory, no streams); plain C ABI.  The batches it returns are what
 * becomes the seg_* arrays of lora_apply: one segment per admitted request and iteration.
 * Not thread-safe: one scheduler is driven by one thread.  All functions return LORA_OK (0) or a
 * negative lora_status of lora_cache.h unless stated otherwise. */
#ifndef LORA_SCHED_H
#define LORA_SCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lora_sched lora_sched_t; /* opaque */

typedef struct {
    int32_t n_queues;          /* K >= 1 */
    const int64_t *quota;      /* [n_queues] tokens each queue owns; queue 0 holds the smallest requests */
    const double *boundaries;  /* [n_queues - 1] ascending request sizes: queue i takes sizes in
                                  [boundaries[i-1], boundaries[i]) */
    int32_t max_input, max_output, max_rank; /* normalisers of the request size, all >= 1 */
    int32_t tokens_per_rank;   /* memory of one rank of an adapter, expressed in tokens (>= 0) */
    double a_input, b_output;  /* the paper's A = 0.4 and B = 0.6 if both are 0 */
} lora_sched_config_t;

/* Weighted request size ("WRS", section 4.3 item 1): (A * input / max_input + B * output / max_output)
 * * rank / max_rank, an estimate of the request's run time used only to pick its queue.  NaN on a
 * normaliser < 1. */
double lora_sched_wrs(int32_t input_len, int32_t output_len, int32_t rank, int32_t max_input, int32_t max_output,
                      int32_t max_rank, double a_input, double b_output);

/* The arrays of cfg are copied.  LORA_E_INVAL on a bad configuration (descending boundaries, negative quota ...). */
int lora_sched_create(const lora_sched_config_t *cfg, lora_sched_t **out);
int lora_sched_destroy(lora_sched_t *s);

/* A request arrives: known input length, predicted output length, its adapter and that adapter's rank.
 * It joins the end of the queue its size selects; *queue (may be NULL) receives which.
 * LORA_E_INVAL on negative lengths, rank < 1 or a req_id that is already waiting or running. */
int lora_sched_submit(lora_sched_t *s, int64_t req_id, int32_t input_len, int32_t output_len, int64_t adapter_id,
                      int32_t rank, int32_t *queue);

/* Form the batch of the next iteration (section 4.3 item 2, both phases): every queue, smallest
 * requests first, admits requests in arrival order out of its own free quota and stops at the
 * first that does not fit -- a request needs input_len + output_len + rank * tokens_per_rank tokens;
 * a queue that ran empty gives its unused quota to a spare bucket; then every queue, in the same
 * order, admits further requests out of the bucket.  Tokens of the bucket are drawn in the order of
 * the queues that gave them and return to those queues when the request ends.
 * req_ids [cap] receives the admitted requests in admission order, *n their number; admission stops
 * early (requests stay queued) when cap is reached.  Admitted requests are "running" until
 * lora_sched_finish. */
int lora_sched_generate_batch(lora_sched_t *s, int64_t *req_ids, int32_t cap, int32_t *n);

/* The request has ended (or was squashed): every token it borrowed returns to the queue it belongs to.
 * LORA_E_NOTFOUND if req_id is not running. */
int lora_sched_finish(lora_sched_t *s, int64_t req_id);

/* State for tests and for the cache manager: free tokens of a queue, number of waiting requests of a
 * queue, and the adapters of all waiting requests (what lora_cache_acquire spares from eviction and
 * what is worth prefetching), queue by queue in arrival order; *n receives how many there are,
 * at most cap are written. */
int lora_sched_queue_state(const lora_sched_t *s, int32_t queue, int64_t *free_tokens, int32_t *n_waiting);
int lora_sched_waiting_adapters(const lora_sched_t *s, int64_t *adapter_ids, int32_t cap, int32_t *n);

/* Number of queues and boundaries from observed request sizes (section 4.3 item 4): exact
 * one-dimensional K-means for K = 1 .. k_max (k_max <= 8; the paper uses 4); the K whose step from
 * K - 1 removes the largest fraction of the remaining within-cluster sum of squares (taken literally,
 * "the K with minimal WCSS" would always be k_max); boundaries = midpoints between consecutive
 * centroids.  boundaries must hold k_max - 1 values; *k receives K.  n >= 1, at most 4096 sizes
 * (the clustering is quadratic in n). */
int lora_sched_fit_queues(const double *sizes, int32_t n, int32_t k_max, int32_t *k, double *boundaries);

/* Least quota of a queue (section 4.3 item 5): S * D * (1 / SLO + lambda) tokens, rounded up, for a largest
 * request of S tokens that takes D seconds, arrivals at lambda per second and a time-in-system bound
 * SLO -- the M/M/1 sojourn time 1 / (mu - lambda) with mu = quota / (S * D).  -1 on a non-positive argument. */
int64_t lora_sched_min_quota(double max_request_tokens, double duration, double slo, double arrival_rate);

/* Every queue its least quota, the remaining tokens in proportion to weights (shares rounded down,
 * the tokens the rounding leaves go one each to queues 0, 1, ...).  LORA_E_NOMEM if total is less than
 * the sum of the least quotas. */
int lora_sched_assign_quotas(int64_t total_tokens, const int64_t *least, const double *weights, int32_t n_queues,
                             int64_t *quota);

#ifdef __cplusplus
}
#endif
#endif
