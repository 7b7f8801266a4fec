// Request scheduler of paper section 4.3 (host side): see include/lora_sched.h for the contract.
#include <algorithm>
#include <cmath>
#include <deque>
#include <limits>
#include <new>
#include <unordered_map>
#include <vector>

#include "lora_cache.h"
#include "lora_sched.h"

namespace {

struct Loan {
    int32_t queue;   // whose quota the tokens are
    int64_t tokens;
};

struct Req {
    int64_t id = 0, adapter = 0;
    int32_t input = 0, output = 0, rank = 0, queue = 0;
    std::vector<Loan> loans;
};

// Tokens on offer to one admission pass: parts of the free quota of one or more queues, spent in order.
struct Purse {
    std::vector<Loan> parts;
    int64_t total() const
    {
        int64_t t = 0;
        for (const Loan &l : parts) t += l.tokens;
        return t;
    }
};

}  // namespace

struct lora_sched {
    std::vector<int64_t> quota, free_tokens;
    std::vector<double> bounds;
    int32_t max_input = 1, max_output = 1, max_rank = 1, tokens_per_rank = 0;
    double a = 0.4, b = 0.6;
    std::vector<std::deque<Req>> lanes;
    std::unordered_map<int64_t, Req> running;
    std::unordered_map<int64_t, int32_t> waiting;  // req id -> queue
};

namespace {

int64_t tokens_needed(const lora_sched &s, const Req &r)
{
    return (int64_t)r.input + r.output + (int64_t)r.rank * s.tokens_per_rank;
}

// Admit from the head of lane q while the purse pays; -> tokens spent.  Stops when `room` requests were taken.
int64_t admit(lora_sched &s, int32_t q, Purse &purse, std::vector<int64_t> &batch, int32_t room)
{
    int64_t spent = 0;
    std::deque<Req> &lane = s.lanes[q];
    while (!lane.empty() && (int32_t)batch.size() < room) {
        Req &head = lane.front();
        const int64_t need = tokens_needed(s, head);
        if (purse.total() < need) break;
        int64_t owed = need;
        for (Loan &part : purse.parts) {
            if (owed == 0) break;
            const int64_t take = std::min(owed, part.tokens);
            if (take == 0) continue;
            part.tokens -= take;
            s.free_tokens[part.queue] -= take;
            head.loans.push_back({part.queue, take});
            owed -= take;
        }
        spent += need;
        batch.push_back(head.id);
        s.waiting.erase(head.id);
        const int64_t id = head.id;
        s.running.emplace(id, std::move(head));
        lane.pop_front();
    }
    return spent;
}

// sum of squared distances to the mean of xs[i..j), from prefix sums of x and x^2
struct Prefix {
    std::vector<double> s1, s2;
    explicit Prefix(const std::vector<double> &xs) : s1(xs.size() + 1, 0.0), s2(xs.size() + 1, 0.0)
    {
        for (size_t i = 0; i < xs.size(); ++i) {
            s1[i + 1] = s1[i] + xs[i];
            s2[i + 1] = s2[i] + xs[i] * xs[i];
        }
    }
    double mean(int i, int j) const { return (s1[j] - s1[i]) / (double)(j - i); }
    double sse(int i, int j) const
    {
        const double m = mean(i, j);
        return std::max(0.0, (s2[j] - s2[i]) - m * (s1[j] - s1[i]));
    }
};

// Exact 1-D K-means over sorted xs by dynamic programming over the last cut; -> WCSS, fills centroids.
double cluster_line(const std::vector<double> &xs, const Prefix &pre, int k, std::vector<double> *centroids)
{
    const int n = (int)xs.size();
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<std::vector<double>> cost(k + 1, std::vector<double>(n + 1, inf));
    std::vector<std::vector<int>> from(k + 1, std::vector<int>(n + 1, 0));
    cost[0][0] = 0.0;
    for (int c = 1; c <= k; ++c)
        for (int end = c; end <= n; ++end)
            for (int start = c - 1; start < end; ++start) {
                if (cost[c - 1][start] == inf) continue;
                const double v = cost[c - 1][start] + pre.sse(start, end);
                if (v < cost[c][end]) {
                    cost[c][end] = v;
                    from[c][end] = start;
                }
            }
    if (centroids) {
        centroids->assign(k, 0.0);
        int end = n;
        for (int c = k; c >= 1; --c) {
            const int start = from[c][end];
            (*centroids)[c - 1] = pre.mean(start, end);
            end = start;
        }
    }
    return cost[k][n];
}

}  // namespace

extern "C" {

double lora_sched_wrs(int32_t input_len, int32_t output_len, int32_t rank, int32_t max_input, int32_t max_output,
                      int32_t max_rank, double a_input, double b_output)
{
    if (max_input < 1 || max_output < 1 || max_rank < 1) return std::numeric_limits<double>::quiet_NaN();
    if (a_input == 0.0 && b_output == 0.0) {
        a_input = 0.4;
        b_output = 0.6;
    }
    const double in = (double)input_len / (double)max_input, out = (double)output_len / (double)max_output;
    return (a_input * in + b_output * out) * ((double)rank / (double)max_rank);
}

int lora_sched_create(const lora_sched_config_t *cfg, lora_sched_t **out)
{
    if (!cfg || !out || cfg->n_queues < 1 || !cfg->quota || (cfg->n_queues > 1 && !cfg->boundaries) || cfg->max_input < 1 ||
        cfg->max_output < 1 || cfg->max_rank < 1 || cfg->tokens_per_rank < 0 || !(cfg->a_input >= 0) || !(cfg->b_output >= 0))
        return LORA_E_INVAL;
    for (int32_t q = 0; q < cfg->n_queues; ++q)
        if (cfg->quota[q] < 0) return LORA_E_INVAL;
    for (int32_t q = 0; q + 1 < cfg->n_queues; ++q) {
        if (!(cfg->boundaries[q] == cfg->boundaries[q])) return LORA_E_INVAL;  // NaN
        if (q > 0 && cfg->boundaries[q] < cfg->boundaries[q - 1]) return LORA_E_INVAL;
    }
    lora_sched *s = new (std::nothrow) lora_sched;
    if (!s) return LORA_E_NOMEM;
    s->quota.assign(cfg->quota, cfg->quota + cfg->n_queues);
    s->free_tokens = s->quota;
    if (cfg->n_queues > 1) s->bounds.assign(cfg->boundaries, cfg->boundaries + cfg->n_queues - 1);
    s->max_input = cfg->max_input;
    s->max_output = cfg->max_output;
    s->max_rank = cfg->max_rank;
    s->tokens_per_rank = cfg->tokens_per_rank;
    if (cfg->a_input != 0.0 || cfg->b_output != 0.0) {
        s->a = cfg->a_input;
        s->b = cfg->b_output;
    }
    s->lanes.resize(cfg->n_queues);
    *out = s;
    return LORA_OK;
}

int lora_sched_destroy(lora_sched_t *s)
{
    delete s;
    return LORA_OK;
}

int lora_sched_submit(lora_sched_t *s, int64_t req_id, int32_t input_len, int32_t output_len, int64_t adapter_id,
                      int32_t rank, int32_t *queue)
{
    if (!s || input_len < 0 || output_len < 0 || rank < 1) return LORA_E_INVAL;
    if (s->waiting.count(req_id) || s->running.count(req_id)) return LORA_E_INVAL;
    const double size = lora_sched_wrs(input_len, output_len, rank, s->max_input, s->max_output, s->max_rank, s->a, s->b);
    // the first boundary above the size names the queue; sizes at a boundary belong to the queue above it
    const int32_t q = (int32_t)(std::upper_bound(s->bounds.begin(), s->bounds.end(), size) - s->bounds.begin());
    Req r;
    r.id = req_id;
    r.adapter = adapter_id;
    r.input = input_len;
    r.output = output_len;
    r.rank = rank;
    r.queue = q;
    s->lanes[q].push_back(std::move(r));
    s->waiting[req_id] = q;
    if (queue) *queue = q;
    return LORA_OK;
}

int lora_sched_generate_batch(lora_sched_t *s, int64_t *req_ids, int32_t cap, int32_t *n)
{
    if (!s || !n || cap < 0 || (cap > 0 && !req_ids)) return LORA_E_INVAL;
    std::vector<int64_t> batch;
    Purse spare;
    const int32_t K = (int32_t)s->lanes.size();
    for (int32_t q = 0; q < K; ++q) {  // initial admission: own quota
        Purse own;
        own.parts.push_back({q, s->free_tokens[q]});
        admit(*s, q, own, batch, cap);
        if (s->lanes[q].empty() && own.parts[0].tokens > 0) spare.parts.push_back(own.parts[0]);
    }
    for (int32_t q = 0; q < K && spare.total() > 0; ++q) admit(*s, q, spare, batch, cap);  // redistribution
    for (size_t i = 0; i < batch.size(); ++i) req_ids[i] = batch[i];
    *n = (int32_t)batch.size();
    return LORA_OK;
}

int lora_sched_finish(lora_sched_t *s, int64_t req_id)
{
    if (!s) return LORA_E_INVAL;
    auto it = s->running.find(req_id);
    if (it == s->running.end()) return LORA_E_NOTFOUND;
    for (const Loan &l : it->second.loans) s->free_tokens[l.queue] += l.tokens;
    s->running.erase(it);
    return LORA_OK;
}

int lora_sched_queue_state(const lora_sched_t *s, int32_t queue, int64_t *free_tokens, int32_t *n_waiting)
{
    if (!s || queue < 0 || queue >= (int32_t)s->lanes.size()) return LORA_E_INVAL;
    if (free_tokens) *free_tokens = s->free_tokens[queue];
    if (n_waiting) *n_waiting = (int32_t)s->lanes[queue].size();
    return LORA_OK;
}

int lora_sched_waiting_adapters(const lora_sched_t *s, int64_t *adapter_ids, int32_t cap, int32_t *n)
{
    if (!s || !n || cap < 0 || (cap > 0 && !adapter_ids)) return LORA_E_INVAL;
    int32_t count = 0;
    for (const auto &lane : s->lanes)
        for (const Req &r : lane) {
            if (count < cap) adapter_ids[count] = r.adapter;
            ++count;
        }
    *n = count;
    return LORA_OK;
}

int lora_sched_fit_queues(const double *sizes, int32_t n, int32_t k_max, int32_t *k, double *boundaries)
{
    if (!sizes || n < 1 || n > 4096 || k_max < 1 || k_max > 8 || !k || (k_max > 1 && !boundaries)) return LORA_E_INVAL;
    std::vector<double> xs(sizes, sizes + n);
    for (double v : xs)
        if (!(v == v)) return LORA_E_INVAL;
    std::sort(xs.begin(), xs.end());
    int n_distinct = 1;
    for (int i = 1; i < n; ++i) n_distinct += xs[i] != xs[i - 1];
    const int top = std::min<int>(k_max, n_distinct);
    const Prefix pre(xs);
    std::vector<double> wcss(top + 1, 0.0);
    for (int c = 1; c <= top; ++c) wcss[c] = cluster_line(xs, pre, c, nullptr);
    int best = 1;
    double best_drop = 0.0;
    for (int c = 2; c <= top; ++c) {
        if (wcss[c - 1] <= 0.0) break;
        const double drop = (wcss[c - 1] - wcss[c]) / wcss[c - 1];
        if (drop > best_drop) {
            best = c;
            best_drop = drop;
        }
    }
    std::vector<double> centroids;
    cluster_line(xs, pre, best, &centroids);
    for (int i = 0; i + 1 < best; ++i) boundaries[i] = (centroids[i] + centroids[i + 1]) / 2;
    *k = best;
    return LORA_OK;
}

int64_t lora_sched_min_quota(double max_request_tokens, double duration, double slo, double arrival_rate)
{
    if (!(max_request_tokens > 0) || !(duration > 0) || !(slo > 0) || !(arrival_rate >= 0)) return -1;
    return (int64_t)std::ceil(max_request_tokens * duration * (1.0 / slo + arrival_rate));
}

int lora_sched_assign_quotas(int64_t total_tokens, const int64_t *least, const double *weights, int32_t n_queues,
                             int64_t *quota)
{
    if (!least || !weights || !quota || n_queues < 1 || total_tokens < 0) return LORA_E_INVAL;
    int64_t need = 0;
    double wsum = 0;
    for (int32_t q = 0; q < n_queues; ++q) {
        if (least[q] < 0 || !(weights[q] >= 0)) return LORA_E_INVAL;
        need += least[q];
        wsum += weights[q];
    }
    if (!(wsum > 0)) return LORA_E_INVAL;
    if (need > total_tokens) return LORA_E_NOMEM;
    const int64_t rest = total_tokens - need;
    int64_t given = 0;
    for (int32_t q = 0; q < n_queues; ++q) {
        quota[q] = least[q] + (int64_t)std::floor((double)rest * (weights[q] / wsum));
        given += quota[q];
    }
    for (int64_t left = total_tokens - given, q = 0; left > 0; --left, ++q) ++quota[q % n_queues];
    return LORA_OK;
}

}  // extern "C"
