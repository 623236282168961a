// Adaptive-Wait-Depth batching of the short queue: host-only decision state (see laps_awd_* in include/laps.h).
//
// Algorithm 1 of the paper keeps a waiting window W and a target depth D.  A round collects short
// requests until the window expires or the target depth is reached, leaves early when the smallest slack
// DDL_i - (t + S_hat) over the batch and the next request falls to sigma (Algorithm 1) or the head of the
// line has waited T_max (Section 3.2a), pads the batch to the nearest captured shape within the memory
// budget, and then adapts: a filled target sets W to the observed fill time (clipped), an unfilled one
// lowers D to the observed depth.  The SLA-constrained mode of Section 3.2a replaces W for the round by
// clip(min(W_SLA, W_GR)) evaluated when the round's timer starts.
//
// The object holds W, D and the timer; the caller owns the queue and the clock and polls at every event
// (arrival, instance free, the wake-up time returned by the previous poll).  The three timed conditions are
// evaluated as instants (slack_i <= sigma  <=>  t >= DDL_i - S_hat - sigma, and so on), so that a poll at a
// returned wake-up time sees the condition it was woken for as true whatever the rounding.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "../../include/laps.h"

void laps_set_error(const char* fmt, ...);

struct laps_awd {
    std::vector<int32_t> len_buckets, depths;
    int64_t mem_budget, fuse_budget;
    double sigma, w_min, w_max, s_hat, t_max, delta, rate_eps;
    bool sla_window, d_regrow;
    double window;          // W
    int32_t target_depth;   // D
    int32_t depth_cap;      // D at creation
    double free_at;         // instance free for the next short batch
    bool timer_running;
    double t_start, w_round;
    std::vector<int32_t> bucket_scratch;
    std::vector<double> s_hat_table;   // [len bucket][depth], NaN = no entry; empty = no table
};

namespace {

const double kInf = std::numeric_limits<double>::infinity();

double clipd(double v, double lo, double hi) { return std::min(std::max(v, lo), hi); }

// smallest length bucket holding n, or -1
int32_t bucket_of(const laps_awd* a, int32_t n) {
    for (int32_t b : a->len_buckets)
        if (b >= n) return b;
    return -1;
}

// smallest captured depth >= rows with len_bucket * depth within the budget, or 0
int32_t nearest_depth(const laps_awd* a, int32_t len_bucket, int32_t rows, int64_t budget) {
    for (int32_t d : a->depths)
        if (d >= rows) return (int64_t)d * len_bucket <= budget ? d : 0;
    return 0;
}

struct Batch {
    int32_t n = 0, len_bucket = 0, next = -1;
};

// Bucket-first greedy fill from the waiting queue (arrival order): the head's bucket first, then the rest;
// a request that would not fit any captured shape within the budget is passed over.
Batch form_batch(laps_awd* a, int32_t n_waiting, const int32_t* new_len, int32_t* take_idx) {
    Batch b;
    a->bucket_scratch.resize((size_t)n_waiting);
    for (int32_t i = 0; i < n_waiting; ++i) a->bucket_scratch[(size_t)i] = bucket_of(a, new_len[i]);
    const int32_t head = a->bucket_scratch[0];
    for (int pass = 0; pass < 2 && b.next < 0; ++pass) {
        for (int32_t i = 0; i < n_waiting; ++i) {
            const int32_t bk = a->bucket_scratch[(size_t)i];
            if ((bk == head) != (pass == 0)) continue;
            if (b.n >= a->target_depth) {
                b.next = i;
                break;
            }
            const int32_t lb = std::max(b.len_bucket, bk);
            // another bucket than the head's joins only while the fused shape stays within the fusion budget
            const int64_t budget = pass == 0 ? a->mem_budget : std::min(a->mem_budget, a->fuse_budget);
            if (nearest_depth(a, lb, b.n + 1, budget) == 0) continue;
            take_idx[b.n++] = i;
            b.len_bucket = lb;
        }
    }
    return b;
}

// service-time estimate for the batch as it stands: the table entry of its shape, else the default
double s_hat_of(const laps_awd* a, const Batch& b) {
    if (b.n == 0 || a->s_hat_table.empty()) return a->s_hat;
    const int32_t d = nearest_depth(a, b.len_bucket, b.n, a->mem_budget);
    size_t li = 0, di = 0;
    while (li < a->len_buckets.size() && a->len_buckets[li] != b.len_bucket) ++li;
    while (di < a->depths.size() && a->depths[di] != d) ++di;
    if (li == a->len_buckets.size() || di == a->depths.size()) return a->s_hat;   // no captured shape: default
    const double v = a->s_hat_table[li * a->depths.size() + di];
    return std::isnan(v) ? a->s_hat : v;
}

}  // namespace

extern "C" int laps_awd_set_service_table(laps_awd* a, const double* s_hat_us) {
    if (!a) {
        laps_set_error("awd_set_service_table: NULL handle");
        return LAPS_EINVAL;
    }
    if (!s_hat_us) {
        a->s_hat_table.clear();
        return LAPS_OK;
    }
    const size_t n = a->len_buckets.size() * a->depths.size();
    for (size_t i = 0; i < n; ++i)
        if (s_hat_us[i] < 0.0) {
            laps_set_error("awd_set_service_table: negative estimate at entry %zu", i);
            return LAPS_EINVAL;
        }
    a->s_hat_table.assign(s_hat_us, s_hat_us + n);
    return LAPS_OK;
}

extern "C" int laps_awd_create(const laps_awd_params* p, double first_slack_us, laps_awd** out) {
    if (!p || !out || !p->len_buckets || !p->depths || p->n_len_buckets <= 0 || p->n_depths <= 0) {
        laps_set_error("awd: NULL argument or empty grid");
        return LAPS_EINVAL;
    }
    for (int i = 0; i < p->n_len_buckets; ++i)
        if (p->len_buckets[i] <= 0 || (i && p->len_buckets[i] <= p->len_buckets[i - 1])) {
            laps_set_error("awd: len_buckets must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    for (int i = 0; i < p->n_depths; ++i)
        if (p->depths[i] <= 0 || (i && p->depths[i] <= p->depths[i - 1])) {
            laps_set_error("awd: depths must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    if (!(p->w_min_us >= 0.0) || !(p->w_max_us >= p->w_min_us) || !std::isfinite(p->w_max_us) || !(p->s_hat_us >= 0.0) ||
        std::isnan(p->sigma_us) || std::isnan(p->t_max_us) || !(p->delta_us >= 0.0) || !(p->rate_eps > 0.0) ||
        std::isnan(first_slack_us)) {
        laps_set_error("awd: need 0 <= w_min <= w_max < inf, s_hat >= 0, delta >= 0, rate_eps > 0 and no NaN");
        return LAPS_EINVAL;
    }
    // every length bucket must fit the budget alone, else a request of that bucket could never leave
    if ((int64_t)p->depths[0] * p->len_buckets[p->n_len_buckets - 1] > p->mem_budget) {
        laps_set_error("awd: mem_budget %lld is below the smallest shape of the largest bucket (%d x %d)",
                       (long long)p->mem_budget, p->len_buckets[p->n_len_buckets - 1], p->depths[0]);
        return LAPS_EINVAL;
    }
    laps_awd* a = new (std::nothrow) laps_awd();
    if (!a) {
        laps_set_error("awd: out of host memory");
        return LAPS_ENOMEM;
    }
    a->len_buckets.assign(p->len_buckets, p->len_buckets + p->n_len_buckets);
    a->depths.assign(p->depths, p->depths + p->n_depths);
    a->mem_budget = p->mem_budget;
    a->fuse_budget = p->fuse_budget < 0 ? p->mem_budget : p->fuse_budget;
    a->sigma = p->sigma_us;
    a->w_min = p->w_min_us;
    a->w_max = p->w_max_us;
    a->s_hat = p->s_hat_us;
    a->t_max = p->t_max_us;
    a->delta = p->delta_us;
    a->rate_eps = p->rate_eps;
    a->sla_window = p->sla_window != 0;
    a->d_regrow = p->d_regrow != 0;
    a->window = clipd(first_slack_us, a->w_min, a->w_max);
    int32_t dmax = 0;
    for (int32_t d : a->depths)
        if ((int64_t)d * a->len_buckets[0] <= a->mem_budget) dmax = d;   // the smallest bucket admits the deepest shape
    a->target_depth = a->depth_cap = dmax;
    a->free_at = -kInf;
    a->timer_running = false;
    a->t_start = a->w_round = 0.0;
    *out = a;
    return LAPS_OK;
}

extern "C" void laps_awd_destroy(laps_awd* a) { delete a; }

extern "C" double laps_awd_window_us(const laps_awd* a) { return a ? a->window : NAN; }

extern "C" int32_t laps_awd_target_depth(const laps_awd* a) { return a ? a->target_depth : -1; }

extern "C" int laps_awd_begin_round(laps_awd* a, double free_at_us) {
    if (!a || std::isnan(free_at_us)) {
        laps_set_error("awd_begin_round: NULL handle or NaN time");
        return LAPS_EINVAL;
    }
    if (a->timer_running) {
        laps_set_error("awd_begin_round: a round is already collecting (poll it to a dispatch first)");
        return LAPS_EINVAL;
    }
    a->free_at = free_at_us;
    return LAPS_OK;
}

extern "C" int laps_awd_poll(laps_awd* a, double now_us, double rate_hat, int32_t n_waiting, const double* arrival_us,
                             const double* ddl_us, const int32_t* new_len, int32_t* action, int32_t* n_take,
                             int32_t* take_idx, int32_t* len_bucket, int32_t* depth, int32_t* reason, double* wake_us) {
    if (!a || !action || !n_take || !len_bucket || !depth || !reason || !wake_us || n_waiting < 0 ||
        (n_waiting > 0 && (!arrival_us || !ddl_us || !new_len || !take_idx)) || std::isnan(now_us) || std::isnan(rate_hat)) {
        laps_set_error("awd_poll: NULL argument, negative count or NaN time");
        return LAPS_EINVAL;
    }
    *action = LAPS_AWD_WAIT;
    *n_take = 0;
    *len_bucket = *depth = 0;
    *reason = LAPS_AWD_NONE;
    *wake_us = kInf;
    if (n_waiting == 0) return LAPS_OK;
    for (int32_t i = 0; i < n_waiting; ++i) {
        if (new_len[i] <= 0 || bucket_of(a, new_len[i]) < 0) {
            laps_set_error("awd_poll: request %d has new_len %d outside the bucket grid", i, new_len[i]);
            return LAPS_EINVAL;
        }
        if (std::isnan(arrival_us[i]) || std::isnan(ddl_us[i]) || arrival_us[i] > now_us ||
            (i && arrival_us[i] < arrival_us[i - 1])) {
            laps_set_error("awd_poll: waiting requests must be in arrival order with arrival <= now (request %d)", i);
            return LAPS_EINVAL;
        }
    }
    if (now_us < a->free_at) {          // the instance is still busy with the previous short step
        *wake_us = a->free_at;
        return LAPS_OK;
    }
    Batch b = form_batch(a, n_waiting, new_len, take_idx);
    if (!a->timer_running) {
        a->timer_running = true;
        a->t_start = std::max(a->free_at, arrival_us[0]);
        a->w_round = a->window;
        if (a->sla_window) {
            double slack = kInf;
            const double sh = s_hat_of(a, b);
            for (int32_t i = 0; i < n_waiting; ++i) slack = std::min(slack, ddl_us[i] - a->t_start - sh);
            const double w_sla = std::max(0.0, slack - a->delta);
            const double w_gr = (double)std::max(0, a->target_depth - b.n) / std::max(rate_hat, a->rate_eps);
            a->w_round = clipd(std::min(w_sla, w_gr), a->w_min, a->w_max);
        }
    }
    double t_sla = kInf;
    const double s_now = s_hat_of(a, b);
    for (int32_t j = 0; j < b.n; ++j) t_sla = std::min(t_sla, ddl_us[take_idx[j]] - s_now - a->sigma);
    if (b.next >= 0) t_sla = std::min(t_sla, ddl_us[b.next] - s_now - a->sigma);
    const double t_cap = arrival_us[0] + a->t_max;
    const double t_win = a->t_start + a->w_round;
    int32_t why = LAPS_AWD_NONE;
    if (b.n >= a->target_depth) why = LAPS_AWD_DEPTH;
    else if (now_us >= t_sla) why = LAPS_AWD_SLA;
    else if (now_us >= t_cap) why = LAPS_AWD_TMAX;
    else if (now_us >= t_win) why = LAPS_AWD_WINDOW;
    if (why == LAPS_AWD_NONE) {
        *wake_us = std::min(t_sla, std::min(t_cap, t_win));
        return LAPS_OK;
    }
    // dispatch: pad to the nearest captured shape, then adapt W and D
    const int32_t d = b.n;
    const double tau = now_us - a->t_start;
    *action = LAPS_AWD_DISPATCH;
    *n_take = d;
    *len_bucket = b.len_bucket;
    *depth = nearest_depth(a, b.len_bucket, d, a->mem_budget);
    *reason = why;
    if (d >= a->target_depth) {
        a->window = clipd(tau, a->w_min, a->w_max);
        if (a->d_regrow && n_waiting - d >= d) {
            for (int32_t x : a->depths)
                if (x > a->target_depth && x <= a->depth_cap) {
                    a->target_depth = x;
                    break;
                }
        }
    } else {
        a->target_depth = d;
    }
    a->timer_running = false;
    a->free_at = now_us;
    return LAPS_OK;
}
