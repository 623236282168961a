// Length-aware bucket plan: host-only, integer-only (see laps_plan_buckets in include/laps.h).
//
// Classification by length into a short and a long queue follows Section 3.2 ("Mutual exclusion");
// the (length, depth) bucket grid, padding up to a bucket and grouping by the same bucket follow
// Section 3.1 ("Graph capture and bucketization"); matching a batch to a captured shape whose depth
// covers it within the budget, else using the standard path, follows Algorithm 1; chunking of long
// requests follows the deadline-free mode of Section 3.2.
//
// Covering n requests of one length bucket with captured depths: every depth is at most the cap
// D = largest depth within the budget, so ceil(n/D) launches are necessary and sufficient.  With
// that count fixed, writing each depth as D - deficit turns "fewest padded rows" into "largest total
// deficit not exceeding the slack ceil(n/D)*D - n" (< D), a tiny subset-sum over the few non-cap
// depths; "larger depths first" then means as few non-cap batches as possible and, among them,
// greedily the largest feasible depth at each position.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <vector>

#include "../../include/laps.h"

void laps_set_error(const char* fmt, ...);

struct laps_plan {
    std::vector<int32_t> req_class, req_bucket, req_batch, req_row;
    std::vector<int32_t> batch_len_bucket, batch_depth, batch_graph_ok, batch_req_offset, batch_req_ids;
    std::vector<int32_t> long_req, long_chunk_offset, long_chunk_len;
};

namespace {

// Depth multiset (descending) covering n rows with depths from `allowed` (ascending, non-empty).
std::vector<int32_t> cover_with_depths(int64_t n, const std::vector<int32_t>& allowed) {
    const int32_t cap = allowed.back();
    const int64_t count = (n + cap - 1) / cap;
    const int32_t slack = (int32_t)(count * cap - n);  // 0 <= slack < cap
    const int nd = (int)allowed.size() - 1;            // non-cap depths: allowed[0..nd)
    const int max_items = (int)std::min<int64_t>(count, slack);
    // g[c][s][j]: exactly c batches, each of a non-cap depth with index < j, deficits summing to s
    auto idx = [&](int c, int s, int j) { return ((size_t)c * (slack + 1) + s) * (nd + 1) + j; };
    std::vector<char> g((size_t)(max_items + 1) * (slack + 1) * (nd + 1), 0);
    for (int j = 0; j <= nd; ++j) g[idx(0, 0, j)] = 1;
    for (int c = 1; c <= max_items; ++c)
        for (int s = 0; s <= slack; ++s)
            for (int j = 1; j <= nd; ++j) {
                const int def = cap - allowed[j - 1];
                char ok = g[idx(c, s, j - 1)];
                if (!ok && def <= s) ok = g[idx(c - 1, s - def, j)];
                g[idx(c, s, j)] = ok;
            }
    int best_s = 0, best_c = 0;
    for (int s = slack; s >= 0; --s) {
        int found = -1;
        for (int c = 0; c <= max_items; ++c)
            if (g[idx(c, s, nd)]) {
                found = c;
                break;
            }
        if (found >= 0) {
            best_s = s;
            best_c = found;
            break;
        }
    }
    std::vector<int32_t> out((size_t)(count - best_c), cap);
    int s = best_s, j = nd;
    for (int c = best_c; c > 0; --c) {
        // largest depth (index < j ... allowing repeats of the same depth) that keeps the rest feasible
        int pick = -1;
        for (int jj = j; jj >= 1; --jj) {
            const int def = cap - allowed[jj - 1];
            if (def <= s && g[idx(c - 1, s - def, jj)]) {
                pick = jj;
                break;
            }
        }
        out.push_back(allowed[pick - 1]);
        s -= cap - allowed[pick - 1];
        j = pick;
    }
    return out;
}

}  // namespace

extern "C" int laps_plan_buckets(const laps_plan_params* p, int32_t n_req, const int32_t* new_len,
                                 const int32_t* prefix_len, laps_plan** out) {
    if (!p || !out || n_req < 0 || (n_req > 0 && (!new_len || !prefix_len))) {
        laps_set_error("plan: NULL argument or negative request count");
        return LAPS_EINVAL;
    }
    if (p->n_len_buckets < 1 || !p->len_buckets || p->n_depths < 1 || !p->depths || p->token_budget < 1 ||
        p->long_chunk < 1 || p->short_max_len < 1) {
        laps_set_error("plan: empty grid or non-positive budget / chunk / boundary");
        return LAPS_EINVAL;
    }
    for (int i = 0; i < p->n_len_buckets; ++i)
        if (p->len_buckets[i] < 1 || (i > 0 && p->len_buckets[i] <= p->len_buckets[i - 1])) {
            laps_set_error("plan: len_buckets must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    for (int i = 0; i < p->n_depths; ++i)
        if (p->depths[i] < 1 || (i > 0 && p->depths[i] <= p->depths[i - 1])) {
            laps_set_error("plan: depths must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    if (p->short_max_len > p->len_buckets[p->n_len_buckets - 1]) {
        laps_set_error("plan: short_max_len %d exceeds the largest length bucket %d", p->short_max_len,
                       p->len_buckets[p->n_len_buckets - 1]);
        return LAPS_EINVAL;
    }
    for (int i = 0; i < n_req; ++i)
        if (new_len[i] < 1 || prefix_len[i] < 0) {
            laps_set_error("plan: request %d has new_len %d, prefix_len %d", i, new_len[i], prefix_len[i]);
            return LAPS_EINVAL;
        }

    laps_plan* pl = new (std::nothrow) laps_plan();
    if (!pl) {
        laps_set_error("plan: out of host memory");
        return LAPS_ENOMEM;
    }
    try {
        pl->req_class.assign(n_req, 0);
        pl->req_bucket.assign(n_req, -1);
        pl->req_batch.assign(n_req, -1);
        pl->req_row.assign(n_req, -1);
        std::vector<std::vector<int32_t>> per_bucket(p->n_len_buckets);
        const int32_t* lb_end = p->len_buckets + p->n_len_buckets;
        for (int i = 0; i < n_req; ++i) {
            if (new_len[i] <= p->short_max_len) {
                const int j = (int)(std::lower_bound(p->len_buckets, lb_end, new_len[i]) - p->len_buckets);
                pl->req_bucket[i] = j;
                per_bucket[j].push_back(i);
            } else {
                pl->req_class[i] = 1;
            }
        }
        pl->batch_req_offset.push_back(0);
        auto emit = [&](int32_t lb, int32_t depth, int32_t ok, const int32_t* ids, int32_t n_real) {
            const int32_t b = (int32_t)pl->batch_len_bucket.size();
            pl->batch_len_bucket.push_back(lb);
            pl->batch_depth.push_back(depth);
            pl->batch_graph_ok.push_back(ok);
            for (int r = 0; r < n_real; ++r) {
                pl->batch_req_ids.push_back(ids[r]);
                pl->req_batch[ids[r]] = b;
                pl->req_row[ids[r]] = r;
            }
            pl->batch_req_offset.push_back((int32_t)pl->batch_req_ids.size());
        };
        for (int j = 0; j < p->n_len_buckets; ++j) {
            const std::vector<int32_t>& reqs = per_bucket[j];
            if (reqs.empty()) continue;
            const int32_t lb = p->len_buckets[j];
            std::vector<int32_t> allowed;
            for (int d = 0; d < p->n_depths; ++d)
                if ((int64_t)p->depths[d] * lb <= p->token_budget) allowed.push_back(p->depths[d]);
            if (!allowed.empty()) {
                size_t o = 0;
                for (int32_t d : cover_with_depths((int64_t)reqs.size(), allowed)) {
                    const int32_t n_real = (int32_t)std::min<size_t>(d, reqs.size() - o);
                    emit(lb, d, 1, reqs.data() + o, n_real);
                    o += n_real;
                }
            } else {
                // un-captured path: fill in arrival order until the un-padded token total would pass the budget
                size_t o = 0;
                while (o < reqs.size()) {
                    int64_t tot = new_len[reqs[o]];
                    size_t e = o + 1;
                    while (e < reqs.size() && tot + new_len[reqs[e]] <= p->token_budget) tot += new_len[reqs[e++]];
                    emit(lb, (int32_t)(e - o), 0, reqs.data() + o, (int32_t)(e - o));
                    o = e;
                }
            }
        }
        pl->long_chunk_offset.push_back(0);
        for (int i = 0; i < n_req; ++i) {
            if (!pl->req_class[i]) continue;
            pl->long_req.push_back(i);
            int32_t left = new_len[i];
            while (left > 0) {
                const int32_t c = std::min(left, p->long_chunk);
                pl->long_chunk_len.push_back(c);
                left -= c;
            }
            pl->long_chunk_offset.push_back((int32_t)pl->long_chunk_len.size());
        }
    } catch (const std::bad_alloc&) {
        delete pl;
        laps_set_error("plan: out of host memory");
        return LAPS_ENOMEM;
    }
    *out = pl;
    return LAPS_OK;
}

extern "C" void laps_plan_free(laps_plan* plan) { delete plan; }
extern "C" int32_t laps_plan_n_requests(const laps_plan* p) { return p ? (int32_t)p->req_class.size() : 0; }
extern "C" const int32_t* laps_plan_req_class(const laps_plan* p) { return p ? p->req_class.data() : nullptr; }
extern "C" const int32_t* laps_plan_req_bucket(const laps_plan* p) { return p ? p->req_bucket.data() : nullptr; }
extern "C" const int32_t* laps_plan_req_batch(const laps_plan* p) { return p ? p->req_batch.data() : nullptr; }
extern "C" const int32_t* laps_plan_req_row(const laps_plan* p) { return p ? p->req_row.data() : nullptr; }
extern "C" int32_t laps_plan_n_batches(const laps_plan* p) { return p ? (int32_t)p->batch_len_bucket.size() : 0; }
extern "C" const int32_t* laps_plan_batch_len_bucket(const laps_plan* p) { return p ? p->batch_len_bucket.data() : nullptr; }
extern "C" const int32_t* laps_plan_batch_depth(const laps_plan* p) { return p ? p->batch_depth.data() : nullptr; }
extern "C" const int32_t* laps_plan_batch_graph_ok(const laps_plan* p) { return p ? p->batch_graph_ok.data() : nullptr; }
extern "C" const int32_t* laps_plan_batch_req_offset(const laps_plan* p) { return p ? p->batch_req_offset.data() : nullptr; }
extern "C" const int32_t* laps_plan_batch_req_ids(const laps_plan* p) { return p ? p->batch_req_ids.data() : nullptr; }
extern "C" int32_t laps_plan_n_long(const laps_plan* p) { return p ? (int32_t)p->long_req.size() : 0; }
extern "C" const int32_t* laps_plan_long_req(const laps_plan* p) { return p ? p->long_req.data() : nullptr; }
extern "C" const int32_t* laps_plan_long_chunk_offset(const laps_plan* p) { return p ? p->long_chunk_offset.data() : nullptr; }
extern "C" const int32_t* laps_plan_long_chunk_len(const laps_plan* p) { return p ? p->long_chunk_len.data() : nullptr; }
