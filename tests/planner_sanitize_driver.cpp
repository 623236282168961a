// Host-only driver for the integer planner under AddressSanitizer / UBSan (built and run by
// tests/test_planner_host.py).  Feeds seeded random request lists and grids, checks structural
// invariants, and exercises every error path.
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../include/laps.h"

void laps_set_error(const char* fmt, ...) { (void)fmt; }

#define CHECK(c) do { if (!(c)) { printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

int main() {
    std::mt19937 rng(11589);
    for (int it = 0; it < 3000; ++it) {
        std::vector<int32_t> lb, dp;
        int v = 0;
        for (int i = 0, n = 1 + rng() % 4; i < n; ++i) lb.push_back(v += 1 + rng() % 40);
        v = 0;
        for (int i = 0, n = 1 + rng() % 6; i < n; ++i) dp.push_back(v += 1 + rng() % 9);
        laps_plan_params p{(int32_t)(1 + rng() % lb.back()), (int32_t)lb.size(), lb.data(), (int32_t)dp.size(), dp.data(),
                           (int32_t)(1 + rng() % 600), (int32_t)(1 + rng() % 300)};
        const int n = rng() % 200;
        std::vector<int32_t> nl(n), pl(n);
        for (int i = 0; i < n; ++i) { nl[i] = 1 + rng() % 400; pl[i] = rng() % 5000; }
        laps_plan* plan = nullptr;
        CHECK(laps_plan_buckets(&p, n, nl.data(), pl.data(), &plan) == LAPS_OK);
        CHECK(laps_plan_n_requests(plan) == n);
        std::vector<int> seen(n, 0);
        const int nb = laps_plan_n_batches(plan);
        const int32_t* off = laps_plan_batch_req_offset(plan);
        const int32_t* ids = laps_plan_batch_req_ids(plan);
        for (int b = 0; b < nb; ++b) {
            const int lbk = laps_plan_batch_len_bucket(plan)[b], d = laps_plan_batch_depth(plan)[b];
            CHECK(off[b + 1] - off[b] >= 1 && off[b + 1] - off[b] <= d);
            if (laps_plan_batch_graph_ok(plan)[b]) CHECK((int64_t)lbk * d <= p.token_budget);
            for (int j = off[b]; j < off[b + 1]; ++j) { CHECK(nl[ids[j]] <= lbk); seen[ids[j]]++; CHECK(laps_plan_req_batch(plan)[ids[j]] == b); }
        }
        const int nlg = laps_plan_n_long(plan);
        for (int i = 0; i < nlg; ++i) {
            const int r = laps_plan_long_req(plan)[i];
            seen[r]++;
            int64_t tot = 0;
            for (int j = laps_plan_long_chunk_offset(plan)[i]; j < laps_plan_long_chunk_offset(plan)[i + 1]; ++j) tot += laps_plan_long_chunk_len(plan)[j];
            CHECK(tot == nl[r]);
        }
        for (int i = 0; i < n; ++i) CHECK(seen[i] == 1);
        laps_plan_free(plan);
    }
    // error paths
    int32_t one = 1, lbs[2] = {16, 8};
    laps_plan* plan = nullptr;
    laps_plan_params bad{8, 2, lbs, 1, &one, 64, 64};
    CHECK(laps_plan_buckets(&bad, 0, nullptr, nullptr, &plan) == LAPS_EINVAL);
    CHECK(laps_plan_buckets(nullptr, 0, nullptr, nullptr, &plan) == LAPS_EINVAL);
    laps_plan_free(nullptr);
    printf("OK\n");
    return 0;
}
