// Host-only driver for the AWD state machine, the pool controller and the latency-model helpers under
// AddressSanitizer / UBSan (built and run by tests/test_planner_host.py).  Seeded random event loops, structural
// invariants, every error path.
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <limits>
#include <random>
#include <vector>

#include "../include/laps.h"

void laps_set_error(const char* fmt, ...) { (void)fmt; }

#define CHECK(c) do { if (!(c)) { printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

static int awd_run(std::mt19937& rng) {
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<int32_t> lb{16, 32, 64}, dp{1, 2, 4, 8, 16};
    if (rng() % 2) lb = {8, 24};
    laps_awd_params p{(int32_t)lb.size(), lb.data(), (int32_t)dp.size(), dp.data(), (int64_t)(lb.back() * (1 + rng() % 20)),
                      (rng() % 3) ? -1 : (int64_t)(rng() % 200), (double)(rng() % 30), 0.0, 50.0 + rng() % 500, 40.0,
                      (rng() % 2) ? inf : 300.0, (double)(rng() % 10), 1e-9, (int32_t)(rng() % 2), (int32_t)(rng() % 2)};
    laps_awd* a = nullptr;
    CHECK(laps_awd_create(&p, (rng() % 2) ? inf : 100.0, &a) == LAPS_OK);
    if (rng() % 2) {
        std::vector<double> tab(lb.size() * dp.size());
        for (auto& v : tab) v = (rng() % 4) ? 30.0 + rng() % 40 : std::nan("");
        CHECK(laps_awd_set_service_table(a, tab.data()) == LAPS_OK);
    }
    const int n = 1 + rng() % 150;
    std::vector<double> arr(n), ddl(n);
    std::vector<int32_t> len(n);
    double t = 0;
    for (int i = 0; i < n; ++i) {
        t += (double)(rng() % 60);
        arr[i] = t;
        ddl[i] = (rng() % 3) ? t + 100 + rng() % 2000 : inf;
        len[i] = 1 + rng() % lb.back();
    }
    std::vector<char> done(n, 0);
    int left = n, guard = 0;
    double now = 0;
    CHECK(laps_awd_begin_round(a, 0.0) == LAPS_OK);
    while (left > 0) {
        CHECK(++guard < 100000);
        std::vector<double> qa, qd;
        std::vector<int32_t> ql, qi;
        for (int i = 0; i < n; ++i)
            if (!done[i] && arr[i] <= now) { qa.push_back(arr[i]); qd.push_back(ddl[i]); ql.push_back(len[i]); qi.push_back(i); }
        std::vector<int32_t> take(qa.size() + 1);
        int32_t action, n_take, lbk, depth, reason;
        double wake;
        CHECK(laps_awd_poll(a, now, 0.01, (int32_t)qa.size(), qa.data(), qd.data(), ql.data(), &action, &n_take, take.data(),
                            &lbk, &depth, &reason, &wake) == LAPS_OK);
        if (action == LAPS_AWD_DISPATCH) {
            CHECK(n_take >= 1 && n_take <= depth && (int64_t)lbk * depth <= p.mem_budget && reason != LAPS_AWD_NONE);
            for (int j = 0; j < n_take; ++j) {
                CHECK(take[j] >= 0 && take[j] < (int32_t)qa.size() && !done[qi[take[j]]] && ql[take[j]] <= lbk);
                done[qi[take[j]]] = 1;
                --left;
            }
            CHECK(laps_awd_window_us(a) >= p.w_min_us && laps_awd_window_us(a) <= p.w_max_us && laps_awd_target_depth(a) >= 1);
            now += 35.0;
            CHECK(laps_awd_begin_round(a, now) == LAPS_OK);
            continue;
        }
        double next = wake;
        for (int i = 0; i < n; ++i)
            if (!done[i] && arr[i] > now && arr[i] < next) next = arr[i];
        CHECK(std::isfinite(next) && next > now);
        now = next;
    }
    // error paths
    int32_t action, n_take, lbk, depth, reason, one_len = 5, idx;
    double wake, a0 = now + 10, d0 = inf;
    CHECK(laps_awd_poll(a, now, 0.0, 1, &a0, &d0, &one_len, &action, &n_take, &idx, &lbk, &depth, &reason, &wake) == LAPS_EINVAL);
    one_len = lb.back() + 1;
    a0 = now;
    CHECK(laps_awd_poll(a, now, 0.0, 1, &a0, &d0, &one_len, &action, &n_take, &idx, &lbk, &depth, &reason, &wake) == LAPS_EINVAL);
    CHECK(laps_awd_poll(nullptr, now, 0.0, 0, nullptr, nullptr, nullptr, &action, &n_take, &idx, &lbk, &depth, &reason, &wake) == LAPS_EINVAL);
    laps_awd_destroy(a);
    return 0;
}

static int ctrl_run(std::mt19937& rng) {
    const int N = 1 + rng() % 12, n_min = rng() % 2;
    int ns = rng() % (N + 1);
    laps_ctrl_params p{N, n_min, (double)(rng() % 5), 0.1 * (rng() % 10), 1.0, 2.0, 0.5, 0.9,
                       (rng() % 2) ? -std::numeric_limits<double>::infinity() : 1.0};
    laps_ctrl* c = nullptr;
    CHECK(laps_ctrl_create(&p, ns, &c) == LAPS_OK);
    for (int step = 0; step < 300; ++step) {
        ns = laps_ctrl_n_short(c);
        const int nl = N - ns;
        std::vector<double> q(N), e(N), u(N);
        for (int i = 0; i < N; ++i) { q[i] = rng() % 20; e[i] = (rng() % 10) / 10.0; u[i] = (rng() % 11) / 10.0; }
        int32_t action;
        double ps, pl;
        CHECK(laps_ctrl_step(c, (double)step, ns, q.data(), e.data(), u.data(), nl, q.data() + ns, e.data() + ns, u.data() + ns,
                             &action, &ps, &pl) == LAPS_OK);
        CHECK(action >= -1 && action <= 1 && laps_ctrl_n_short(c) == ns + action);
        CHECK(laps_ctrl_n_short(c) >= 0 && laps_ctrl_n_short(c) <= N);
        if (action == 1) CHECK(nl > n_min);
        if (action == -1) CHECK(ns > n_min);
    }
    int32_t action;
    double ps, pl, z = 0;
    CHECK(laps_ctrl_step(c, 0.0, laps_ctrl_n_short(c) + 1, &z, &z, &z, 0, nullptr, nullptr, nullptr, &action, &ps, &pl) == LAPS_EINVAL);
    laps_ctrl_destroy(c);
    return 0;
}

int main() {
    std::mt19937 rng(115890);
    for (int it = 0; it < 300; ++it)
        if (awd_run(rng)) return 1;
    for (int it = 0; it < 200; ++it)
        if (ctrl_run(rng)) return 1;
    // latency model
    CHECK(laps_lm_boundary_prefill(1.0, 2.0, 10.0) == 8.0 && laps_lm_boundary_prefill(1.0, 12.0, 10.0) == 0.0);
    CHECK(std::isnan(laps_lm_boundary_prefill(0.0, 1.0, 1.0)) && std::isnan(laps_lm_boundary_reprefill(1, 1, 1, 1, -2)));
    CHECK(std::fabs(laps_lm_boundary_reprefill(1.0, 2.0, 10.0, 3.0, 4.0) - std::sqrt(12.0)) < 1e-12);
    std::vector<double> L, H, tc, tm;
    for (int i = 0; i < 50; ++i) {
        L.push_back(1 + rng() % 500);
        H.push_back(rng() % 4000);
        tc.push_back(2e-3 * L[i] * (L[i] + 2 * H[i]) + 0.5 * L[i]);
        tm.push_back(1.5 * L[i] + 0.25 * H[i]);
    }
    double coef[4];
    CHECK(laps_lm_fit(50, L.data(), H.data(), tc.data(), tm.data(), coef) == LAPS_OK);
    CHECK(std::fabs(coef[0] - 2e-3) < 1e-9 && std::fabs(coef[1] - 0.5) < 1e-6 && std::fabs(coef[2] - 1.5) < 1e-9 &&
          std::fabs(coef[3] - 0.25) < 1e-9);
    CHECK(laps_lm_fit(1, L.data(), H.data(), tc.data(), tm.data(), coef) == LAPS_EINVAL);
    CHECK(laps_lm_fit(50, L.data(), L.data(), tc.data(), tm.data(), coef) == LAPS_EINVAL);
    // knee with a weight-streaming floor and the parameters derived from a fit
    CHECK(std::fabs(laps_lm_knee(1.0, 2.0, 10.0, 3.0, 9.0, 4.0) - std::sqrt(21.0)) < 1e-12);
    CHECK(std::isnan(laps_lm_knee(0.0, 1.0, 1.0, 1.0, 1.0, 0.0)));
    {
        const int32_t lb[3] = {16, 32, 64}, dp[7] = {1, 2, 4, 8, 16, 32, 64};
        const double c1[4] = {1.0, 0.0, 0.0, 0.0};
        laps_lm_params prm;
        CHECK(laps_lm_derive_params(c1, 200.0 * 200.0, 0.0, 3, lb, 7, dp, &prm) == LAPS_OK);
        CHECK(prm.short_max_len == 64 && prm.short_token_budget == 128 && prm.fuse_budget == 128);
        CHECK(laps_lm_derive_params(c1, 10.0 * 10.0, 0.0, 3, lb, 7, dp, &prm) == LAPS_OK && prm.short_max_len == 16);
        CHECK(laps_lm_derive_params(c1, 1.0, -1.0, 3, lb, 7, dp, &prm) == LAPS_EINVAL);
        CHECK(laps_lm_derive_params(c1, 1.0, 0.0, 0, lb, 7, dp, &prm) == LAPS_EINVAL);
    }
    // fixed-window dispatch over random queues: every output is written, grids and lengths are only read in range
    for (int it = 0; it < 2000; ++it) {
        const int32_t lb[3] = {16, 32, 64};
        const int n = (int)(rng() % 40);
        std::vector<double> arr(n);
        std::vector<int32_t> nl(n);
        double t = 0;
        for (int i = 0; i < n; ++i) {
            t += (double)(rng() % 300);
            arr[i] = t;
            nl[i] = 1 + (int32_t)(rng() % 64);
        }
        laps_window_params wp = {3, lb, (double)(rng() % 2000), (int64_t)(1 + rng() % 2048), (int64_t)(rng() % 300)};
        int32_t action = -1, fused = -1;
        int64_t padded = -1;
        double wake = -1;
        CHECK(laps_window_poll(&wp, t + (double)(rng() % 500), n, arr.data(), nl.data(), (int32_t)(rng() % 2), &action, &fused,
                               &padded, &wake) == LAPS_OK);
        CHECK((action == LAPS_AWD_WAIT || action == LAPS_AWD_DISPATCH) && padded >= 16 * n && padded <= 64 * n);
        CHECK(fused == 0 || fused == 16 || fused == 32 || fused == 64);
        if (n == 0) CHECK(action == LAPS_AWD_WAIT && std::isinf(wake));
        if (n > 0) {
            nl[n - 1] = 65;
            CHECK(laps_window_poll(&wp, t, n, arr.data(), nl.data(), 0, &action, &fused, &padded, &wake) == LAPS_EINVAL);
        }
    }
    printf("OK\n");
    return 0;
}
