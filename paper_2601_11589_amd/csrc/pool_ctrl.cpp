// Instance-pressure controller of spatial disaggregation: host-only decision state (laps_ctrl_* in include/laps.h).
//
// Algorithm 2 of the paper: per control period every instance reports backlog q, SLA deviation e and utilisation u;
// psi = alpha q + beta e - gamma u; pool pressure = a robust aggregate (P90) of its instances' psi; outside the
// cool-down, one instance moves towards the pool whose pressure exceeds the other's by the hysteresis factor
// (1 + tau), never leaving a pool below its minimum allocation.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "../../include/laps.h"

void laps_set_error(const char* fmt, ...);

struct laps_ctrl {
    laps_ctrl_params p;
    int32_t n_short, n_long;
    double t_last;
    std::vector<double> scratch;
};

namespace {
// nearest-rank quantile: the smallest member with at least q of the set at or below it; 0 for an empty set
double pool_pressure(laps_ctrl* c, int32_t n, const double* q, const double* e, const double* u) {
    if (n == 0) return 0.0;
    c->scratch.resize((size_t)n);
    for (int32_t k = 0; k < n; ++k) c->scratch[(size_t)k] = c->p.w_q * q[k] + c->p.w_e * e[k] - c->p.w_u * u[k];
    std::sort(c->scratch.begin(), c->scratch.end());
    int64_t rank = (int64_t)std::ceil(c->p.quantile * n);
    rank = rank < 1 ? 1 : (rank > n ? n : rank);
    return c->scratch[(size_t)(rank - 1)];
}
}  // namespace

extern "C" int laps_ctrl_create(const laps_ctrl_params* p, int32_t n_short, laps_ctrl** out) {
    if (!p || !out || p->n_total < 1 || n_short < 0 || n_short > p->n_total || p->n_min < 0 || !(p->cool_us >= 0.0) ||
        !(p->tau >= 0.0) || !(p->quantile > 0.0 && p->quantile <= 1.0) || std::isnan(p->w_q) || std::isnan(p->w_e) ||
        std::isnan(p->w_u) || std::isnan(p->min_pressure)) {
        laps_set_error("ctrl: need n_total >= 1, 0 <= n_short <= n_total, n_min >= 0, cool >= 0, tau >= 0, 0 < quantile <= 1");
        return LAPS_EINVAL;
    }
    laps_ctrl* c = new (std::nothrow) laps_ctrl();
    if (!c) {
        laps_set_error("ctrl: out of host memory");
        return LAPS_ENOMEM;
    }
    c->p = *p;
    c->n_short = n_short;
    c->n_long = p->n_total - n_short;
    c->t_last = -std::numeric_limits<double>::infinity();
    *out = c;
    return LAPS_OK;
}

extern "C" void laps_ctrl_destroy(laps_ctrl* c) { delete c; }

extern "C" int32_t laps_ctrl_n_short(const laps_ctrl* c) { return c ? c->n_short : -1; }

extern "C" int laps_ctrl_step(laps_ctrl* c, double now_us, int32_t n_short, const double* q_s, const double* e_s,
                              const double* u_s, int32_t n_long, const double* q_l, const double* e_l, const double* u_l,
                              int32_t* action, double* p_short, double* p_long) {
    if (!c || !action || !p_short || !p_long || std::isnan(now_us) || (n_short > 0 && (!q_s || !e_s || !u_s)) ||
        (n_long > 0 && (!q_l || !e_l || !u_l))) {
        laps_set_error("ctrl_step: NULL argument or NaN time");
        return LAPS_EINVAL;
    }
    if (n_short != c->n_short || n_long != c->n_long) {
        laps_set_error("ctrl_step: got signals of %d short / %d long instances, the pools hold %d / %d", n_short, n_long,
                       c->n_short, c->n_long);
        return LAPS_EINVAL;
    }
    for (int32_t k = 0; k < n_short; ++k)
        if (std::isnan(q_s[k]) || std::isnan(e_s[k]) || std::isnan(u_s[k])) {
            laps_set_error("ctrl_step: NaN signal of short instance %d", k);
            return LAPS_EINVAL;
        }
    for (int32_t k = 0; k < n_long; ++k)
        if (std::isnan(q_l[k]) || std::isnan(e_l[k]) || std::isnan(u_l[k])) {
            laps_set_error("ctrl_step: NaN signal of long instance %d", k);
            return LAPS_EINVAL;
        }
    const double ps = pool_pressure(c, n_short, q_s, e_s, u_s);
    const double pl = pool_pressure(c, n_long, q_l, e_l, u_l);
    *p_short = ps;
    *p_long = pl;
    *action = 0;
    if (now_us - c->t_last < c->p.cool_us) return LAPS_OK;
    if (ps > (1.0 + c->p.tau) * pl && ps > c->p.min_pressure && c->n_long > c->p.n_min) {
        ++c->n_short;
        --c->n_long;
        c->t_last = now_us;
        *action = 1;
    } else if (pl > (1.0 + c->p.tau) * ps && pl > c->p.min_pressure && c->n_short > c->p.n_min) {
        ++c->n_long;
        --c->n_short;
        c->t_last = now_us;
        *action = -1;
    }
    return LAPS_OK;
}
