// Compute / memory latency model of (re-)prefill and its boundary lengths (host only, double).
//
// Section 2.1 of the paper: T_comp(L,H) = alpha*L*(L+2H) + beta*L, T_mem(L,H) = gamma_w*L + gamma_r*H for
// L new and H historical tokens; the boundary L_m is where the two are equal (closed forms for H = 0
// and H > 0); the four coefficients are fitted at run time from samples (T_comp, T_mem, L, H).
#include <cmath>
#include <cstdint>
#include <new>

#include "../../include/laps.h"

void laps_set_error(const char* fmt, ...);

extern "C" double laps_lm_boundary_prefill(double alpha, double beta, double gamma_w) {
    if (!(alpha > 0.0)) return NAN;
    const double v = (gamma_w - beta) / alpha;
    return v > 0.0 ? v : 0.0;
}

extern "C" double laps_lm_boundary_reprefill(double alpha, double beta, double gamma_w, double gamma_r, double h) {
    if (!(alpha > 0.0) || h < 0.0) return NAN;
    // positive root of alpha L^2 + (2 alpha H + beta - gamma_w) L - gamma_r H = 0
    const double b = 2.0 * alpha * h + beta - gamma_w;
    const double disc = b * b + 4.0 * alpha * gamma_r * h;
    if (disc < 0.0) return 0.0;
    const double root = (-b + std::sqrt(disc)) / (2.0 * alpha);
    return root > 0.0 ? root : 0.0;
}

// The same balance with a constant on the memory side: on this GPU a short batch is bounded by streaming the
// weights once per pass (floor), which the printed T_mem has no term for.  Knee = positive root of
// alpha L^2 + (2 alpha H + beta - gamma_w) L - (floor + gamma_r H) = 0; floor = 0 gives the printed boundary.
extern "C" double laps_lm_knee(double alpha, double beta, double gamma_w, double gamma_r, double floor_t, double h) {
    if (!(alpha > 0.0) || h < 0.0 || floor_t < 0.0 || std::isnan(beta) || std::isnan(gamma_w) || std::isnan(gamma_r) ||
        std::isnan(floor_t))
        return NAN;
    const double b = 2.0 * alpha * h + beta - gamma_w;
    const double c = floor_t + gamma_r * h;
    const double disc = b * b + 4.0 * alpha * c;
    if (disc < 0.0) return 0.0;
    const double root = (-b + std::sqrt(disc)) / (2.0 * alpha);
    return root > 0.0 ? root : 0.0;
}

// Scheduling parameters from a fit.  A batch of up to `knee` padded tokens costs one pass over the weights whatever
// its shape, so (a) a request longer than the knee is not "short", (b) a latency-oriented graph should not hold more
// padded tokens than that, (c) requests of other length buckets may share a graph up to that size.
extern "C" int laps_lm_derive_params(const double* coef, double floor_t, double hist_max, int32_t n_len_buckets,
                                     const int32_t* len_buckets, int32_t n_depths, const int32_t* depths,
                                     laps_lm_params* out) {
    if (!coef || !out || !len_buckets || !depths || n_len_buckets < 1 || n_depths < 1 || hist_max < 0.0) {
        laps_set_error("lm_derive_params: NULL pointer, empty grid or negative history length");
        return LAPS_EINVAL;
    }
    for (int i = 0; i < n_len_buckets; ++i)
        if (len_buckets[i] < 1 || (i > 0 && len_buckets[i] <= len_buckets[i - 1])) {
            laps_set_error("lm_derive_params: length buckets must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    for (int i = 0; i < n_depths; ++i)
        if (depths[i] < 1 || (i > 0 && depths[i] <= depths[i - 1])) {
            laps_set_error("lm_derive_params: depths must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    const double k0 = laps_lm_knee(coef[0], coef[1], coef[2], coef[3], floor_t, 0.0);
    const double kh = laps_lm_knee(coef[0], coef[1], coef[2], coef[3], floor_t, hist_max);
    if (std::isnan(k0) || std::isnan(kh)) {
        laps_set_error("lm_derive_params: the fit has no knee (alpha must be positive, the floor non-negative)");
        return LAPS_EINVAL;
    }
    const double knee = k0 < kh ? k0 : kh;
    int32_t sml = len_buckets[0];                       // never below the smallest bucket
    for (int i = 0; i < n_len_buckets; ++i)
        if ((double)len_buckets[i] <= knee) sml = len_buckets[i];
    // largest captured shape (padded tokens) within the knee, but at least one request of the longest short bucket
    int64_t budget = (int64_t)sml * depths[0];
    for (int i = 0; i < n_len_buckets && len_buckets[i] <= sml; ++i)
        for (int j = 0; j < n_depths; ++j) {
            const int64_t t = (int64_t)len_buckets[i] * depths[j];
            if ((double)t <= knee && t > budget) budget = t;
        }
    out->knee_fresh = k0;
    out->knee_hist = kh;
    out->short_max_len = sml;
    out->short_token_budget = (int32_t)budget;
    out->fuse_budget = (int32_t)budget;
    return LAPS_OK;
}

// Two independent two-parameter least-squares problems through the origin (normal equations):
//   t_comp ~ alpha * L(L+2H) + beta * L        t_mem ~ gamma_w * L + gamma_r * H
static int fit2(int n, const double* x1, const double* x2, const double* y, double* c1, double* c2) {
    double a11 = 0, a12 = 0, a22 = 0, b1 = 0, b2 = 0;
    for (int i = 0; i < n; ++i) {
        a11 += x1[i] * x1[i];
        a12 += x1[i] * x2[i];
        a22 += x2[i] * x2[i];
        b1 += x1[i] * y[i];
        b2 += x2[i] * y[i];
    }
    const double det = a11 * a22 - a12 * a12;
    if (!(std::fabs(det) > 1e-12 * (a11 * a22 + 1e-300))) return 0;
    *c1 = (b1 * a22 - b2 * a12) / det;
    *c2 = (a11 * b2 - a12 * b1) / det;
    return 1;
}

extern "C" int laps_lm_fit(int32_t n, const double* new_len, const double* hist_len, const double* t_comp,
                           const double* t_mem, double* coef_out) {
    if (n < 2 || !new_len || !hist_len || (!t_comp && !t_mem) || !coef_out) {
        laps_set_error("lm_fit: need at least 2 samples, L, H, one of the two time arrays and an output");
        return LAPS_EINVAL;
    }
    int ok1 = 1, ok2 = 1;
    if (t_comp) {
        double* q = new (std::nothrow) double[(size_t)n];
        if (!q) {
            laps_set_error("lm_fit: out of host memory");
            return LAPS_ENOMEM;
        }
        for (int i = 0; i < n; ++i) q[i] = new_len[i] * (new_len[i] + 2.0 * hist_len[i]);
        ok1 = fit2(n, q, new_len, t_comp, &coef_out[0], &coef_out[1]);
        delete[] q;
    }
    if (t_mem) ok2 = fit2(n, new_len, hist_len, t_mem, &coef_out[2], &coef_out[3]);
    if (!ok1 || !ok2) {
        laps_set_error("lm_fit: samples do not determine the coefficients (vary L and H independently)");
        return LAPS_EINVAL;
    }
    return LAPS_OK;
}
