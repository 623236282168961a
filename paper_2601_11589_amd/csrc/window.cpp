// Fixed-window dispatch of the short queue on one GPU (host only).
//
// Section 3.2 of the paper keeps a short and a long queue and lets an instance run one class at a time; Section 3.1
// batches short requests into captured (length, depth) shapes after a waiting window and mentions fusing graphs.
// Read for one GPU: at every decision instant the waiting short requests leave together when the oldest has waited
// the window, when their padded tokens fill the graph budget, or when nothing else could use the GPU; otherwise a
// long chunk runs.  When so few padded tokens wait that one replay costs one pass over the weights whatever its
// shape, all of them share the largest length bucket any of them needs (one replay instead of one per bucket).
#include <cmath>
#include <cstdint>

#include "../../include/laps.h"

void laps_set_error(const char* fmt, ...);

extern "C" int laps_window_poll(const laps_window_params* p, double now_us, int32_t n_waiting, const double* arrival_us,
                                const int32_t* new_len, int32_t nothing_else, int32_t* action, int32_t* fused_len_bucket,
                                int64_t* padded_tokens, double* wake_us) {
    if (!p || !action || !fused_len_bucket || !padded_tokens || !wake_us || n_waiting < 0 ||
        (n_waiting > 0 && (!arrival_us || !new_len))) {
        laps_set_error("window_poll: NULL pointer or negative count");
        return LAPS_EINVAL;
    }
    if (p->n_len_buckets < 1 || !p->len_buckets || std::isnan(p->window_us) || p->window_us < 0.0 || std::isnan(now_us) ||
        p->token_budget < 1 || p->merge_below < 0) {
        laps_set_error("window_poll: bad parameters (empty grid, negative window, budget < 1 or NaN time)");
        return LAPS_EINVAL;
    }
    for (int i = 0; i < p->n_len_buckets; ++i)
        if (p->len_buckets[i] < 1 || (i > 0 && p->len_buckets[i] <= p->len_buckets[i - 1])) {
            laps_set_error("window_poll: length buckets must be positive and strictly ascending");
            return LAPS_EINVAL;
        }
    int64_t total = 0;
    int32_t widest = 0;
    for (int i = 0; i < n_waiting; ++i) {
        if (new_len[i] < 1 || new_len[i] > p->len_buckets[p->n_len_buckets - 1] || std::isnan(arrival_us[i]) ||
            arrival_us[i] > now_us || (i > 0 && arrival_us[i] < arrival_us[i - 1])) {
            laps_set_error("window_poll: request %d: length outside the grid, or arrivals unordered / after now", i);
            return LAPS_EINVAL;
        }
        int32_t need = 0;
        for (int j = 0; j < p->n_len_buckets; ++j)
            if (p->len_buckets[j] >= new_len[i]) {
                need = p->len_buckets[j];
                break;
            }
        total += need;
        widest = need > widest ? need : widest;
    }
    *padded_tokens = total;
    *fused_len_bucket = 0;
    *wake_us = INFINITY;
    *action = LAPS_AWD_WAIT;
    if (n_waiting == 0) return LAPS_OK;
    const bool due = (now_us - arrival_us[0] >= p->window_us) || total >= p->token_budget || nothing_else != 0;
    if (due) {
        *action = LAPS_AWD_DISPATCH;
        if (total < p->merge_below) *fused_len_bucket = widest;
    } else {
        *wake_us = arrival_us[0] + p->window_us;
    }
    return LAPS_OK;
}
