"""Oracle for Adaptive-Wait-Depth batching of the short queue on a virtual clock.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

What the paper fixes (Algorithm 1; Section 3.1 "Graph-aware memory-based batching"; Section 3.2,
SLA-constrained and deadline-free modes):
  * two thresholds: a waiting window W and a target depth D.  W starts as
    clip(min_i(DDL_i - t - S_hat), [W_min, W_max]), D as the largest depth of a captured shape whose
    memory is within the budget M;
  * a round starts a timer and an empty batch B and adds short requests while elapsed < W and
    depth(B) < D; it stops early when the smallest slack DDL_i - (t + S_hat) over B and the next request
    is <= sigma (and, Section 3.2, when the head of the line has waited T_max);
  * requests are added bucket-first and only if the batch still fits the memory budget;
  * B is padded to NearestGraph(B, H, M): the closest captured shape with depth >= depth(B), mem <= M;
  * after dispatch, with d = depth(B) and tau the time it took to collect B: d >= D sets
    W <- clip(tau, [W_min, W_max]), otherwise D <- d;
  * SLA-constrained mode (Section 3.2a) takes, at the start of a decision epoch,
    W = clip(min(W_SLA, W_GR), [W_min, W_max]) with W_SLA = max(0, min_{i in Q_s}(DDL_i - t - S_hat) - delta)
    and W_GR = max(0, D - depth(B)) / max(r_hat, eps).
Readings taken where the paper is silent:
  * one request's memory is its padded length bucket; mem(G) = L_b(G) * depth(G) padded tokens;
  * the timer of a round starts when the instance is free AND a short request is waiting;
  * "bucket-first": among waiting requests (arrival order), those in the length bucket of the oldest one
    are taken first, then the others; a request that would push mem(NearestGraph) above M is skipped and
    stays queued;  the batch is re-formed from the waiting queue at every decision instant;
  * a batch of mixed buckets runs in the shape of its largest bucket; requests of another bucket than the
    oldest one's join only while the fused shape stays within `fuse_budget` padded tokens (the "graph fusion"
    of Section 3.1 pays only while a step costs one pass over the weights whatever its shape);
  * r_hat is supplied by the caller (requests per microsecond) for the epoch; S_hat is one number, or a table
    per captured shape supplied by the caller (the entry of the shape the current batch would run in);
  * optional growth of D (off in the printed algorithm, where D can only fall): when a round fills its
    target while at least as many requests again are still waiting, D moves to the next larger captured depth
    within the budget.
Times are in microseconds (float), decisions happen at event times only (arrival, timer expiry, slack
trigger, head-of-line cap, instance free).

Pins (tests/test_awd.py): hand-worked traces under tests/golden/awd_cases.json, the deadline-free /
all-arrived case reducing to token-max fills, and invariants (every request once, memory within M,
no dispatch later than the window allows, W within its bounds, D never above its start value).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

INF = math.inf


@dataclass
class AwdParams:
    len_buckets: tuple
    depths: tuple
    mem_budget: int                 # M, padded tokens
    sigma: float = 0.0              # slack trigger
    w_min: float = 0.0
    w_max: float = 10_000.0
    s_hat: float = 1_000.0          # service-time estimate of one short step
    t_max: float = INF              # head-of-line cap
    delta: float = 0.0              # safety margin of the SLA window
    sla_window: bool = False        # Section 3.2a window instead of the adapted W
    rate_eps: float = 1e-9
    d_regrow: bool = False
    fuse_budget: int = -1           # padded tokens up to which other length buckets may join (-1: mem_budget)


def clip(v, lo, hi):
    return min(max(v, lo), hi)


def bucket_of(p: AwdParams, n: int) -> int:
    return min(b for b in p.len_buckets if b >= n)


def nearest_graph(p: AwdParams, len_bucket: int, depth: int, budget=None):
    """Closest captured shape for a batch of `depth` rows of `len_bucket`: smallest captured depth >= depth
    whose padded tokens fit the budget (M unless given), or None."""
    budget = p.mem_budget if budget is None else budget
    ok = [d for d in p.depths if d >= depth and d * len_bucket <= budget]
    return (len_bucket, min(ok)) if ok else None


def initial_depth(p: AwdParams) -> int:
    return max(d for d in p.depths for b in p.len_buckets if d * b <= p.mem_budget)


def form_batch(p: AwdParams, waiting, new_len, target_depth):
    """waiting: request ids in arrival order.  Returns (batch ids, next id or None)."""
    if not waiting:
        return [], None
    head_bucket = bucket_of(p, new_len[waiting[0]])
    order = [r for r in waiting if bucket_of(p, new_len[r]) == head_bucket] + \
            [r for r in waiting if bucket_of(p, new_len[r]) != head_bucket]
    batch, cur_len = [], 0
    nxt = None
    for r in order:
        if len(batch) >= target_depth:
            nxt = r
            break
        lb = max(cur_len, bucket_of(p, new_len[r]))
        budget = p.mem_budget
        if bucket_of(p, new_len[r]) != head_bucket and p.fuse_budget >= 0:
            budget = min(budget, p.fuse_budget)         # another bucket joins only while padding stays cheap
        if nearest_graph(p, lb, len(batch) + 1, budget) is None:
            continue
        batch.append(r)
        cur_len = lb
    return batch, nxt


@dataclass
class Dispatch:
    t: float
    req_ids: list
    len_bucket: int
    depth: int
    reason: str
    w_after: float
    d_after: int
    tau: float


def simulate(p: AwdParams, arrival, ddl, new_len, service_us, rate_hat=0.0, t0=0.0, s_hat_table=None):
    """Runs the short queue alone.  service_us(len_bucket, depth) -> duration of one dispatched step.
    s_hat_table: optional {(len_bucket, depth): estimate}; the estimate S_hat used at a decision instant is then
    the entry of the shape the batch formed at that instant would run in (p.s_hat where there is no entry).
    Returns the list of Dispatch records."""
    def s_hat_of(batch):
        if not batch or not s_hat_table:
            return p.s_hat
        g = nearest_graph(p, max(bucket_of(p, new_len[r]) for r in batch), len(batch))
        return s_hat_table.get(g, p.s_hat)

    n = len(arrival)
    order = sorted(range(n), key=lambda i: (arrival[i], i))
    known = [i for i in order if arrival[i] <= t0]
    first_slack = min((ddl[i] - t0 - p.s_hat for i in known), default=INF)
    W = clip(first_slack, p.w_min, p.w_max)
    D = initial_depth(p)
    d_cap = D
    done = [False] * n
    out = []
    free_at = t0
    while not all(done):
        pending = [i for i in order if not done[i]]
        t_start = max(free_at, arrival[pending[0]])           # timer start
        t = t_start
        w_round = W
        if p.sla_window:
            waiting = [i for i in pending if arrival[i] <= t]
            b0, _ = form_batch(p, waiting, new_len, D)
            w_sla = max(0.0, min(ddl[i] - t - s_hat_of(b0) for i in waiting) - p.delta)
            w_gr = max(0, D - len(b0)) / max(rate_hat, p.rate_eps)
            w_round = clip(min(w_sla, w_gr), p.w_min, p.w_max)
        while True:
            waiting = [i for i in pending if arrival[i] <= t]
            batch, nxt = form_batch(p, waiting, new_len, D)
            watch = batch + ([nxt] if nxt is not None else [])
            # the three timed conditions as instants: slack_i <= sigma  <=>  t >= DDL_i - S_hat - sigma, etc.
            t_sla = min((ddl[i] - s_hat_of(batch) - p.sigma for i in watch), default=INF)
            t_cap = arrival[waiting[0]] + p.t_max
            t_win = t_start + w_round
            reason = None
            if len(batch) >= D:
                reason = "depth"
            elif t >= t_sla:
                reason = "sla"
            elif t >= t_cap:
                reason = "tmax"
            elif t >= t_win:
                reason = "window"
            if reason:
                break
            events = [t_sla, t_cap, t_win] + [arrival[i] for i in pending if arrival[i] > t]
            t = min(e for e in events if e > t)
        d, tau = len(batch), t - t_start
        lb = max(bucket_of(p, new_len[r]) for r in batch)
        g = nearest_graph(p, lb, d)
        if d >= D:
            W = clip(tau, p.w_min, p.w_max)
            if p.d_regrow and len(waiting) - d >= d:
                bigger = [x for x in p.depths if x > D and x <= d_cap]
                if bigger:
                    D = min(bigger)
        else:
            D = d
        for r in batch:
            done[r] = True
        out.append(Dispatch(t, list(batch), g[0], g[1], reason, W, D, tau))
        free_at = t + service_us(g[0], g[1])
    return out
