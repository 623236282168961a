"""Adaptive-Wait-Depth batching (Algorithm 1, Section 3.2): the oracle against hand-worked traces and invariants."""
import json
import math
import os

import numpy as np
import pytest

from oracle import awd_oracle as AO

GOLD = os.path.join(os.path.dirname(__file__), "golden", "awd_cases.json")


def load_cases():
    with open(GOLD) as f:
        return json.load(f)["cases"]


def params_of(d):
    d = dict(d)
    d["t_max"] = math.inf if d["t_max"] is None else d["t_max"]
    d["len_buckets"], d["depths"] = tuple(d["len_buckets"]), tuple(d["depths"])
    return AO.AwdParams(**d)


def table_of(case):
    t = case.get("s_hat_table")
    return {(lb, d): v for lb, d, v in t} if t else None


def inf_none(v):
    return [math.inf if x is None else float(x) for x in v]


@pytest.mark.parametrize("case", load_cases(), ids=lambda c: c["name"])
def test_oracle_reproduces_hand_worked_traces(case):
    p = params_of(case["params"])
    got = AO.simulate(p, [float(a) for a in case["arrival"]], inf_none(case["ddl"]), case["new_len"],
                      lambda lb, d: case["service_us"], rate_hat=case["rate_hat"], s_hat_table=table_of(case))
    assert len(got) == len(case["trace"])
    for g, w in zip(got, case["trace"]):
        assert (g.t, g.req_ids, g.len_bucket, g.depth, g.reason, g.w_after, g.d_after, g.tau) == \
               (w["t"], w["req_ids"], w["len_bucket"], w["depth"], w["reason"], w["w_after"], w["d_after"], w["tau"])


def random_workload(rng, n, with_ddl):
    arrival = np.cumsum(rng.exponential(40.0, n))
    new_len = rng.integers(1, 65, n)
    ddl = arrival + rng.uniform(200, 3000, n) if with_ddl else np.full(n, math.inf)
    return list(arrival), list(ddl), [int(x) for x in new_len]


@pytest.mark.parametrize("seed", range(6))
def test_oracle_invariants(seed):
    rng = np.random.default_rng(1000 + seed)
    p = AO.AwdParams(len_buckets=(16, 32, 64), depths=(1, 2, 4, 8, 16), mem_budget=int(rng.choice([64, 256, 1024])),
                     sigma=20.0, w_min=10.0, w_max=500.0, s_hat=100.0, t_max=float(rng.choice([math.inf, 800.0])),
                     sla_window=bool(seed % 2), d_regrow=bool(seed % 3 == 0))
    arrival, ddl, new_len = random_workload(rng, 200, with_ddl=seed >= 2)
    svc = lambda lb, d: 80.0 + 0.05 * lb * d
    tr = AO.simulate(p, arrival, ddl, new_len, svc, rate_hat=1 / 40.0)
    seen = sorted(r for x in tr for r in x.req_ids)
    assert seen == list(range(200))                                   # every request exactly once
    d0 = AO.initial_depth(p)
    free_at, prev_t = 0.0, 0.0
    for x in tr:
        assert x.len_bucket * x.depth <= p.mem_budget and x.depth in p.depths and x.depth >= len(x.req_ids)
        assert x.len_bucket == max(AO.bucket_of(p, new_len[r]) for r in x.req_ids)
        assert all(arrival[r] <= x.t for r in x.req_ids)
        assert x.t >= free_at and x.t >= prev_t                        # one step at a time
        assert p.w_min <= x.w_after <= p.w_max and 1 <= x.d_after <= d0
        assert x.tau <= p.w_max + 1e-9                                 # never waits beyond the window bound
        oldest = min(arrival[r] for r in x.req_ids)
        assert x.t - max(oldest, free_at) <= min(p.w_max, p.t_max) + 1e-9
        free_at, prev_t = x.t + svc(x.len_bucket, x.depth), x.t


def test_oracle_all_arrived_deadline_free_is_token_max():
    """With every request waiting at t = 0 and no deadlines, each round fills the target depth at once:
    floor(n / D) full batches of the largest depth that fits the budget, then the remainder (Section 3.2b)."""
    p = AO.AwdParams(len_buckets=(16,), depths=(1, 2, 4, 8), mem_budget=128, w_min=0.0, w_max=1000.0, s_hat=10.0)
    n = 27
    tr = AO.simulate(p, [0.0] * n, [math.inf] * n, [9] * n, lambda lb, d: 10.0)
    assert [len(x.req_ids) for x in tr[:3]] == [8, 8, 8] and all(x.reason == "depth" and x.tau == 0 for x in tr[:3])
    assert [x.req_ids for x in tr[:3]] == [list(range(0, 8)), list(range(8, 16)), list(range(16, 24))]
    # the last three requests cannot fill D = 8; W has collapsed to the observed fill time 0, so they leave at once
    assert tr[3].req_ids == [24, 25, 26] and tr[3].depth == 4 and tr[3].reason == "window" and tr[3].d_after == 3


# ------------------------------------------------------------------ the library's state machine against the oracle
def drive_library(p: AO.AwdParams, arrival, ddl, new_len, service_us, rate_hat=0.0, t0=0.0, s_hat_table=None):
    """Event loop around laps_awd_poll: polls at arrivals, at the returned wake-up times and when the instance
    becomes free; the same clock rules as the oracle's simulation, none of its code."""
    from paper_2601_11589_amd import api
    n = len(arrival)
    order = sorted(range(n), key=lambda i: (arrival[i], i))
    known = [ddl[i] - t0 - p.s_hat for i in order if arrival[i] <= t0]
    awd = api.LapsAwd(p.len_buckets, p.depths, p.mem_budget, p.sigma, p.w_min, p.w_max, p.s_hat, p.t_max, p.delta,
                      p.rate_eps, p.sla_window, p.d_regrow, first_slack_us=min(known, default=math.inf),
                      fuse_budget=p.fuse_budget)
    if s_hat_table is not None:
        tab = np.full((len(p.len_buckets), len(p.depths)), np.nan)
        for (lb, d), v in s_hat_table.items():
            tab[p.len_buckets.index(lb), p.depths.index(d)] = v
        awd.laps_awd_set_service_table(tab)
    awd.laps_awd_begin_round(t0)
    done, trace, t = set(), [], t0
    while len(done) < n:
        waiting = [i for i in order if i not in done and arrival[i] <= t]
        r = awd.laps_awd_poll(t, [arrival[i] for i in waiting], [ddl[i] for i in waiting], [new_len[i] for i in waiting],
                              rate_hat)
        if r["dispatch"]:
            ids = [waiting[j] for j in r["take"]]
            done.update(ids)
            trace.append((t, ids, r["len_bucket"], r["depth"], r["reason"], awd.window_us, awd.target_depth))
            free = t + service_us(r["len_bucket"], r["depth"])
            awd.laps_awd_begin_round(free)
            future = [arrival[i] for i in order if i not in done and arrival[i] > t]
            pend = [arrival[i] for i in order if i not in done]
            if pend:
                t = max(free, min(pend))
            continue
        future = [arrival[i] for i in order if i not in done and arrival[i] > t]
        t = min([r["wake_us"]] + future)
        assert math.isfinite(t)
    awd.close()
    return trace


@pytest.mark.parametrize("case", load_cases(), ids=lambda c: c["name"])
def test_library_reproduces_hand_worked_traces(case):
    p = params_of(case["params"])
    got = drive_library(p, [float(a) for a in case["arrival"]], inf_none(case["ddl"]), case["new_len"],
                        lambda lb, d: case["service_us"], rate_hat=case["rate_hat"], s_hat_table=table_of(case))
    want = [(w["t"], w["req_ids"], w["len_bucket"], w["depth"], w["reason"], w["w_after"], w["d_after"]) for w in case["trace"]]
    assert got == want


@pytest.mark.parametrize("seed", range(12))
def test_library_matches_oracle_on_random_workloads(seed):
    rng = np.random.default_rng(2000 + seed)
    p = AO.AwdParams(len_buckets=(16, 32, 64), depths=(1, 2, 4, 8, 16, 32), mem_budget=int(rng.choice([64, 128, 512, 2048])),
                     sigma=float(rng.choice([0.0, 25.0])), w_min=float(rng.choice([0.0, 15.0])), w_max=float(rng.choice([300.0, 2000.0])),
                     s_hat=90.0, t_max=float(rng.choice([math.inf, 700.0])), delta=float(rng.choice([0.0, 10.0])),
                     sla_window=bool(seed % 2), d_regrow=bool(seed % 3 == 0), fuse_budget=int(rng.choice([-1, 0, 64, 128])))
    arrival, ddl, new_len = random_workload(rng, 300, with_ddl=seed % 4 != 0)
    svc = lambda lb, d: 70.0 + 0.04 * lb * d
    table = None
    if seed >= 6:       # per-shape estimates: exact for some shapes, absent (default) for the others
        table = {(lb, d): svc(lb, d) for lb in p.len_buckets for d in p.depths if (lb // 16 + d) % 3}
    want = AO.simulate(p, arrival, ddl, new_len, svc, rate_hat=0.02, s_hat_table=table)
    got = drive_library(p, arrival, ddl, new_len, svc, rate_hat=0.02, s_hat_table=table)
    assert len(got) == len(want)
    for g, w in zip(got, want):
        assert g == (w.t, w.req_ids, w.len_bucket, w.depth, w.reason, w.w_after, w.d_after)


def test_library_awd_argument_errors():
    from paper_2601_11589_amd import api
    with pytest.raises(api.LapsError):
        api.LapsAwd((16, 16), (1, 2), 64)                      # buckets not strictly ascending
    with pytest.raises(api.LapsError):
        api.LapsAwd((16, 64), (2, 4), 64)                      # largest bucket never fits
    with pytest.raises(api.LapsError):
        api.LapsAwd((16,), (1, 2), 64, w_min_us=5.0, w_max_us=1.0)
    awd = api.LapsAwd((16, 32), (1, 2, 4), 64)
    assert awd.target_depth == 4 and awd.window_us == 10_000.0
    assert awd.laps_awd_poll(0.0, [], [], [])["wake_us"] == math.inf
    with pytest.raises(api.LapsError):
        awd.laps_awd_poll(5.0, [0.0], [math.inf], [33])        # longer than the largest bucket
    with pytest.raises(api.LapsError):
        awd.laps_awd_poll(5.0, [3.0, 1.0], [math.inf] * 2, [4, 4])   # not in arrival order
    with pytest.raises(api.LapsError):
        awd.laps_awd_poll(5.0, [9.0], [math.inf], [4])         # arrival after now
    r = awd.laps_awd_poll(5.0, [1.0], [math.inf], [4])
    assert not r["dispatch"] and r["wake_us"] == 1.0 + 10_000.0
    with pytest.raises(api.LapsError):
        awd.laps_awd_begin_round(6.0)                          # a round is collecting
    awd.close()
