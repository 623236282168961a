"""Spatial disaggregation over N virtual instances, driven by single-GPU service times (host-only simulation).

Section 3.2 of the paper (spatial mode, Algorithm 2): N prefill instances form a SHORT and a LONG pool; two global
queues Q_s and Q_l, each instance pulls only from the queue of its pool; a controller looks at backlog, SLA
deviation and utilisation of every instance once per control period and moves at most one instance between the
pools.  There is one GPU here, so the instances are virtual: a step takes the time the same step was measured to
take on the real GPU (a table of short replay times per depth, a long chunk time), and only the queueing and the
controller are simulated.  The controller's decision is the library's (`laps_ctrl_step`); this module only owns
the clock and the queues.

Readings where the paper is silent: an idle SHORT instance takes up to `short_depth` waiting requests as one
step; an idle LONG instance takes the oldest long request and runs all of its chunks; the signals of instance k
over the last period are q_k = (length of its pool's queue) / (pool size), e_k = mean over the requests it
finished of max(0, latency - SLO) / SLO, u_k = busy fraction; the instance that migrates is the one of the donor
pool that becomes free first, and it changes pool when its current step ends.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import api


@dataclass
class PoolSimParams:
    n_total: int = 8
    n_short0: int = 4
    n_min: int = 1
    period_us: float = 200_000.0
    cool_us: float = 1_000_000.0
    tau: float = 0.25
    w_q: float = 1.0
    w_e: float = 4.0
    w_u: float = 0.5
    min_pressure: float = 0.5          # a pool gains an instance only when it has a backlog to show for it
    slo_us: float = 400_000.0          # TTFT objective used for the SLA deviation (the paper's 0.4 s)
    short_depth: int = 8
    long_chunk: int = 2048


def simulate(arrival_us, new_len, is_long, short_step_us, long_chunk_us, p: PoolSimParams, controller: bool = True):
    """short_step_us(depth) and long_chunk_us: measured durations of one short replay of `depth` requests and of
    one long chunk.  Returns a summary dict."""
    arrival = np.asarray(arrival_us, np.float64)
    n = len(arrival)
    order = np.argsort(arrival, kind="stable")
    ctrl = api.LapsCtrl(p.n_total, p.n_short0, p.n_min, p.cool_us, p.tau, p.w_q, p.w_e, p.w_u, 0.9, p.min_pressure)
    pool = ["S"] * p.n_short0 + ["L"] * (p.n_total - p.n_short0)     # current pool of every instance
    pending_move = [None] * p.n_total                                 # pool to switch to when the current step ends
    free_at = np.zeros(p.n_total)
    steps = [[] for _ in range(p.n_total)]       # (start, end) of the steps not yet fully accounted for
    devs = [[] for _ in range(p.n_total)]        # (finish time, SLA deviation) of requests not yet reported
    finish = np.zeros(n)
    q_s, q_l = [], []
    nxt, t, next_tick = 0, 0.0, p.period_us
    moves = []
    trace_ns = []
    done = 0

    def start_work(k, now):
        nonlocal done
        if pending_move[k] is not None:
            pool[k], pending_move[k] = pending_move[k], None
        if pool[k] == "S" and q_s:
            take, q_s[:] = q_s[:p.short_depth], q_s[p.short_depth:]
            dur = float(short_step_us(len(take)))
        elif pool[k] == "L" and q_l:
            take = [q_l.pop(0)]
            dur = float(long_chunk_us) * -(-int(new_len[take[0]]) // p.long_chunk)
        else:
            return False
        free_at[k] = now + dur
        steps[k].append((now, now + dur))
        for r in take:
            finish[r] = now + dur
            devs[k].append((now + dur, max(0.0, (now + dur - arrival[r]) - p.slo_us) / p.slo_us))
        done += len(take)
        return True

    while done < n:
        while nxt < n and arrival[order[nxt]] <= t:
            r = int(order[nxt])
            (q_l if is_long[r] else q_s).append(r)
            nxt += 1
        for k in range(p.n_total):
            if free_at[k] <= t:
                start_work(k, t)
        if controller and t >= next_tick:
            ids_s = [k for k in range(p.n_total) if pool[k] == "S" and pending_move[k] is None] + \
                    [k for k in range(p.n_total) if pending_move[k] == "S"]
            ids_l = [k for k in range(p.n_total) if k not in ids_s]
            def signals(ids, queue_len):
                out = []
                for k in ids:
                    busy = sum(max(0.0, min(e, t) - max(s0, t - p.period_us)) for s0, e in steps[k])
                    fin = [d for e, d in devs[k] if e <= t]
                    out.append((queue_len / max(len(ids), 1), float(np.mean(fin)) if fin else 0.0, busy / p.period_us))
                return out
            action, ps, pl = ctrl.laps_ctrl_step(t, signals(ids_s, len(q_s)), signals(ids_l, len(q_l)))
            if action != 0:
                donors = ids_l if action > 0 else ids_s
                k = min(donors, key=lambda j: free_at[j])
                pending_move[k] = "S" if action > 0 else "L"
                moves.append((t, action, k))
            trace_ns.append((t, ctrl.n_short, ps, pl))
            for k in range(p.n_total):      # keep what reaches beyond this tick for the next period
                steps[k] = [(s0, e) for s0, e in steps[k] if e > t]
                devs[k] = [(e, d) for e, d in devs[k] if e > t]
            next_tick += p.period_us
            continue
        events = [free_at[k] for k in range(p.n_total) if free_at[k] > t]
        if nxt < n:
            events.append(arrival[order[nxt]])
        if controller:
            events.append(next_tick)
        if not events:
            break
        t = min(events)
    ctrl.close()
    lat = finish - arrival
    is_long = np.asarray(is_long, bool)
    pc = lambda v, q: float(np.percentile(v, q)) / 1e3 if len(v) else None
    return {"controller": controller, "makespan_ms": float(finish.max()) / 1e3, "migrations": len(moves),
            "moves": [(round(tm / 1e3, 1), a) for tm, a, _ in moves],
            "n_short_over_time": [(round(tm / 1e3, 1), ns) for tm, ns, _, _ in trace_ns[:: max(1, len(trace_ns) // 16)]],
            "short_latency_ms": {"p50": pc(lat[~is_long], 50), "p99": pc(lat[~is_long], 99)},
            "long_latency_ms": {"p50": pc(lat[is_long], 50), "p99": pc(lat[is_long], 99)},
            "slo_violation_frac": float(np.mean(lat > p.slo_us))}


def shifting_workload(seed: int, horizon_us: float, short_rate_a: float, long_rate_a: float, short_rate_b: float,
                      long_rate_b: float):
    """Two phases of Poisson arrivals (requests per second per class): phase A over the first half of the horizon,
    phase B over the second.  Short lengths U[1,64], long lengths U[2048,8192]."""
    rng = np.random.default_rng(seed)
    arr, ln, lg = [], [], []
    for lo, hi, rs, rl in ((0.0, horizon_us / 2, short_rate_a, long_rate_a), (horizon_us / 2, horizon_us, short_rate_b, long_rate_b)):
        for rate, long_cls in ((rs, False), (rl, True)):
            t = lo
            while rate > 0:
                t += rng.exponential(1e6 / rate)
                if t >= hi:
                    break
                arr.append(t)
                lg.append(long_cls)
                ln.append(int(rng.integers(2048, 8193)) if long_cls else int(rng.integers(1, 65)))
    o = np.argsort(arr, kind="stable")
    return np.asarray(arr)[o], np.asarray(ln)[o], np.asarray(lg)[o]
