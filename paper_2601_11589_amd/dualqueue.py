"""Single-GPU dual-queue step loop: temporal long/short disaggregation against a unified mixed batch.

Section 3.2 of the paper keeps two queues, Q_s and Q_l, classified by prompt length, and lets an
instance execute one class at a time; short batches fill captured bucket shapes after a waiting window
(Section 3.1), long requests advance alone in fixed chunks.  Written for instances, the rule is read
here for one GPU as: every GPU step is either the planned bucket batches of the waiting short requests
(each one captured-graph replay) or one chunk of the oldest long request; short requests are dispatched
when the oldest has waited `window_us` or when `short_token_budget` padded tokens are waiting, otherwise
the next long chunk runs.  When few tokens wait, the buckets are fused into the largest one needed (the
paper's "graph fusion", Section 3.1): a replay then costs one pass over the weights whatever its shape.
`run_awd` replaces the fixed window by Adaptive-Wait-Depth batching (Algorithm 1, Section 3.2a): the
library's laps_awd_* state decides when the short queue leaves and in which captured shape, one replay per
dispatch; long chunks fill the time in which the short round is still collecting.
The baseline is the policy the paper argues against (Section 2.3): one FCFS queue, each step a
token-budget batch that mixes the next long chunk with whatever short requests fit - with a budget of
one chunk (a mixed, chunked batch), or with a budget that takes a long prompt whole (memory-based
batching as Section 2.3 states it: the short requests behind a long prompt wait for all of it).

Arrivals are virtual timestamps; the clock advances by the measured GPU time of every step (HIP events
around the step, host launch overhead included when it stalls the GPU) and jumps over idle gaps.
Only sequencing lives here: every step runs through the C-ABI binding.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from . import api, runner


@dataclass
class DQParams:
    short_max_len: int = 64
    len_buckets: tuple = (16, 32, 64)
    depths: tuple = (1, 2, 4, 8, 16, 32, 64)
    short_token_budget: int = 2048     # padded tokens per captured short graph (token-max rule M_s)
    long_chunk: int = 2048             # C_l
    unified_budget: int = 2048         # tokens per step of the unified baseline
    window_us: float = 1000.0          # fixed waiting window W
    fuse_budget: int = 128             # AWD: other length buckets join a batch only up to this many padded tokens
    merge_below: int = 128             # graph fusion: below this many waiting padded tokens (where a replay
                                       # costs one pass over the weights whatever its shape) all waiting short
                                       # requests share the largest needed length bucket: one replay, not three

    @classmethod
    def from_fit(cls, coef, weight_floor_us: float, hist_max: float, len_buckets=(16, 32, 64),
                 depths=(1, 2, 4, 8, 16, 32, 64), **kw):
        """Parameters taken from a run-time fit of the latency model (Section 2.1) instead of constants: the library
        (laps_lm_derive_params) turns (alpha, beta, gamma_w, gamma_r) and the measured weight-streaming floor into the
        classification boundary, and the padded-token size up to which a replay costs one pass over the weights - the
        budget below which waiting requests are fused into one graph and up to which AWD lets other buckets join."""
        d = api.laps_lm_derive_params(coef, weight_floor_us, hist_max, list(len_buckets), list(depths))
        buckets = tuple(b for b in len_buckets if b <= d["short_max_len"])
        return cls(short_max_len=d["short_max_len"], len_buckets=buckets, depths=tuple(depths),
                   fuse_budget=d["fuse_budget"], merge_below=d["fuse_budget"], **kw)


@dataclass
class DQResult:
    mode: str
    makespan_us: float
    gpu_busy_us: float
    n_steps: int
    finish_us: np.ndarray
    latency_us: np.ndarray
    step_kinds: dict = field(default_factory=dict)

    def summary(self, new_len, is_long) -> dict:
        lat_s, lat_l = self.latency_us[~is_long], self.latency_us[is_long]
        pc = lambda v, q: float(np.percentile(v, q)) / 1e3 if len(v) else None
        return {"mode": self.mode, "makespan_ms": self.makespan_us / 1e3, "gpu_busy_ms": self.gpu_busy_us / 1e3,
                "steps": self.n_steps, "step_kinds": self.step_kinds,
                "tokens_per_s": float(np.sum(new_len)) / (self.makespan_us * 1e-6),
                "slo_400ms_violation_frac": float(np.mean(self.latency_us > 400_000.0)),
                "short_latency_ms": {"p50": pc(lat_s, 50), "p90": pc(lat_s, 90), "mean": float(lat_s.mean()) / 1e3},
                "long_latency_ms": {"p50": pc(lat_l, 50), "p90": pc(lat_l, 90), "mean": float(lat_l.mean()) / 1e3}}


class DualQueue:
    """Holds the device-resident workload (packed activations, page tables, pools) and runs either policy."""

    def __init__(self, ctx: api.LapsCtx, layers, new_len, prefix_len, page_table, d_x: torch.Tensor, k_pools, v_pools,
                 params: DQParams, keep_outputs: bool = False, step_model=None):
        """step_model: None runs every step on the GPU.  Otherwise an object with
        `varlen_us(segs)` (segs = [(request, first new token, count, cached tokens before it)]) and
        `graph_us(len_bucket, depth, new_lens)` that returns the duration of a step instead of running it: the
        policies below then work on the clock alone (no GPU, no device memory; ctx, layers, page_table, d_x and the
        pools may be None) - for tests of the step loops against queueing theory and for what-if studies."""
        self.ctx, self.layers, self.p = ctx, layers, params
        self.new_len = np.asarray(new_len, np.int64)
        self.prefix_len = np.asarray(prefix_len, np.int64)
        self.n = len(self.new_len)
        self.is_long = self.new_len > params.short_max_len
        self.cu = np.concatenate([[0], np.cumsum(self.new_len)])
        self.step_model = step_model
        self.out = None
        if step_model is not None:
            self.short = None
            return
        self.page_table = np.ascontiguousarray(page_table, np.int32)
        self.d_page_table = torch.from_numpy(self.page_table).cuda()
        self.d_x, self.k_pools, self.v_pools = d_x, k_pools, v_pools
        self.stream = torch.cuda.Stream()
        self.short = runner.ShortRunner(ctx, layers, k_pools, v_pools, self.page_table.shape[1], self.stream)
        self.out = torch.zeros_like(d_x) if keep_outputs else None
        ctx.workspace(max(params.unified_budget, params.long_chunk), min(self.n, params.unified_budget))
        self._ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        self.stream.wait_stream(torch.cuda.current_stream())   # self.out and the page table were filled on that stream

    # ------------------------------------------------------------------ timed execution of one step
    def _timed(self, fn) -> float:
        e0, e1 = self._ev
        e0.record(self.stream)
        fn()
        e1.record(self.stream)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3   # microseconds

    def _run_varlen(self, segs) -> float:
        """segs: list of (request, first new token, count).  One un-captured packed batch."""
        if self.step_model is not None:
            return float(self.step_model.varlen_us([(r, a, c, int(self.prefix_len[r]) + a) for r, a, c in segs]))
        with torch.cuda.stream(self.stream):
            ids = [s[0] for s in segs]
            x = torch.cat([self.d_x[self.cu[r] + a: self.cu[r] + a + c] for r, a, c in segs])
            cu = torch.tensor(np.concatenate([[0], np.cumsum([c for _, _, c in segs])]), dtype=torch.int32, device="cuda")
            pre = torch.tensor([int(self.prefix_len[r]) + a for r, a, _ in segs], dtype=torch.int32, device="cuda")
            pt = self.d_page_table[torch.tensor(ids, device="cuda")].contiguous()
            out = torch.empty_like(x)
            self.stream.synchronize()          # input placement is not part of the step
            us = self._timed(lambda: self.ctx.laps_prefill_stack(self.layers, cu, None, pre, pt, self.k_pools,
                                                                 self.v_pools, x, out, self.stream))
            if self.out is not None:
                o = 0
                for r, a, c in segs:
                    self.out[self.cu[r] + a: self.cu[r] + a + c] = out[o:o + c]
                    o += c
                self.stream.synchronize()
        return us

    def _run_short_batches(self, req_ids, fused_len_bucket: int = 0):
        """Plans the waiting short requests and replays one captured graph per planned batch; with fused_len_bucket
        (the library's decision, laps_window_poll) every request runs in that one length bucket.
        Returns a list of (request ids, microseconds) per batch."""
        p = self.p
        ids = list(req_ids)
        buckets = [fused_len_bucket] if fused_len_bucket else list(p.len_buckets)
        plan = api.laps_plan_buckets(min(p.short_max_len, buckets[-1]), buckets, list(p.depths), p.short_token_budget,
                                     p.long_chunk, self.new_len[ids], self.prefix_len[ids])
        assert not plan["longs"]
        return self._run_planned(ids, plan)

    def _run_planned(self, ids, plan):
        """Replays one captured graph per batch of `plan` (request ids local to `ids`)."""
        if self.step_model is not None:
            return [([ids[j] for j in b["req_ids"]],
                     float(self.step_model.graph_us(b["len_bucket"], b["depth"], [int(self.new_len[ids[j]]) for j in b["req_ids"]])))
                    for b in plan["batches"]]
        cu_local = np.concatenate([[0], np.cumsum(self.new_len[ids])])
        with torch.cuda.stream(self.stream):
            x_local = torch.cat([self.d_x[self.cu[r]: self.cu[r + 1]] for r in ids])
            staged = runner.stage_short_batches(plan, self.new_len[ids], self.prefix_len[ids], self.page_table[ids],
                                                cu_local, x_local, self.d_x.shape[1])
            self.stream.synchronize()
        res = []
        for sb in staged:
            out = None
            if self.out is not None:
                out = torch.empty((sb.real_tokens, self.d_x.shape[1]), dtype=torch.float32, device="cuda")
            self.short.graph_for(sb.len_bucket, sb.depth)      # capture (first use) is not part of the step
            us = self._timed(lambda: self.short.run(sb, out))
            if out is not None:
                row = 0
                for j in sb.req_ids:
                    r = ids[j]
                    self.out[self.cu[r]: self.cu[r + 1]] = out[row: row + int(self.new_len[r])]
                    row += int(self.new_len[r])
                self.stream.synchronize()
            res.append(([ids[j] for j in sb.req_ids], us))
        return res

    # ------------------------------------------------------------------ policies
    def run_unified(self, arrival_us, budget: int | None = None) -> DQResult:
        """One FCFS queue, every step a token-budget batch of whatever waits.  budget None: `unified_budget` tokens per
        step (the head long request advances in chunks of what is left of it: a mixed, chunked batch).  A budget of at
        least the longest prompt gives the memory-based batching of Section 2.3 as the paper states it: a long prompt
        enters whole, together with the short requests that fit behind it."""
        step_budget = self.p.unified_budget if budget is None else int(budget)
        arrival = np.asarray(arrival_us, np.float64)
        order = list(np.argsort(arrival, kind="stable"))
        done = np.zeros(self.n, np.int64)
        finish = np.zeros(self.n)
        t, busy, steps, nxt = 0.0, 0.0, 0, 0
        queue = []
        while nxt < self.n or queue:
            while nxt < self.n and arrival[order[nxt]] <= t:
                queue.append(order[nxt])
                nxt += 1
            if not queue:
                t = arrival[order[nxt]]
                continue
            budget, segs = step_budget, []
            for r in queue:                                   # FCFS, the head long request is chunked by what is left
                if budget == 0:
                    break
                c = int(min(self.new_len[r] - done[r], budget))
                segs.append((r, int(done[r]), c))
                budget -= c
            us = self._run_varlen(segs)
            t += us
            busy += us
            steps += 1
            for r, a, c in segs:
                done[r] += c
                if done[r] == self.new_len[r]:
                    finish[r] = t
            queue = [r for r in queue if done[r] < self.new_len[r]]
        mode = "unified" if step_budget == self.p.unified_budget else f"unified(budget={step_budget})"
        return DQResult(mode, t, busy, steps, finish, finish - arrival, {"mixed": steps})

    def run_disaggregated(self, arrival_us, window_us=None) -> DQResult:
        p = self.p
        window = p.window_us if window_us is None else window_us
        arrival = np.asarray(arrival_us, np.float64)
        order = list(np.argsort(arrival, kind="stable"))
        done = np.zeros(self.n, np.int64)
        finish = np.zeros(self.n)
        t, busy, nxt = 0.0, 0.0, 0
        kinds = {"short_graph": 0, "long_chunk": 0, "short_busy_us": 0.0}
        q_s, q_l = [], []
        while nxt < self.n or q_s or q_l:
            while nxt < self.n and arrival[order[nxt]] <= t:
                r = order[nxt]
                (q_l if self.is_long[r] else q_s).append(r)
                nxt += 1
            # the dispatch rule (window, budget, nothing else to run) and the fusion rule live in the library
            dec = api.laps_window_poll(p.len_buckets, window, p.short_token_budget, p.merge_below, t, arrival[q_s],
                                       self.new_len[q_s], not q_l and nxt >= self.n)
            if dec["dispatch"]:
                batch, q_s = q_s, []
                for ids, us in self._run_short_batches(batch, dec["fused_len_bucket"]):
                    t += us
                    busy += us
                    kinds["short_graph"] += 1
                    kinds["short_busy_us"] += us
                    for r in ids:
                        done[r] = self.new_len[r]
                        finish[r] = t
            elif q_l:
                r = q_l[0]
                c = int(min(self.new_len[r] - done[r], p.long_chunk))
                us = self._run_varlen([(r, int(done[r]), c)])
                t += us
                busy += us
                kinds["long_chunk"] += 1
                done[r] += c
                if done[r] == self.new_len[r]:
                    finish[r] = t
                    q_l.pop(0)
            else:
                wake = [arrival[order[nxt]]] if nxt < self.n else []
                if q_s:
                    wake.append(dec["wake_us"])
                t = max(t, min(wake))
        return DQResult(f"disaggregated(W={window:g}us)", t, busy, kinds["short_graph"] + kinds["long_chunk"], finish,
                        finish - arrival, kinds)

    def run_awd(self, arrival_us, ddl_us=None, s_hat_us=2000.0, sigma_us=0.0, w_min_us=0.0, w_max_us=20000.0,
                t_max_us=float("inf"), delta_us=0.0, sla_window=False, d_regrow=True, rate_ewma=0.2) -> DQResult:
        """Temporal disaggregation with the short queue batched by laps_awd_*.  ddl_us: absolute deadlines of the
        requests (None: deadline-free).  The arrival-rate estimate for the SLA window is an exponentially
        weighted mean of the short inter-arrival gaps."""
        p = self.p
        arrival = np.asarray(arrival_us, np.float64)
        ddl = np.full(self.n, np.inf) if ddl_us is None else np.asarray(ddl_us, np.float64)
        order = list(np.argsort(arrival, kind="stable"))
        known = [ddl[r] - s_hat_us for r in order if arrival[r] <= 0.0 and not self.is_long[r]]
        awd = api.LapsAwd(p.len_buckets, p.depths, p.short_token_budget, sigma_us, w_min_us, w_max_us, s_hat_us, t_max_us,
                          delta_us, 1e-9, sla_window, d_regrow, first_slack_us=min(known, default=float("inf")),
                          fuse_budget=p.fuse_budget)
        done = np.zeros(self.n, np.int64)
        finish = np.zeros(self.n)
        t, busy, nxt = 0.0, 0.0, 0
        kinds = {"short_graph": 0, "long_chunk": 0, "short_busy_us": 0.0}
        reasons, depths_used = {}, []
        q_s, q_l = [], []
        gap, last_s = None, None
        # measured replay time per captured shape (exponentially weighted), handed to the library as S_hat
        s_tab = np.full((len(p.len_buckets), len(p.depths)), np.nan)
        while nxt < self.n or q_s or q_l:
            while nxt < self.n and arrival[order[nxt]] <= t:
                r = order[nxt]
                if self.is_long[r]:
                    q_l.append(r)
                else:
                    if last_s is not None:
                        g = arrival[r] - last_s
                        gap = g if gap is None else (1 - rate_ewma) * gap + rate_ewma * g
                    last_s = arrival[r]
                    q_s.append(r)
                nxt += 1
            wake = float("inf")
            if q_s:
                rate = 1.0 / gap if gap else 0.0
                dec = awd.laps_awd_poll(t, arrival[q_s], ddl[q_s], self.new_len[q_s], rate)
                if dec["dispatch"]:
                    ids = [q_s[j] for j in dec["take"]]
                    q_s = [r for r in q_s if r not in set(ids)]
                    plan = {"batches": [{"len_bucket": dec["len_bucket"], "depth": dec["depth"], "graph_ok": 1,
                                         "req_ids": list(range(len(ids)))}]}
                    (_, us), = self._run_planned(ids, plan)
                    t += us
                    busy += us
                    kinds["short_graph"] += 1
                    kinds["short_busy_us"] += us
                    reasons[dec["reason"]] = reasons.get(dec["reason"], 0) + 1
                    depths_used.append(len(ids))
                    li, di = list(p.len_buckets).index(dec["len_bucket"]), list(p.depths).index(dec["depth"])
                    s_tab[li, di] = us if np.isnan(s_tab[li, di]) else 0.5 * s_tab[li, di] + 0.5 * us
                    awd.laps_awd_set_service_table(s_tab)
                    for r in ids:
                        done[r] = self.new_len[r]
                        finish[r] = t
                    awd.laps_awd_begin_round(t)
                    continue
                wake = dec["wake_us"]
            if q_l:
                r = q_l[0]
                c = int(min(self.new_len[r] - done[r], p.long_chunk))
                us = self._run_varlen([(r, int(done[r]), c)])
                t += us
                busy += us
                kinds["long_chunk"] += 1
                done[r] += c
                if done[r] == self.new_len[r]:
                    finish[r] = t
                    q_l.pop(0)
            else:
                nxt_arr = arrival[order[nxt]] if nxt < self.n else float("inf")
                t = max(t, min(wake, nxt_arr))
        kinds["dispatch_reasons"] = reasons
        kinds["mean_short_depth"] = float(np.mean(depths_used)) if depths_used else 0.0
        kinds["final_W_us"], kinds["final_D"] = awd.window_us, awd.target_depth
        awd.close()
        mode = "awd(" + ("sla-window" if sla_window else "adaptive") + ")"
        return DQResult(mode, t, busy, kinds["short_graph"] + kinds["long_chunk"], finish, finish - arrival, kinds)

    def close(self):
        if self.short is not None:
            self.short.close()
