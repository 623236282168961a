"""Host-only tests of the dual-queue step loops (paper_2601_11589_amd/dualqueue.py) on a step-time model.

The loops are what turns measured GPU step times into request latencies; here the step times come from a model
instead of the GPU, and the loops are pinned to what queueing theory fixes for them (Section 2.2 of the paper:
M/G/1 first-come-first-served, the Pollaczek-Khinchine mean wait W = lambda E[S^2] / (2 (1 - rho)) and the
head-of-line penalty lambda p (1 - p) (S_l - S_s)^2 / (2 (1 - rho)) that a long / short mix adds to it) and to the
properties Section 3.2 asks of temporal disaggregation (one class per step, every request served once, short
requests do not wait for a whole long request).  The adaptive batcher inside `run_awd` is the library's host object.
"""
import numpy as np
import pytest

from paper_2601_11589_amd import dualqueue


class LinearSteps:
    """Step durations: an un-captured batch costs `a + b * tokens`, a graph replay `c + d * depth * len_bucket`."""

    def __init__(self, a=0.0, b=1.0, c=200.0, d=1.0):
        self.a, self.b, self.c, self.d = a, b, c, d
        self.log = []

    def varlen_us(self, segs):
        self.log.append(("varlen", [(r, cnt) for r, _, cnt, _ in segs]))
        return self.a + self.b * sum(cnt for _, _, cnt, _ in segs)

    def graph_us(self, len_bucket, depth, new_lens):
        assert len(new_lens) <= depth and max(new_lens) <= len_bucket
        self.log.append(("graph", len_bucket, depth, list(new_lens)))
        return self.c + self.d * depth * len_bucket


def host_queue(new_len, params, model):
    new_len = np.asarray(new_len)
    return dualqueue.DualQueue(None, None, new_len, np.zeros_like(new_len), None, None, None, None, params,
                               step_model=model)


def poisson(seed, n, rate_per_us):
    rng = np.random.default_rng(seed)
    return np.cumsum(rng.exponential(1.0 / rate_per_us, n))


def test_unified_fcfs_is_m_d_1_for_equal_requests():
    """One request per step, constant service S: mean wait in queue = rho S / (2 (1 - rho))."""
    n, S, rho = 40_000, 64.0, 0.6
    p = dualqueue.DQParams(unified_budget=64)
    dq = host_queue(np.full(n, 64), p, LinearSteps(a=0.0, b=1.0))
    arr = poisson(1, n, rho / S)
    res = dq.run_unified(arr)
    wait = res.latency_us - S
    assert wait.min() >= -1e-9
    assert wait.mean() == pytest.approx(rho * S / (2 * (1 - rho)), rel=0.05)
    assert res.gpu_busy_us == pytest.approx(n * S)


def test_unified_fcfs_matches_pollaczek_khinchine_and_the_hol_penalty():
    """Two classes, the head request served to completion (budget = one short request): W = lambda E[S^2] / (2 (1 - rho));
    against the same load with every service time equal to the mean, the wait grows by the head-of-line term."""
    n, S_s, k, p_short, rho = 60_000, 64.0, 16, 0.9, 0.6
    S_l = k * S_s
    rng = np.random.default_rng(2)
    is_short = rng.random(n) < p_short
    new_len = np.where(is_short, 64, 64 * k)
    ES = p_short * S_s + (1 - p_short) * S_l
    ES2 = p_short * S_s ** 2 + (1 - p_short) * S_l ** 2
    lam = rho / ES
    params = dualqueue.DQParams(unified_budget=64)
    arr = poisson(3, n, lam)
    mixed = host_queue(new_len, params, LinearSteps(a=0.0, b=1.0)).run_unified(arr)
    service = np.where(is_short, S_s, S_l)
    w_mixed = (mixed.latency_us - service).mean()
    assert w_mixed == pytest.approx(lam * ES2 / (2 * (1 - rho)), rel=0.06)
    hol = lam * p_short * (1 - p_short) * (S_l - S_s) ** 2 / (2 * (1 - rho))
    w_flat = lam * ES ** 2 / (2 * (1 - rho))            # M/D/1 at the same mean service time
    assert w_mixed - w_flat == pytest.approx(hol, rel=0.08)
    # the convoy effect: the same queueing term weighs far more on a short request's normalised latency
    assert (mixed.latency_us[is_short] / S_s).mean() > 2.5 * (mixed.latency_us[~is_short] / S_l).mean()


def mixed_workload(seed, n_short=400, n_long=6):
    rng = np.random.default_rng(seed)
    new_len = np.concatenate([rng.integers(1, 65, n_short), rng.integers(4096, 8193, n_long)])
    arr = np.concatenate([np.sort(rng.uniform(0, 400_000.0, n_short)), np.linspace(0, 300_000.0, n_long)])
    return new_len, arr


def test_disaggregation_serves_every_request_once_one_class_per_step():
    new_len, arr = mixed_workload(5)
    model = LinearSteps(a=100.0, b=4.0, c=900.0, d=0.5)
    params = dualqueue.DQParams(short_token_budget=128)
    dq = host_queue(new_len, params, model)
    res = dq.run_disaggregated(arr, 2000.0)
    assert np.all(res.finish_us > arr)
    served = {}
    for step in model.log:
        if step[0] == "varlen":
            (r, cnt), = step[1]                              # a long step is one chunk of one request
            assert new_len[r] > params.short_max_len and cnt <= params.long_chunk
            served[r] = served.get(r, 0) + cnt
        else:
            _, lb, depth, lens = step
            assert depth * lb <= params.short_token_budget and all(l <= params.short_max_len for l in lens)
    assert all(served[r] == new_len[r] for r in np.nonzero(new_len > 64)[0])
    n_short_served = sum(len(s[3]) for s in model.log if s[0] == "graph")
    assert n_short_served == int(np.sum(new_len <= 64))
    assert res.gpu_busy_us <= res.makespan_us + 1e-6
    assert res.n_steps == len(model.log)


def test_a_short_request_waits_for_a_chunk_not_for_a_whole_long_request():
    """Section 3.2: with long work always pending, a short request that arrives alone waits at most the window, the
    long chunk in flight and its own replay - under the unified baseline it waits for everything queued before it."""
    model = LinearSteps(a=0.0, b=10.0, c=1000.0, d=0.0)     # a 2048-token chunk: 20.48 ms; a replay: 1 ms
    new_len = np.array([8192, 8192, 8192, 16, 16, 16])
    arr = np.array([0.0, 0.0, 0.0, 30_000.0, 90_000.0, 150_000.0])
    params = dualqueue.DQParams()
    window = 2000.0
    dis = host_queue(new_len, params, model).run_disaggregated(arr, window)
    chunk, replay = 10.0 * 2048, 1000.0
    assert np.all(dis.latency_us[3:] <= window + chunk + replay + 1e-6)
    uni = host_queue(new_len, params, LinearSteps(a=0.0, b=10.0)).run_unified(arr)
    # FCFS: the first short request is behind 3 x 8192 tokens of long work
    assert uni.latency_us[3] >= 3 * 8192 * 10.0 - 30_000.0
    assert dis.latency_us[3:].max() < uni.latency_us[3:].min()
    # the price: the last long request finishes later than under FCFS by exactly the short replays that cut in
    assert dis.finish_us[:3].max() == pytest.approx(uni.finish_us[:3].max() + 3 * replay)


def test_awd_loop_on_the_step_model_serves_everything_within_the_captured_grid():
    new_len, arr = mixed_workload(7, n_short=300, n_long=3)
    model = LinearSteps(a=100.0, b=4.0, c=900.0, d=0.5)
    params = dualqueue.DQParams(short_token_budget=512)
    dq = host_queue(new_len, params, model)
    ddl = arr + 50_000.0
    res = dq.run_awd(arr, ddl_us=ddl, s_hat_us=1000.0, sigma_us=2000.0, w_max_us=10_000.0, t_max_us=25_000.0,
                     delta_us=1000.0, sla_window=True)
    assert np.all(res.finish_us > arr)
    graphs = [s for s in model.log if s[0] == "graph"]
    assert sum(len(s[3]) for s in graphs) == 300
    for _, lb, depth, lens in graphs:
        assert lb in params.len_buckets and depth in params.depths and lb * depth <= params.short_token_budget
    assert res.step_kinds["short_graph"] == len(graphs)
    assert set(res.step_kinds["dispatch_reasons"]) <= {"depth", "sla", "tmax", "window"}
    # head-of-line cap: no short request waits longer than T_max plus the long chunk that may be in flight and the replay
    short = new_len <= 64
    assert res.latency_us[short].max() <= 25_000.0 + (100.0 + 4.0 * 2048) + (900.0 + 0.5 * 512) + 1e-6


def test_schedule_parameters_follow_the_runtime_fit():
    """Section 2.1 "runtime fitting", closed into the schedule: samples (T_comp, T_mem, L, H) planted from two
    different machines go through the library's fit and parameter derivation, and the dual-queue parameters move with
    them - the classification boundary, the bucket grid in use, the fusion budget - and with them what the step
    loop does with the same requests."""
    from paper_2601_11589_amd import api
    rng = np.random.default_rng(5)
    L = rng.integers(1, 2049, 120).astype(float)
    H = rng.choice([0.0, 1024.0, 4096.0], 120)
    grid = dict(len_buckets=(8, 16, 32, 64, 128, 256), depths=(1, 2, 4, 8, 16, 32, 64))

    def params_for(alpha, beta, gamma_w, gamma_r, floor_us):
        tc = alpha * L * (L + 2 * H) + beta * L
        tm = gamma_w * L + gamma_r * H
        coef = api.laps_lm_fit(L, H, tc * (1 + 0.01 * rng.standard_normal(120)), tm * (1 + 0.01 * rng.standard_normal(120)))
        assert coef == pytest.approx((alpha, beta, gamma_w, gamma_r), rel=0.05)
        return dualqueue.DQParams.from_fit(coef, floor_us, 4096.0, **grid), coef

    # machine A: the figures measured on MI355X (microseconds, 4 layers): the knee lies near 200 padded tokens
    pa, ca = params_for(5.6e-5, 3.6, 0.1, 0.02, 700.0)
    assert 150 < api.laps_lm_knee(*ca, 700.0, 4096.0) < api.laps_lm_knee(*ca, 700.0, 0.0) < 250
    assert (pa.short_max_len, pa.fuse_budget, pa.merge_below) == (128, 128, 128) and pa.len_buckets == (8, 16, 32, 64, 128)
    # machine B: four times the bandwidth for the same arithmetic (floor 175 us): the knee drops to ~49 tokens for a
    # fresh prompt (175 / (beta - gamma_w)); with history the cache read adds to the memory side and it is a little higher
    pb, cb = params_for(5.6e-5, 3.6, 0.1, 0.02, 175.0)
    assert 32 < api.laps_lm_knee(*cb, 175.0, 0.0) < 64 and api.laps_lm_knee(*cb, 175.0, 4096.0) > api.laps_lm_knee(*cb, 175.0, 0.0)
    assert (pb.short_max_len, pb.fuse_budget, pb.merge_below) == (32, 32, 32) and pb.len_buckets == (8, 16, 32)
    # the same five requests, all waiting at t = 0: under A all but the 300-token one are short and (8+16+64+128 = 216
    # padded tokens, not below 128) run bucket by bucket; under B only the 8- and 12-token requests are short, and being
    # 8 + 16 = 24 < 32 padded tokens they are fused into one 16-token graph
    new_len = [8, 12, 50, 100, 300]
    for prm, n_long, graphs in ((pa, 1, [(8, 1), (16, 1), (64, 1), (128, 1)]), (pb, 3, [(16, 2)])):
        model = LinearSteps()
        dq = host_queue(new_len, prm, model)
        assert int(dq.is_long.sum()) == n_long
        res = dq.run_disaggregated(np.zeros(5), window_us=0.0)
        assert np.all(res.finish_us > 0)
        assert sorted((e[1], e[2]) for e in model.log if e[0] == "graph") == graphs
