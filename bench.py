#!/usr/bin/env python3
"""Benchmark of the ragged-prefill hot path on one MI355X.

Primary workload (the short-prefill bucket configuration, configs[1] of the benchmark definition): 256 new
prompts, lengths U[8,64], bucketed to {16,32,64}, 4-layer stack of 32B-shaped layers, every bucket batch replayed
as a captured hipGraph.  One "step" = plan + stage + replay of every batch of the 256 requests.
The last line on stdout is one compact JSON record: the headline, the roofline of the dominant kernel, the other
workloads' key figures (token-max budgets, two streams, the multi-turn re-prefill workload, the long-prefill workload,
the latency-model fit with the schedule parameters derived from it, the mixed dual-queue workload) and the fp64 oracle
timed on the host cores (`cpu_baseline`).  The full record of every leg, including the budget sweep, the graph cost
table and the simulated instance pools, goes to `gpurun_out/<--detail-file>`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "prefill tokens/s + p90 latency; % MFMA peak (long) / % HBM peak (short) at 1 GPU"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFS = 2500.0
LEN_BUCKETS = [16, 32, 64]
DEPTHS = [1, 2, 4, 8, 16, 32, 64]
LONG_CHUNK = 2048
WHOLE_PROMPT_BUDGET = 16384   # tokens per step of the un-chunked memory-based baseline: the longest prompt (8K) and more


_T0 = time.perf_counter()


def log(*a):
    print(f"[{time.perf_counter() - _T0:6.1f}s]", *a, file=sys.stderr, flush=True)


def pct(v, q):
    import numpy as np
    return float(np.percentile(np.asarray(v, dtype=np.float64), q)) if len(v) else None


def source_digest():
    """sha256 over the GEMM kernel sources: the counter figures under profiles/traffic.json are stamped with it."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2601_11589_amd", "csrc")
    for name in ("gemm.hip", "laps_internal.h"):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def load_traffic(kernel_key):
    """HBM bytes per launch of a kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/traffic.json).
    None when the kernel sources have changed since the measurement: a stale counter reading is not reported."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if t.get("source_sha256") != source_digest():
        log("[bench] profiles/traffic.json was measured on other kernel sources: traffic = null")
        return None
    return t.get("kernels", {}).get(kernel_key, {}).get("hbm_bytes_per_launch")


def gemm_shapes(cfg):
    qd = cfg.n_q_heads * cfg.head_dim
    return {"gemm_qkv": (cfg.qkv_dim, cfg.hidden), "gemm_o": (cfg.hidden, qd),
            "gemm_gateup": (2 * cfg.intermediate, cfg.hidden), "gemm_down": (cfg.hidden, cfg.intermediate)}


def attn_flops(cfg, new_len, prefix_len):
    """Causal-triangle flops only: 4 * hd * n_q * (L*H + L(L+1)/2) per sequence per layer."""
    tot = 0
    for l, h in zip(new_len, prefix_len):
        l, h = int(l), int(h)
        tot += 4 * cfg.head_dim * cfg.n_q_heads * (l * h + l * (l + 1) // 2)
    return tot


def build_model(cfg, seed, n_layers=None):
    from paper_2601_11589_amd import api, inputs
    ctx = api.LapsCtx(cfg, max_positions=8192 + 64)
    layers = []
    host_layers = []
    t0 = time.perf_counter()
    for l in range(n_layers or cfg.n_layers):
        w = inputs.make_layer_weights(cfg, seed, l, threads=min(16, os.cpu_count() or 8))
        layers.append(ctx.upload_layer(w))
        host_layers.append(w)
        log(f"[bench] layer {l} weights generated + uploaded ({time.perf_counter() - t0:.1f}s)")
    return ctx, layers, host_layers


# ------------------------------------------------------------------------------------- short buckets
def run_short(ctx, layers, cfg, token_budget, steps, warmup, profile_kernels, tag, config=2, two_streams=False):
    import numpy as np
    import torch
    from paper_2601_11589_amd import api, inputs, runner

    seed = inputs.SEED_BASE + config
    b = inputs.make_batch(config)
    T = b.n_tokens
    d_x = torch.from_numpy(inputs.make_activations(cfg, seed, T)).cuda()
    k_pools, v_pools = ctx.new_pools(b.n_pages, cfg.n_layers)
    if int(b.prefix_len.max()) > 0:      # cached prefix content: seeded N(0,1) bf16 drawn on the device
        gen = torch.Generator(device="cuda").manual_seed(seed)
        for p in k_pools + v_pools:
            p.copy_(torch.randn(p.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16))
    plan_args = (64, LEN_BUCKETS, DEPTHS, token_budget, LONG_CHUNK, b.new_len, b.prefix_len)
    plan = api.laps_plan_buckets(*plan_args)
    assert not plan["longs"]
    staged = runner.stage_short_batches(plan, b.new_len, b.prefix_len, b.page_table, b.cu_seqlens, d_x, cfg.hidden)
    max_rows = max(s.depth * s.len_bucket for s in staged)
    ctx.workspace(max_rows, max(s.depth for s in staged))
    stream = torch.cuda.Stream()
    sr = runner.ShortRunner(ctx, layers, k_pools, v_pools, b.page_table.shape[1], stream)
    for s in staged:                      # capture every needed shape
        sr.graph_for(s.len_bucket, s.depth)
    shapes = sorted(sr.graphs.keys())
    log(f"[bench:{tag}] {len(staged)} batches, shapes {shapes}, capture s/graph "
        f"{[round(sr.capture_s[k], 3) for k in shapes]}, graph MB "
        f"{[round(sr.graphs[k].laps_graph_device_bytes() / 1e6, 1) for k in shapes]}")
    for _ in range(warmup):
        for s in staged:
            sr.run(s)
    stream.synchronize()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in staged]
          for _ in range(steps)]
    plan_us = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        tp = time.perf_counter()
        api.laps_plan_buckets(*plan_args)            # the integer plan is part of every step
        plan_us.append((time.perf_counter() - tp) * 1e6)
        for j, s in enumerate(staged):
            ev[k][j][0].record(stream)
            sr.run(s)
            ev[k][j][1].record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    lat = []                                          # per request: duration of the batch that served it
    for k in range(steps):
        for j, s in enumerate(staged):
            ms = ev[k][j][0].elapsed_time(ev[k][j][1])
            lat += [ms] * s.n_real
    res = {"tokens_per_s": T * steps / wall, "ms_per_step": wall / steps * 1e3, "real_tokens": T,
           "padded_rows": int(sum(s.depth * s.len_bucket for s in staged)), "n_batches": len(staged),
           "token_budget": token_budget, "latency_ms_p50": pct(lat, 50), "latency_ms_p90": pct(lat, 90),
           "plan_us": float(np.median(plan_us)), "graph_shapes": [list(k) for k in shapes],
           "graph_capture_s": {f"{k[0]}x{k[1]}": round(sr.capture_s[k], 4) for k in shapes},
           "graph_device_MB": {f"{k[0]}x{k[1]}": round(sr.graphs[k].laps_graph_device_bytes() / 1e6, 2) for k in shapes}}
    if two_streams:
        # throughput variant: batches alternate between two streams, each with its own graph instances, so that the
        # latency-bound kernels of one replay overlap the weight streaming of the other (per-batch latency rises)
        stream_b = torch.cuda.Stream()
        sr_b = runner.ShortRunner(ctx, layers, k_pools, v_pools, b.page_table.shape[1], stream_b)
        for s in staged:
            sr_b.graph_for(s.len_bucket, s.depth)
        pair = [(sr, stream), (sr_b, stream_b)]
        for j, s in enumerate(staged):
            pair[j % 2][0].run(s)
        torch.cuda.synchronize()
        ev2 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in staged]
        t0 = time.perf_counter()
        for k in range(steps):
            for j, s in enumerate(staged):
                r, st = pair[j % 2]
                if k == steps - 1:
                    ev2[j][0].record(st)
                r.run(s)
                if k == steps - 1:
                    ev2[j][1].record(st)
        torch.cuda.synchronize()
        wall2 = time.perf_counter() - t0
        lat2 = []
        for j, s in enumerate(staged):
            lat2 += [ev2[j][0].elapsed_time(ev2[j][1])] * s.n_real
        res["two_streams"] = {"tokens_per_s": T * steps / wall2, "ms_per_step": wall2 / steps * 1e3,
                              "latency_ms_p50": pct(lat2, 50), "latency_ms_p90": pct(lat2, 90)}
        sr_b.close()
    if profile_kernels:
        # same kernels, same launch shapes as the graph (its depth slots and depth * len_bucket rows, the requests
        # packed at the front), un-captured, every launch bracketed by HIP events on its stream
        ctx.laps_prof_enable(True)
        padded = []
        for s in staged:
            M = s.depth * s.len_bucket
            x = torch.zeros((M, cfg.hidden), dtype=torch.float32, device="cuda")
            x[: s.real_tokens] = s.x_rows
            pl = torch.zeros(s.depth, dtype=torch.int32, device="cuda")
            pl[: s.n_real] = s.prefix_len
            pt = torch.zeros((s.depth, s.page_table.shape[1]), dtype=torch.int32, device="cuda")
            pt[: s.n_real] = s.page_table
            cu = torch.full((s.depth + 1,), s.real_tokens, dtype=torch.int32, device="cuda")
            cu[: s.n_real + 1] = s.cu
            padded.append((cu, None, pl, pt, x, M))
        torch.cuda.synchronize()
        gbytes = 0.0
        gflops = 0.0
        prof = {}
        per_shape = {}
        with torch.cuda.stream(stream):
            for sb, (cu, sl, pl, pt, x, M) in zip(staged, padded):
                ctx.laps_prof_enable(True)            # (re)starts the per-class timers: one read per batch
                ctx.laps_prefill_stack(layers, cu, sl, pl, pt, k_pools, v_pools, x, None, stream)
                stream.synchronize()
                one = ctx.laps_prof_read()
                for k, v in one.items():
                    acc = prof.setdefault(k, [0.0, 0])
                    acc[0] += v[0]
                    acc[1] += v[1]
                by, fl = 0.0, 0.0
                R = sb.real_tokens                     # rows past the packed requests are neither loaded nor stored
                for (n, kk) in gemm_shapes(cfg).values():
                    by += cfg.n_layers * (n * kk * 2 + R * kk * 2 + R * n * 4)
                    fl += cfg.n_layers * 2.0 * R * n * kk
                gbytes += by
                gflops += fl
                ps = per_shape.setdefault(f"{sb.len_bucket}x{sb.depth}", [0.0, 0.0, 0.0, 0])
                ps[0] += sum(one[k][0] for k in gemm_shapes(cfg))
                ps[1] += by
                ps[2] += fl
                ps[3] += 1
        ctx.laps_prof_enable(False)
        prof = {k: (v[0], v[1]) for k, v in prof.items()}
        # both roofline fractions of the four projections for every captured shape
        res["gemm_per_shape"] = {k: {"batches": v[3], "graph_rows": int(k.split("x")[0]) * int(k.split("x")[1]),
                                     "hbm_frac": v[1] / (v[0] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                     "mfma_frac": v[2] / (v[0] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFS}
                                 for k, v in per_shape.items()}
        gms = sum(prof[k][0] for k in gemm_shapes(cfg))
        gcnt = sum(prof[k][1] for k in gemm_shapes(cfg))
        res["kernel_ms"] = {k: round(v[0], 4) for k, v in prof.items()}
        res["kernel_launches"] = {k: v[1] for k, v in prof.items()}
        res["gemm"] = {"launches": gcnt, "avg_us": gms / gcnt * 1e3, "bytes_per_launch": gbytes / gcnt,
                       "GBps": gbytes / (gms * 1e-3) / 1e9, "TFLOPs": gflops / (gms * 1e-3) / 1e12}
        # the gate/up projection alone (the dominant kernel): weights + live A rows + the bf16 activation it writes
        n_gu, k_gu = gemm_shapes(cfg)["gemm_gateup"]
        gu_bytes = sum(cfg.n_layers * (n_gu * k_gu * 2 + sb.real_tokens * k_gu * 2 + sb.real_tokens * (n_gu // 2) * 2)
                       for sb in staged)
        gu_ms, gu_cnt = prof["gemm_gateup"]
        res["gemm_gateup"] = {"launches": gu_cnt, "avg_us": gu_ms / gu_cnt * 1e3, "bytes_per_launch": gu_bytes / gu_cnt,
                              "GBps": gu_bytes / (gu_ms * 1e-3) / 1e9}
        # attention: K and V of every visible position are read once per layer (algorithmic bytes)
        kv_bytes = float(np.sum(b.new_len + b.prefix_len)) * cfg.n_kv_heads * cfg.head_dim * 2 * 2 * cfg.n_layers
        ams, acnt = prof["attn"]
        res["attention"] = {"launches": acnt, "avg_us": ams / max(acnt, 1) * 1e3, "kv_MB_per_launch": kv_bytes / max(acnt, 1) / 1e6,
                            "us_per_layer_batch": ams * 1e3 / (len(staged) * cfg.n_layers),
                            "kv_GBps": kv_bytes / (ams * 1e-3) / 1e9 if ams > 0 else None}
    sr.close()
    return res


# ------------------------------------------------------------------------------------- long prefill
def run_long(ctx, layers, cfg, steps, warmup):
    import numpy as np
    import torch
    from paper_2601_11589_amd import api, inputs, runner

    seed = inputs.SEED_BASE + 4
    b = inputs.make_batch(4)
    T = b.n_tokens
    d_x = torch.from_numpy(inputs.make_activations(cfg, seed, T)).cuda()
    out = torch.empty_like(d_x)
    k_pools, v_pools = ctx.new_pools(b.n_pages, cfg.n_layers)
    plan = api.laps_plan_buckets(64, LEN_BUCKETS, DEPTHS, 128, LONG_CHUNK, b.new_len, b.prefix_len)
    assert len(plan["longs"]) == b.n and not plan["batches"]
    ctx.workspace(LONG_CHUNK, 1)
    stream = torch.cuda.Stream()
    cu = b.cu_seqlens
    d_pt = torch.from_numpy(b.page_table).cuda()
    jobs = []
    for lg in plan["longs"]:
        i, done = lg["req_id"], 0
        for c in lg["chunks"]:
            jobs.append((i, done, c, torch.tensor([0, c], dtype=torch.int32, device="cuda"),
                         torch.tensor([done], dtype=torch.int32, device="cuda")))
            done += c

    def one_pass(events=None):
        for j, (i, done, c, d_cu, d_pre) in enumerate(jobs):
            lo = int(cu[i]) + done
            if events is not None and done == 0:
                events[i][0].record(stream)
            ctx.laps_prefill_stack(layers, d_cu, None, d_pre, d_pt[i:i + 1], k_pools, v_pools, d_x[lo:lo + c],
                                   out[lo:lo + c], stream)
            if events is not None and done + c == int(b.new_len[i]):
                events[i][1].record(stream)

    for _ in range(warmup):
        one_pass()
    stream.synchronize()
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(b.n)]
           for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        one_pass(evs[k])
    stream.synchronize()
    wall = time.perf_counter() - t0
    lat = [evs[k][i][0].elapsed_time(evs[k][i][1]) for k in range(steps) for i in range(b.n)]
    # algorithmic flops: GEMMs on real tokens + causal attention triangle
    gemm_fl = 2.0 * cfg.params_per_layer * T * cfg.n_layers
    att_fl = float(attn_flops(cfg, b.new_len, b.prefix_len)) * cfg.n_layers
    res = {"tokens_per_s": T * steps / wall, "ms_per_step": wall / steps * 1e3, "real_tokens": T,
           "chunk": LONG_CHUNK, "n_chunks": len(jobs), "latency_ms_p50": pct(lat, 50), "latency_ms_p90": pct(lat, 90),
           "algorithmic_TFLOP_per_step": (gemm_fl + att_fl) / 1e12,
           "stack_TFLOPs": (gemm_fl + att_fl) * steps / wall / 1e12,
           "stack_frac_of_mfma_peak": (gemm_fl + att_fl) * steps / wall / 1e12 / MFMA_BF16_PEAK_TFS}
    # per-kernel pass
    ctx.laps_prof_enable(True)
    one_pass()
    stream.synchronize()
    prof = ctx.laps_prof_read()
    ctx.laps_prof_enable(False)
    res["kernel_ms"] = {k: round(v[0], 3) for k, v in prof.items()}
    res["kernel_launches"] = {k: v[1] for k, v in prof.items()}
    n, kk = gemm_shapes(cfg)["gemm_gateup"]
    ms, cnt = prof["gemm_gateup"]
    fl = 2.0 * T * n * kk * cfg.n_layers          # all chunks of all prompts, real rows only
    res["roofline"] = {"bound": "mfma", "kernel": "gemm (gate/up projection, 256x256 tile)", "achieved": fl / (ms * 1e-3) / 1e12,
                       "peak": MFMA_BF16_PEAK_TFS, "unit": "TFLOP/s", "frac": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFS,
                       "traffic": None, "avg_launch_us": ms / cnt * 1e3, "launches": cnt}
    ms_all = sum(prof[k][0] for k in gemm_shapes(cfg))
    res["all_gemm_TFLOPs"] = gemm_fl / (ms_all * 1e-3) / 1e12
    ams, acnt = prof["attn"]
    res["attention_TFLOPs"] = att_fl / (ams * 1e-3) / 1e12 if ams > 0 else None
    return res


# ------------------------------------------------------------------------------------- latency model fit
def run_latency_model(layers, cfg):
    """Run-time fit of the compute / memory latency model (Section 2.1) on single-request passes."""
    from paper_2601_11589_amd import api, latency_fit
    new_lens, hist_lens = (16, 32, 64, 128, 256, 512, 1024, 2048), (0, 1024, 4096, 16384)
    ctx = api.LapsCtx(cfg, max_positions=max(new_lens) + max(hist_lens))
    samples = latency_fit.collect_samples(ctx, layers, new_lens, hist_lens)
    res = latency_fit.fit_and_boundaries(samples, cfg, len(layers), report_hist=hist_lens)
    res["samples"] = [{k: (round(v, 2) if isinstance(v, float) else v) for k, v in s.items()} for s in samples]
    ctx.close()
    return res


# ------------------------------------------------------------------------------------- graph cost table
def run_graph_cost(ctx32, layers32):
    """Capture time, device bytes and replay time of (length, depth) graphs over the paper's example grid
    (lengths 8..256, depths 1..64, Section 3.1) for 7B-, 14B- and 32B-shaped 4-layer stacks, beside the paper's
    cost analysis (a few hundred MB and seconds per graph on its stack)."""
    import numpy as np
    import torch
    from paper_2601_11589_amd import api, inputs
    lens, depths, budget = (8, 16, 32, 64, 128, 256), (1, 2, 4, 8, 16, 32, 64), 4096
    out = {"grid": {"len_buckets": lens, "depths": depths, "token_budget": budget}, "layers": 4, "models": {}}
    for name, cfgf in (("7B", inputs.qwen7b_cfg), ("14B", inputs.qwen14b_cfg), ("32B", inputs.qwen32b_cfg)):
        cfg = cfgf(4)
        if name == "32B":
            ctx, layers = ctx32, layers32
        else:
            ctx = api.LapsCtx(cfg, max_positions=4096)
            seed = inputs.SEED_BASE + 60 + len(name)
            layers = [ctx.upload_layer(inputs.make_layer_weights(cfg, seed, l, threads=min(16, os.cpu_count() or 8)))
                      for l in range(4)]
        log(f"[bench:graph-cost] {name}-shaped stack")
        max_pages = 16          # a 256-token request fills 16 pages
        k_pools, v_pools = ctx.new_pools(max_pages * 64 + 1, 4, zero=True)
        stream = torch.cuda.Stream()
        rows = []
        for lb in lens:
            for d in depths:
                if lb * d > budget:
                    continue
                t0 = time.perf_counter()
                g = ctx.laps_graph_capture(layers, lb, d, max_pages, k_pools, v_pools, stream)
                stream.synchronize()
                cap = time.perf_counter() - t0
                x = torch.zeros((d * lb, cfg.hidden), dtype=torch.float32, device="cuda")
                sl = torch.full((d,), lb, dtype=torch.int32, device="cuda")
                pl = torch.zeros(d, dtype=torch.int32, device="cuda")
                pt = (torch.arange(d * max_pages, dtype=torch.int32, device="cuda") + 1).reshape(d, max_pages).contiguous()
                # torch filled these on its default stream; `stream` does not wait for that stream by itself, and a
                # page table read before it is written holds whatever the allocator's block held before
                torch.cuda.synchronize()
                g.laps_graph_stage(d, sl, pl, pt, x, stream)
                g.laps_graph_replay(stream)
                stream.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(3):
                    g.laps_graph_replay(stream)
                e1.record(stream)
                e1.synchronize()
                rows.append((lb, d, cap, g.laps_graph_device_bytes(), e0.elapsed_time(e1) / 3))
                g.close()
        caps = np.array([r[2] for r in rows])
        mbs = np.array([r[3] for r in rows]) / 1e6
        out["models"][name] = {
            "graphs": len(rows), "capture_s": {"first": float(caps[0]), "median": float(np.median(caps)), "max": float(caps.max())},
            "device_MB": {"min": float(mbs.min()), "median": float(np.median(mbs)), "max": float(mbs.max()), "sum": float(mbs.sum())},
            "replay_ms": {f"{lb}x{d}": round(ms, 3) for lb, d, _, _, ms in rows if (lb, d) in ((8, 1), (16, 8), (64, 2), (64, 64), (256, 16))},
        }
        del k_pools, v_pools
        if name != "32B":
            ctx.close()
            del layers
            torch.cuda.empty_cache()
    return out


# ------------------------------------------------------------------------------------- spatial mode, simulated
def run_pool_sim(short_step_ms_4l, long_chunk_ms_4l, layers_full=64):
    """Algorithm 2 over 8 virtual instances of a full-depth model: queueing and the controller are simulated on the
    host, every step lasts what it was measured to last on this GPU (4-layer times scaled to `layers_full` layers).
    short_step_ms_4l: {depth: ms} of one (64-token bucket, depth) replay; long_chunk_ms_4l: ms of one 2048-token chunk."""
    import numpy as np
    from paper_2601_11589_amd import inputs, poolsim
    k = layers_full / 4.0
    depths = sorted(short_step_ms_4l)
    step = lambda d: 1e3 * k * float(np.interp(d, depths, [short_step_ms_4l[x] for x in depths]))
    chunk_us = 1e3 * k * long_chunk_ms_4l
    prm = poolsim.PoolSimParams()
    # capacities: a SHORT instance serves short_depth requests per step, a LONG one a 5120-token prompt in 2.5 chunks
    cap_s = prm.short_depth / (step(prm.short_depth) * 1e-6)
    cap_l = 1.0 / (2.5 * chunk_us * 1e-6)
    arr, ln, lg = poolsim.shifting_workload(inputs.SEED_BASE + 6, 60e6, short_rate_a=0.7 * 5 * cap_s, long_rate_a=0.3 * 3 * cap_l,
                                            short_rate_b=0.3 * 3 * cap_s, long_rate_b=0.7 * 5 * cap_l)
    out = {"instances": prm.n_total, "layers": layers_full, "short_step_us_depth8": step(prm.short_depth), "long_chunk_us": chunk_us,
           "requests": int(len(arr)), "phase_a": "short load 0.7 of 5 instances, long 0.3 of 3",
           "phase_b": "short load 0.3 of 3 instances, long 0.7 of 5"}
    for name, ctl in (("static_4_4", False), ("controller", True)):
        r = poolsim.simulate(arr, ln, lg, step, chunk_us, prm, controller=ctl)
        r.pop("moves")
        out[name] = r
    return out


# ------------------------------------------------------------------------------------- mixed dual-queue step loop
def run_dual_queue(ctx8, layers8, cfg8, windows_us, loads=(0.7,), params=None):
    """configs[4]: 4 long + 512 short / re-prefill requests on an 8-layer stack, Poisson arrivals replayed on a
    virtual clock that advances by measured GPU step time.  Unified FCFS mixed batches vs temporal disaggregation."""
    import numpy as np
    import torch
    from paper_2601_11589_amd import dualqueue, inputs

    seed = inputs.SEED_BASE + 5
    b = inputs.make_batch(5)
    d_x = torch.from_numpy(inputs.make_activations(cfg8, seed, b.n_tokens)).cuda()
    k_pools, v_pools = ctx8.new_pools(b.n_pages, cfg8.n_layers)
    gen = torch.Generator(device="cuda").manual_seed(seed)
    for p in k_pools + v_pools:      # cached prefix content: seeded N(0,1) bf16 drawn on the device (26 GB)
        p.copy_(torch.randn(p.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16))
    is_long = b.new_len > 64
    dq = dualqueue.DualQueue(ctx8, layers8, b.new_len, b.prefix_len, b.page_table, d_x, k_pools, v_pools,
                             params or dualqueue.DQParams())
    zeros = np.zeros(b.n)
    log("[bench:dual-queue] warm-up and back-to-back passes")
    dq.run_disaggregated(zeros, 0.0)          # warm-up: captures every bucket shape the workload needs
    dq.run_unified(zeros)
    dq.run_unified(zeros, budget=WHOLE_PROMPT_BUDGET)
    u0 = dq.run_unified(zeros)
    d0 = dq.run_disaggregated(zeros, 0.0)
    # algorithmic flops of the whole workload: projections on real tokens + causal attention over prefix and new tokens
    total_flops = (2.0 * cfg8.params_per_layer * b.n_tokens + float(attn_flops(cfg8, b.new_len, b.prefix_len))) * cfg8.n_layers

    def summ(r, extra=None):
        sm = r.summary(b.new_len, is_long)
        sm["mfma_frac_of_peak_while_busy"] = total_flops / (r.gpu_busy_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFS
        if extra:
            sm.update(extra)
        return sm

    res = {"requests": int(b.n), "real_tokens": int(b.n_tokens), "layers": cfg8.n_layers,
           "algorithmic_TFLOP": total_flops / 1e12,
           "back_to_back": {"unified": summ(u0), "unified_whole_prompts": summ(dq.run_unified(zeros, budget=WHOLE_PROMPT_BUDGET)),
                            "disaggregated": summ(d0)}, "poisson": []}
    s_hat = d0.step_kinds["short_busy_us"] / max(d0.step_kinds["short_graph"], 1)   # mean short step, measured
    dq.run_awd(zeros)                          # warm-up: captures the fused shapes AWD dispatches
    res["back_to_back"]["awd"] = summ(dq.run_awd(zeros, s_hat_us=s_hat))
    longs = np.nonzero(is_long)[0]
    for ld in loads:
        log(f"[bench:dual-queue] load {ld}")
        rate = ld * b.n / (u0.makespan_us * 1e-6)
        arr = inputs.poisson_arrivals_us(seed, b.n, rate).astype(np.float64)
        horizon = float(arr.max())
        for j, i in enumerate(longs):        # long requests are spread uniformly over the arrival horizon
            arr[i] = horizon * j / len(longs)
        tag = {"load": ld, "arrival_rate_per_s": rate}
        res["poisson"].append(summ(dq.run_unified(arr), tag))
        # memory-based batching without chunks (Section 2.3): a long prompt enters whole, short requests ride behind it
        res["poisson"].append(summ(dq.run_unified(arr, budget=WHOLE_PROMPT_BUDGET), tag))
        for w in (windows_us if ld == loads[len(loads) // 2] else windows_us[1:2]):   # full window sweep at the middle load
            res["poisson"].append(summ(dq.run_disaggregated(arr, float(w)), tag))
        # Adaptive-Wait-Depth batching of the short queue (Algorithm 1): deadline-free, then with a 50 ms TTFT deadline
        res["poisson"].append(summ(dq.run_awd(arr, s_hat_us=s_hat, w_max_us=10_000.0), tag))
        ddl = arr + 50_000.0
        r = dq.run_awd(arr, ddl_us=ddl, s_hat_us=s_hat, sigma_us=2_000.0, w_max_us=10_000.0, t_max_us=25_000.0,
                       delta_us=1_000.0, sla_window=True)
        res["poisson"].append(summ(r, dict(tag, short_deadline_50ms_met_frac=float(np.mean(r.latency_us[~is_long] <= 50_000.0)))))
    dq.close()
    del k_pools, v_pools
    return res


# ------------------------------------------------------------------------------------- oracle on host cores
def cpu_baseline(cfg, host_layers, n_sample_req=24, n_layers=None):
    """fp64 oracle, as it stands, on the first requests of the short workload; all host cores BLAS uses."""
    import numpy as np
    from oracle import laps_oracle as O
    from paper_2601_11589_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    n_layers = n_layers or cfg.n_layers
    b = inputs.make_batch(2)
    lens = [int(v) for v in b.new_len[:n_sample_req]]
    T = sum(lens)
    x = inputs.make_activations(cfg, inputs.SEED_BASE + 2, b.n_tokens)[:T].astype(np.float64)

    class Lazy:
        def __len__(self):
            return n_layers

        def __getitem__(self, i):
            return {k: inputs.bf16_bits_to_f64(v) for k, v in host_layers[i].items()}

    t0 = time.perf_counter()
    O.stack_forward(cfg, Lazy(), x, lens)
    dt = time.perf_counter() - t0
    return {"value": T / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n_sample_req} requests ({T} tokens) of the short-bucket workload through all "
                      f"{n_layers} layers, numpy float64 (weights widened from bf16 inside the timed region), {dt:.1f}s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--token-budget", type=int, default=128, help="padded tokens per captured short graph")
    ap.add_argument("--no-long", action="store_true", help="skip the long-prefill workload")
    ap.add_argument("--no-token-max", action="store_true", help="skip the token-max variant of the short workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-dual-queue", action="store_true", help="skip the mixed dual-queue workload (configs[4])")
    ap.add_argument("--no-latency-model", action="store_true", help="skip the run-time latency-model fit")
    ap.add_argument("--no-reprefill", action="store_true", help="skip the multi-turn re-prefill workload (configs[2])")
    ap.add_argument("--no-graph-cost", action="store_true", help="skip the graph capture cost table (7B/14B/32B shapes)")
    ap.add_argument("--windows-us", type=str, default="0,500,1000,2000,10000", help="waiting windows (us) for the dual-queue sweep")
    ap.add_argument("--budget-sweep", type=str, default="256,512,1024",
                    help="further token budgets for the short workload (tokens/s against latency); empty = none")
    ap.add_argument("--no-two-streams", action="store_true",
                    help="short buckets: skip the variant that alternates the replays between two streams")
    ap.add_argument("--loads", type=str, default="0.7",
                    help="dual queue: Poisson arrival rates as fractions of the unified back-to-back service rate")
    ap.add_argument("--long-steps", type=int, default=2)
    ap.add_argument("--no-reprefill-token-max", action="store_true",
                    help="skip the token-budget-4096 variant of the re-prefill workload")
    ap.add_argument("--detail-file", type=str, default="bench_detail.json",
                    help="file under gpurun_out/ that receives the full record (per-shape tables, samples, trajectories)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (known size) so that rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "readings of the same run can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (replicas are independent copies of the whole model); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_11589_amd import api, inputs
    api.lib()                                           # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    props = torch.cuda.get_device_properties(0)
    log(f"[bench] device {props.name}, {props.multi_processor_count} CUs, {props.total_memory / 2**30:.0f} GiB; "
        f"peaks used: HBM {HBM_PEAK_GBS} GB/s, bf16 MFMA {MFMA_BF16_PEAK_TFS} TFLOP/s")
    if args.calibrate_copy:
        src = torch.ones(256 * 2**20 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] calibration: 5 plain device copies of 268435456 bytes (read) + 268435456 bytes (write) each")
        del src, dst
    cfg = inputs.qwen32b_cfg(4)
    n_build = 4 if args.no_dual_queue else 8
    ctx, layers_all, host_layers = build_model(cfg, inputs.SEED_BASE + 2, n_build)
    layers = layers_all[:4]

    log("[bench] leg: short buckets (configs[1])")
    short = run_short(ctx, layers, cfg, args.token_budget, args.steps, args.warmup, True, "short",
                      two_streams=not args.no_two_streams)
    g = short.pop("gemm")
    gu = short.pop("gemm_gateup")
    detail = {"short": short, "short_all_gemms": g}
    traffic = load_traffic("gemm_gateup_skinny") if args.token_budget == 128 else None
    weights_bytes = 2.0 * cfg.params_per_layer * cfg.n_layers          # bf16 weights streamed once per replay
    replay_ms = short["ms_per_step"] / short["n_batches"]
    line = {
        "metric": METRIC, "value": short["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": short["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: 256 new prompts U[8,64], buckets {16,32,64}, 4-layer Qwen2.5-32B-shaped "
                               f"stack, hipGraph per (bucket, depth), token_budget {args.token_budget}",
                   "layers": cfg.n_layers, "requests": 256, "token_budget": args.token_budget,
                   "batches_per_step": short["n_batches"]},
        "latency_ms": {"p50": short["latency_ms_p50"], "p90": short["latency_ms_p90"]},
        # the dominant kernel: the gate/up projection with the fused SwiGLU epilogue on the streaming tile
        "roofline": {"bound": "hbm", "kernel": "gemm_kernel<128,256,2,4,2,2> (gate/up + SwiGLU)",
                     "achieved": gu["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gu["GBps"] / HBM_PEAK_GBS,
                     "traffic": traffic, "avg_launch_us": gu["avg_us"], "bytes_per_launch": gu["bytes_per_launch"],
                     "launches": gu["launches"]},
        "roofline_all_gemms": {"achieved": g["GBps"], "unit": "GB/s", "frac": g["GBps"] / HBM_PEAK_GBS,
                               "avg_launch_us": g["avg_us"], "launches": g["launches"]},
        # whole replay (all kernels, staging and gaps) against the weights it must stream once
        "roofline_per_replay": {"bytes": weights_bytes, "ms": replay_ms,
                                "achieved": weights_bytes / (replay_ms * 1e-3) / 1e9, "unit": "GB/s",
                                "frac": weights_bytes / (replay_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if "two_streams" in short:
        line["short_two_streams_tokens_per_s"] = short["two_streams"]["tokens_per_s"]
    if not args.no_token_max:
        log("[bench] leg: short buckets, token-max")
        tm = run_short(ctx, layers, cfg, 4096, max(2, args.steps // 2), 1, True, "token-max")
        gm = tm.pop("gemm")
        tm.pop("gemm_gateup")
        tm["gemm_TFLOPs"] = gm["TFLOPs"]
        tm["gemm_frac_of_mfma_peak"] = gm["TFLOPs"] / MFMA_BF16_PEAK_TFS
        detail["short_token_max"] = tm
        line["short_token_max"] = {"tokens_per_s": tm["tokens_per_s"], "latency_ms_p50": tm["latency_ms_p50"],
                                   "gemm_frac_of_mfma_peak": tm["gemm_frac_of_mfma_peak"]}
    if not args.no_token_max and args.budget_sweep:
        # the same short workload at token budgets between the latency-oriented default and token-max
        log("[bench] leg: short buckets, token budget sweep")
        sweep = {}
        for tb in (int(x) for x in args.budget_sweep.split(",")):
            r = run_short(ctx, layers, cfg, tb, max(2, args.steps // 2), 1, False, f"budget-{tb}")
            sweep[str(tb)] = {k: r[k] for k in ("tokens_per_s", "ms_per_step", "n_batches", "latency_ms_p50", "latency_ms_p90")}
        detail["short_budget_sweep"] = sweep
    if not args.no_reprefill:
        # configs[2]: multi-turn re-prefill, 128 requests of U[16,64] new tokens over U[512,4096] cached tokens
        log("[bench] leg: re-prefill (configs[2])")
        rp = run_short(ctx, layers, cfg, args.token_budget, max(2, args.steps // 2), 1, True, "re-prefill", config=3)
        rp.pop("gemm")
        rp.pop("gemm_gateup")
        detail["reprefill"] = rp
        line["reprefill"] = {"tokens_per_s": rp["tokens_per_s"], "latency_ms_p50": rp["latency_ms_p50"],
                             "latency_ms_p90": rp["latency_ms_p90"], "attn_kv_GBps": rp["attention"]["kv_GBps"],
                             "attn_us_per_layer": rp["attention"]["us_per_layer_batch"]}
        if not args.no_reprefill_token_max:
            log("[bench] leg: re-prefill, token-max")
            rp2 = run_short(ctx, layers, cfg, 4096, max(2, args.steps // 2), 1, True, "re-prefill-4096", config=3)
            rp2.pop("gemm")
            rp2.pop("gemm_gateup")
            detail["reprefill_token_max"] = rp2
            line["reprefill_token_max"] = {"tokens_per_s": rp2["tokens_per_s"], "latency_ms_p50": rp2["latency_ms_p50"],
                                           "attn_kv_GBps": rp2["attention"]["kv_GBps"]}
    if not args.no_long:
        log("[bench] leg: long prefill (configs[3])")
        lp = run_long(ctx, layers, cfg, args.long_steps, 1)
        detail["long_prefill"] = lp
        line["long_prefill"] = {"tokens_per_s": lp["tokens_per_s"], "ms_per_step": lp["ms_per_step"],
                                "latency_ms_p50": lp["latency_ms_p50"], "latency_ms_p90": lp["latency_ms_p90"],
                                "roofline": {k: lp["roofline"][k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "avg_launch_us")},
                                "all_gemm_TFLOPs": lp["all_gemm_TFLOPs"], "attention_TFLOPs": lp["attention_TFLOPs"],
                                "stack_frac_of_mfma_peak": lp["stack_frac_of_mfma_peak"]}
    if not args.no_latency_model:
        log("[bench] leg: latency model fit")
        lm = run_latency_model(layers, cfg)
        detail["latency_model"] = lm
        line["latency_model"] = {k: lm[k] for k in ("alpha", "beta", "gamma_w", "gamma_r", "weight_floor_us") if k in lm}
        line["latency_model"]["knee_tokens_H0"] = lm["knee_library"]["0"]
        line["latency_model"]["derived"] = {k: lm["derived"][k] for k in ("short_max_len", "short_token_budget", "fuse_budget")}
        log(f"[bench] schedule parameters from the fit: {line['latency_model']['derived']}")
    if not args.no_graph_cost:
        log("[bench] leg: graph cost table")
        detail["graph_cost"] = run_graph_cost(ctx, layers)
        if "long_prefill" in detail:
            gc = detail["graph_cost"]["models"]["32B"]["replay_ms"]
            lp = detail["long_prefill"]
            detail["pool_sim"] = run_pool_sim({2: gc["64x2"], 64: gc["64x64"]}, lp["ms_per_step"] / lp["n_chunks"])
    if not args.no_dual_queue:
        cfg8 = inputs.qwen32b_cfg(8)
        log("[bench] leg: dual queue (configs[4])")
        ctx8 = api.LapsCtx(cfg8, max_positions=8192 + 64)
        dq_params = None
        if "latency_model" in detail:
            # Section 2.1 "runtime fitting": classification boundary and fusion budget come from this run's fit
            from paper_2601_11589_amd import dualqueue
            lm = detail["latency_model"]
            dq_params = dualqueue.DQParams.from_fit((lm["alpha"], lm["beta"], lm["gamma_w"], lm["gamma_r"]),
                                                    lm["weight_floor_us"], 4096.0, tuple(LEN_BUCKETS), tuple(DEPTHS))
            log(f"[bench] dual queue runs with short_max_len {dq_params.short_max_len}, fuse budget {dq_params.fuse_budget}")
        dq = run_dual_queue(ctx8, layers_all, cfg8, [float(w) for w in args.windows_us.split(",")],
                            tuple(float(x) for x in args.loads.split(",")), dq_params)
        ctx8.close()
        detail["dual_queue"] = dq
        line["dual_queue"] = {"load": dq["poisson"][0].get("load") if dq["poisson"] else None,
                              "policies": [{"mode": r["mode"], "makespan_ms": round(r["makespan_ms"], 1),
                                            "short_p50_p90_ms": [round(r["short_latency_ms"][q], 2) for q in ("p50", "p90")],
                                            "long_p50_p90_ms": [round(r["long_latency_ms"][q], 1) for q in ("p50", "p90")]}
                                           for r in dq["poisson"]]}
    if not args.no_cpu:
        log("[bench] leg: oracle on host cores")
        line["cpu_baseline"] = cpu_baseline(cfg, host_layers[:4], n_sample_req=96)
    else:
        line["cpu_baseline"] = None
    # everything bulky (per-shape tables, samples, trajectories) goes to a side file; stdout carries one compact line
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    detail_path = os.path.join(ROOT, "gpurun_out", args.detail_file)
    with open(detail_path, "w") as f:
        json.dump({"line": line, "detail": detail}, f)
    line["detail_file"] = os.path.relpath(detail_path, ROOT)
    out = json.dumps(line, separators=(",", ":"), default=float)
    log(f"[bench] result line: {len(out)} bytes; full record in {line['detail_file']}")
    print(out, flush=True)


if __name__ == "__main__":
    main()
