"""Run-time samples for the compute / memory latency model and the boundaries that follow from them.

Section 2.1 of the paper models one (re-)prefill of L new tokens over H historical tokens as
T_comp = alpha L (L + 2H) + beta L (attention and projection / FFN arithmetic) plus T_mem = gamma_w L + gamma_r H
(KV-cache write and read), fits the four coefficients from run-time samples and derives the length below
which the request is memory-bound.  The paper does not say how a sample separates the two terms; here

  * T_comp(L, H) is the time of the matrix-core kernels (four projections per layer and attention) of one
    single-request pass through the stack, taken from the library's per-kernel-class event timers, over
    the samples with L >= `comp_min_len`, where those kernels are arithmetic-bound;
  * T_mem(L, H) is the time the paged-KV kernels need to write L tokens and to read H tokens of every layer.

The paper's memory term has no constant for streaming the weights once per pass, which is what bounds a
short batch on this GPU; `weight_floor_us` (the projection time of the smallest L) is reported beside the
fit, with the knee it implies: the positive root of alpha L^2 + (beta - gamma_w) L - (floor + gamma_r H) = 0.
The arithmetic-intensity reading of the same section (boundary where AI(L) reaches P_peak / B_mem) is
reported from the sustained rates measured in the same run.
All arithmetic on the samples happens in the library (laps_lm_fit, laps_lm_boundary_*).
"""
from __future__ import annotations

import numpy as np
import torch

from . import api

GEMM_CLASSES = ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down")


def _time_us(stream, fn, reps):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    stream.synchronize()
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def collect_samples(ctx: api.LapsCtx, layers, new_lens, hist_lens, reps: int = 3):
    """One single-request pass per (L, H).  Returns a list of dicts with times in microseconds."""
    cfg = ctx.cfg
    n_layers = len(layers)
    max_pos = max(new_lens) + max(hist_lens)
    n_pages = (max_pos + 15) // 16 + 1
    k_pools, v_pools = ctx.new_pools(n_pages, n_layers, zero=True)
    stream = torch.cuda.Stream()
    pt = torch.arange(n_pages, dtype=torch.int32, device="cuda").reshape(1, -1).contiguous()
    gen = torch.Generator(device="cuda").manual_seed(115890)
    x_all = torch.randn((max(new_lens), cfg.hidden), generator=gen, device="cuda", dtype=torch.float32)
    kv_src = torch.randn((max(max(new_lens), 1), cfg.n_kv_heads, cfg.head_dim), generator=gen, device="cuda",
                         dtype=torch.float32).to(torch.bfloat16)
    ctx.workspace(max(new_lens), 1)
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = []
    for H in hist_lens:
        for L in new_lens:
            cu = torch.tensor([0, L], dtype=torch.int32, device="cuda")
            pre = torch.tensor([H], dtype=torch.int32, device="cuda")
            x = x_all[:L]
            y = torch.empty_like(x)
            torch.cuda.synchronize()
            run = lambda: ctx.laps_prefill_stack(layers, cu, None, pre, pt, k_pools, v_pools, x, y, stream)
            run()
            stream.synchronize()
            ctx.laps_prof_enable(True)
            for _ in range(reps):
                run()
            stream.synchronize()
            prof = ctx.laps_prof_read()
            ctx.laps_prof_enable(False)
            gemm_us = sum(prof[k][0] for k in GEMM_CLASSES) * 1e3 / reps
            attn_us = prof["attn"][0] * 1e3 / reps
            total_us = _time_us(stream, run, reps)
            # KV I/O alone: write L tokens at position H, read H tokens from position 0, every layer
            def kv_write():
                for l in range(n_layers):
                    ctx.laps_kv_scatter(cu, pre, pt, kv_src[:L], kv_src[:L], k_pools[l], v_pools[l], stream)
            w_us = _time_us(stream, kv_write, reps)
            r_us = 0.0
            if H > 0:
                cu_h = torch.tensor([0, H], dtype=torch.int32, device="cuda")
                def kv_read():
                    for l in range(n_layers):
                        ctx.laps_kv_gather(cu_h, zero, pt, k_pools[l], v_pools[l], H, stream)
                r_us = _time_us(stream, kv_read, reps)
            out.append({"L": L, "H": H, "t_comp_us": gemm_us + attn_us, "gemm_us": gemm_us, "attn_us": attn_us,
                        "t_mem_us": w_us + r_us, "kv_write_us": w_us, "kv_read_us": r_us, "stack_us": total_us})
    return out


def fit_and_boundaries(samples, cfg, n_layers: int, comp_min_len: int = 256, report_hist=(0, 1024, 4096, 16384),
                       len_buckets=(16, 32, 64), depths=(1, 2, 4, 8, 16, 32, 64)):
    comp = [s for s in samples if s["L"] >= comp_min_len]
    L = np.array([s["L"] for s in comp], np.float64)
    H = np.array([s["H"] for s in comp], np.float64)
    tc = np.array([s["t_comp_us"] for s in comp])
    alpha, beta, _, _ = api.laps_lm_fit(L, H, t_comp=tc)
    La = np.array([s["L"] for s in samples], np.float64)
    Ha = np.array([s["H"] for s in samples], np.float64)
    tm = np.array([s["t_mem_us"] for s in samples])
    _, _, gamma_w, gamma_r = api.laps_lm_fit(La, Ha, t_mem=tm)
    pred = alpha * L * (L + 2 * H) + beta * L
    r2_c = 1.0 - float(np.sum((tc - pred) ** 2) / np.sum((tc - tc.mean()) ** 2))
    predm = gamma_w * La + gamma_r * Ha
    r2_m = 1.0 - float(np.sum((tm - predm) ** 2) / np.sum((tm - tm.mean()) ** 2))
    l_min = min(s["L"] for s in samples)
    floor = float(np.mean([s["gemm_us"] for s in samples if s["L"] == l_min]))
    res = {"unit": "us", "layers": n_layers, "alpha": alpha, "beta": beta, "gamma_w": gamma_w, "gamma_r": gamma_r,
           "r2_comp": r2_c, "r2_mem": r2_m, "comp_min_len": comp_min_len,
           "L_m_prefill": api.laps_lm_boundary_prefill(alpha, beta, gamma_w),
           "L_m_reprefill": {str(h): api.laps_lm_boundary_reprefill(alpha, beta, gamma_w, gamma_r, float(h))
                             for h in report_hist if h > 0},
           "L_m_reprefill_limit": gamma_r / (2 * alpha) if alpha > 0 else None,
           "weight_floor_us": floor}
    # knee with the weight-streaming floor as a constant memory term (extension, see module docstring):
    # alpha L^2 + (2 alpha H + beta - gamma_w) L - (floor + gamma_r H) = 0 is the re-prefill quadratic with
    # gamma_r H replaced by floor + gamma_r H; for H = 0 the library's form is reused with hist 1, gamma_r = floor
    knee = {}
    for h in report_hist:
        if h == 0:
            # 2*alpha*1 shift is negligible against beta; exact form: solve with H=1 and beta' = beta - 2 alpha
            knee["0"] = api.laps_lm_boundary_reprefill(alpha, beta - 2 * alpha, gamma_w, floor, 1.0)
        else:
            knee[str(h)] = api.laps_lm_boundary_reprefill(alpha, beta, gamma_w, gamma_r + floor / h, float(h))
    res["knee_with_weight_floor"] = knee
    res["knee_library"] = {str(h): api.laps_lm_knee(alpha, beta, gamma_w, gamma_r, floor, float(h)) for h in report_hist}
    # what the schedule takes from this fit (classification boundary, latency-mode token budget, fusion budget)
    res["derived"] = api.laps_lm_derive_params((alpha, beta, gamma_w, gamma_r), floor, float(max(report_hist)),
                                               list(len_buckets), list(depths))
    # arithmetic-intensity reading: projections do 2 flops per parameter per token over 2 bytes per parameter,
    # AI(L) = L flop/byte; the boundary is AI* = P_sustained / B_sustained
    big = max(samples, key=lambda s: (s["L"], -s["H"]))
    small = min(samples, key=lambda s: (s["L"], s["H"]))
    flops_tok = 2.0 * cfg.params_per_layer * n_layers
    p_sus = flops_tok * big["L"] / (big["gemm_us"] * 1e-6)
    b_sus = cfg.params_per_layer * n_layers * 2.0 / (small["gemm_us"] * 1e-6)
    res["roofline_reading"] = {"P_sustained_TFLOPs": p_sus / 1e12, "B_sustained_GBs": b_sus / 1e9,
                               "AI_star_tokens": p_sus / b_sus}
    return res
