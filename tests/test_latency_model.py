"""Latency model (Section 2.1): the oracle against hand-worked values and limits, the library against the oracle."""
import math

import numpy as np
import pytest

from oracle import latency_oracle as LO
from paper_2601_11589_amd import api


def test_oracle_hand_worked_boundaries():
    # prefill: (gamma_w - beta) / alpha = (10 - 2) / 1 = 8 ; compute-bound from the start if gamma_w <= beta
    assert LO.boundary(1.0, 2.0, 10.0, 3.0, 0.0) == pytest.approx(8.0, abs=1e-12)
    assert LO.boundary(1.0, 12.0, 10.0, 3.0, 0.0) == 0.0
    # re-prefill, alpha=1 beta=2 gamma_w=10 gamma_r=3 H=4: the linear coefficient 2*1*4 + 2 - 10 vanishes,
    # so L^2 = gamma_r H = 12 and L = sqrt(12)
    assert LO.boundary(1.0, 2.0, 10.0, 3.0, 4.0) == pytest.approx(math.sqrt(12.0), abs=1e-12)
    # alpha=0.5 beta=1 gamma_w=2 gamma_r=6 H=1: 0.5 L^2 + 0 L - 6 = 0 -> L = sqrt(12)
    assert LO.boundary(0.5, 1.0, 2.0, 6.0, 1.0) == pytest.approx(math.sqrt(12.0), abs=1e-12)
    # the two costs are equal at the boundary, compute below memory just under it
    a, b, gw, gr, H = 0.003, 0.7, 1.1, 0.05, 900.0
    Lm = LO.boundary(a, b, gw, gr, H)
    assert LO.t_comp(a, b, Lm, H) == pytest.approx(LO.t_mem(gw, gr, Lm, H), rel=1e-10)
    assert LO.t_comp(a, b, 0.9 * Lm, H) < LO.t_mem(gw, gr, 0.9 * Lm, H)
    # saturation for long histories: gamma_r / (2 alpha)
    assert LO.boundary(a, b, gw, gr, 1e9) == pytest.approx(gr / (2 * a), rel=1e-5)


def test_library_closed_forms_match_oracle():
    rng = np.random.default_rng(11589)
    for _ in range(300):
        a, b, gw, gr = rng.uniform(1e-4, 2), rng.uniform(0, 5), rng.uniform(0, 8), rng.uniform(0, 4)
        H = float(rng.choice([0, 1, 17, 512, 4096, 1e6]))
        want = LO.boundary(a, b, gw, gr, H)
        got = api.laps_lm_boundary_reprefill(a, b, gw, gr, H)
        assert got == pytest.approx(want, rel=1e-9, abs=1e-9)
        if H == 0:
            assert api.laps_lm_boundary_prefill(a, b, gw) == pytest.approx(want, rel=1e-12, abs=1e-12)
    assert math.isnan(api.laps_lm_boundary_prefill(0.0, 1.0, 2.0))
    assert math.isnan(api.laps_lm_boundary_reprefill(1.0, 1.0, 2.0, 1.0, -1.0))


def test_library_fit_matches_lstsq_and_recovers_planted_coefficients():
    rng = np.random.default_rng(7)
    L = rng.integers(1, 300, 80).astype(float)
    H = rng.integers(0, 5000, 80).astype(float)
    a, b, gw, gr = 2e-3, 0.9, 1.4, 0.02
    tc = LO.t_comp(a, b, L, H)
    tm = LO.t_mem(gw, gr, L, H)
    got = api.laps_lm_fit(L, H, tc, tm)
    assert got == pytest.approx((a, b, gw, gr), rel=1e-8)
    tc_n = tc * (1 + 0.05 * rng.standard_normal(80))
    tm_n = tm * (1 + 0.05 * rng.standard_normal(80))
    assert api.laps_lm_fit(L, H, tc_n, tm_n) == pytest.approx(LO.fit(L, H, tc_n, tm_n), rel=1e-8)
    with pytest.raises(api.LapsError):
        api.laps_lm_fit(L, 2 * L, tc, tm)            # H proportional to L: gamma_w and gamma_r not separable
    with pytest.raises(api.LapsError):
        api.laps_lm_fit(L[:1], H[:1], tc[:1], tm[:1])
    half = api.laps_lm_fit(L, H, t_mem=tm)                 # one half only: the other pair is not touched
    assert math.isnan(half[0]) and math.isnan(half[1]) and half[2:] == pytest.approx((gw, gr), rel=1e-8)
    with pytest.raises(api.LapsError):
        api.laps_lm_fit(L, H)


def test_fit_and_boundaries_on_planted_samples():
    """The sample post-processing (no GPU needed): planted coefficients come back, the reported boundaries are the
    oracle's roots, and the knee with a constant weight-streaming floor solves its own balance equation."""
    from paper_2601_11589_amd import inputs, latency_fit
    cfg = inputs.qwen32b_cfg(4)
    a, b, gw, gr, floor = 6e-5, 3.7, 0.03, 0.017, 740.0
    samples = []
    for H in (0, 1024, 4096, 16384):
        for L in (16, 32, 64, 128, 256, 512, 1024, 2048):
            gemm, attn = max(floor, b * L), a * L * (L + 2 * H)
            samples.append(dict(L=L, H=H, t_comp_us=gemm + attn, gemm_us=gemm, attn_us=attn, t_mem_us=gw * L + gr * H,
                                kv_write_us=gw * L, kv_read_us=gr * H, stack_us=gemm + attn))
    r = latency_fit.fit_and_boundaries(samples, cfg, 4)
    assert (r["alpha"], r["beta"], r["gamma_w"], r["gamma_r"]) == pytest.approx((a, b, gw, gr), rel=2e-3)
    assert r["L_m_prefill"] == LO.boundary(r["alpha"], r["beta"], r["gamma_w"], r["gamma_r"], 0.0) == 0.0
    for h, v in r["L_m_reprefill"].items():
        assert v == pytest.approx(LO.boundary(r["alpha"], r["beta"], r["gamma_w"], r["gamma_r"], float(h)), rel=1e-9)
    assert r["L_m_reprefill_limit"] == pytest.approx(gr / (2 * a), rel=5e-3)
    assert r["weight_floor_us"] == floor
    for h, knee in r["knee_with_weight_floor"].items():
        H = float(h)
        comp = r["alpha"] * knee * (knee + 2 * H) + r["beta"] * knee
        mem = r["gamma_w"] * knee + r["gamma_r"] * H + floor
        assert comp == pytest.approx(mem, rel=1e-9)
    assert 150 < r["knee_with_weight_floor"]["0"] < 250
