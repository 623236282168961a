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


def test_oracle_knee_with_weight_floor_hand_worked():
    # alpha=1 beta=2 gamma_w=10 gamma_r=3 H=4: the linear coefficient 2*1*4 + 2 - 10 vanishes: L^2 = floor + gamma_r H = 9 + 12
    assert LO.knee(1.0, 2.0, 10.0, 3.0, 9.0, 4.0) == pytest.approx(math.sqrt(21.0), abs=1e-12)
    # H=0, beta = gamma_w: alpha L^2 = floor -> L = sqrt(floor / alpha) = sqrt(9 / 4)
    assert LO.knee(4.0, 7.0, 7.0, 1.0, 9.0, 0.0) == pytest.approx(1.5, abs=1e-12)
    # H=0, alpha=2 beta=5 gamma_w=1 floor=6: 2 L^2 + 4 L - 6 = 0 -> L = 1
    assert LO.knee(2.0, 5.0, 1.0, 0.3, 6.0, 0.0) == pytest.approx(1.0, abs=1e-12)
    # no floor: the printed re-prefill boundary
    for H in (0.0, 5.0, 900.0):
        assert LO.knee(0.003, 0.7, 1.1, 0.05, 0.0, H) == pytest.approx(LO.boundary(0.003, 0.7, 1.1, 0.05, H), rel=1e-12, abs=1e-12)
    # both sides of the balance are equal at the knee
    a, b, gw, gr, fl, H = 6e-5, 3.6, 0.1, 0.02, 700.0, 4096.0
    L = LO.knee(a, b, gw, gr, fl, H)
    assert LO.t_comp(a, b, L, H) == pytest.approx(fl + LO.t_mem(gw, gr, L, H), rel=1e-10)
    assert 150 < L < 250        # the order of magnitude measured on MI355X


def test_oracle_derived_parameters_hand_worked():
    grid = ([16, 32, 64], [1, 2, 4, 8, 16, 32, 64])
    mk = lambda k: (1.0, 0.0, 0.0, 0.0)     # alpha=1, everything else 0, no history: L^2 = floor, knee = sqrt(floor)
    # knee 200: longest bucket 64 fits; shapes within 200 padded tokens: 128 = 64x2 = 32x4 = 16x8 is the largest
    assert LO.derive_params(mk(0), 200.0 ** 2, 0.0, *grid) == {"short_max_len": 64, "short_token_budget": 128, "fuse_budget": 128}
    # knee 100: 64 still fits, largest shape 64 (96 is not a product of the grid)
    assert LO.derive_params(mk(0), 100.0 ** 2, 0.0, *grid) == {"short_max_len": 64, "short_token_budget": 64, "fuse_budget": 64}
    # knee 40: only the 16- and 32-token buckets are short; shapes 32 = 32x1 = 16x2
    assert LO.derive_params(mk(0), 40.0 ** 2, 0.0, *grid) == {"short_max_len": 32, "short_token_budget": 32, "fuse_budget": 32}
    # knee 10: below the smallest bucket - one request of that bucket
    assert LO.derive_params(mk(0), 10.0 ** 2, 0.0, *grid) == {"short_max_len": 16, "short_token_budget": 16, "fuse_budget": 16}
    # the paper's wider example grid, knee 300: bucket 256 fits, 256x1 = 128x2 = ... is the largest shape
    wide = ([8, 16, 32, 64, 128, 256], [1, 2, 4, 8, 16, 32, 64])
    assert LO.derive_params(mk(0), 300.0 ** 2, 0.0, *wide) == {"short_max_len": 256, "short_token_budget": 256, "fuse_budget": 256}
    # a long history lowers the knee (each new token also attends to H cached ones) and the lower one decides:
    # alpha=0.01 beta=1 floor=300: knee(0) = root of 0.01 L^2 + L - 300 = 131.7; knee(H=1000) with 2 alpha H = 20:
    # 0.01 L^2 + 21 L - 300 = 0 -> 14.2: only the 8-token bucket of the wide grid is short there
    p = LO.derive_params((0.01, 1.0, 0.0, 0.0), 300.0, 1000.0, *wide)
    assert p == {"short_max_len": 8, "short_token_budget": 8, "fuse_budget": 8}


def test_library_knee_and_derived_parameters_match_oracle():
    rng = np.random.default_rng(2601)
    grids = [([16, 32, 64], [1, 2, 4, 8, 16, 32, 64]), ([8, 16, 32, 64, 128, 256], [1, 2, 4, 8, 16, 32, 64]), ([24, 40], [1, 3, 5])]
    for _ in range(400):
        a, b, gw, gr = 10 ** rng.uniform(-6, 0), rng.uniform(0, 5), rng.uniform(0, 8), rng.uniform(0, 1)
        fl = float(rng.choice([0.0, 1.0, 50.0, 700.0, 1e4]))
        H = float(rng.choice([0, 1, 17, 512, 4096, 16384]))
        assert api.laps_lm_knee(a, b, gw, gr, fl, H) == pytest.approx(LO.knee(a, b, gw, gr, fl, H), rel=1e-9, abs=1e-9)
        lbs, dps = grids[int(rng.integers(len(grids)))]
        got = api.laps_lm_derive_params((a, b, gw, gr), fl, H, lbs, dps)
        want = LO.derive_params((a, b, gw, gr), fl, H, lbs, dps)
        assert {k: got[k] for k in want} == want, (a, b, gw, gr, fl, H, got, want)
        assert got["knee_fresh"] == pytest.approx(LO.knee(a, b, gw, gr, fl, 0.0), rel=1e-9, abs=1e-9)
    assert math.isnan(api.laps_lm_knee(0.0, 1.0, 1.0, 1.0, 1.0, 0.0)) and math.isnan(api.laps_lm_knee(1.0, 1.0, 1.0, 1.0, -1.0, 0.0))
    with pytest.raises(api.LapsError):
        api.laps_lm_derive_params((1.0, 0.0, 0.0, 0.0), 1.0, 0.0, [32, 16], [1, 2])
    with pytest.raises(api.LapsError):
        api.laps_lm_derive_params((0.0, 0.0, 0.0, 0.0), 1.0, 0.0, [16], [1])
