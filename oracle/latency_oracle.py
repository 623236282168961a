"""Oracle for the compute / memory latency model and its boundaries.  TEST INFRASTRUCTURE ONLY.

Section 2.1 of the paper: T_comp = alpha L (L + 2H) + beta L, T_mem = gamma_w L + gamma_r H; the boundary
is the length at which the two are equal.  Instead of the printed closed forms, this oracle solves
T_comp(L) - T_mem(L) = 0 numerically as a polynomial (numpy.roots) and fits the coefficients with
numpy.linalg.lstsq, so that the library's closed forms and normal equations are checked against
independent routines.  Pins (tests/test_latency_model.py): worked values computed by hand from the
printed formulas, the H = 0 reduction, the large-H limit gamma_r / (2 alpha), T_comp == T_mem at the root;
for the knee with a weight-streaming floor and the parameters derived from it: hand-worked roots, the
floor = 0 reduction to the printed boundary, hand-worked parameter sets on the paper's example grids.
"""
from __future__ import annotations

import numpy as np


def t_comp(alpha, beta, L, H):
    return alpha * L * (L + 2.0 * H) + beta * L


def t_mem(gamma_w, gamma_r, L, H):
    return gamma_w * L + gamma_r * H


def boundary(alpha, beta, gamma_w, gamma_r, H):
    """Largest non-negative real L with T_comp(L,H) = T_mem(L,H); 0 if there is none."""
    roots = np.roots([alpha, 2.0 * alpha * H + beta - gamma_w, -gamma_r * H])
    real = [float(r.real) for r in roots if abs(r.imag) < 1e-12 and r.real > 0]
    return max(real) if real else 0.0


def knee(alpha, beta, gamma_w, gamma_r, floor_t, H):
    """The same balance with a constant memory term (the time to stream the weights once): largest positive real L
    with alpha L (L + 2H) + beta L = floor_t + gamma_w L + gamma_r H, by numpy.roots; 0 if there is none."""
    roots = np.roots([alpha, 2.0 * alpha * H + beta - gamma_w, -(floor_t + gamma_r * H)])
    real = [float(r.real) for r in roots if abs(r.imag) < 1e-12 and r.real > 0]
    return max(real) if real else 0.0


def derive_params(coef, floor_t, hist_max, len_buckets, depths):
    """Scheduling parameters from a fit, by enumeration: the knee is the smaller of the knees at H = 0 and at
    H = hist_max; short_max_len = the largest length bucket within it (the smallest bucket if none is); the token
    budget of a latency-oriented graph and the fusion budget = the largest padded size len_bucket * depth within the
    knee among buckets up to short_max_len (at least one request of short_max_len at the smallest depth)."""
    a, b, gw, gr = coef
    k = min(knee(a, b, gw, gr, floor_t, 0.0), knee(a, b, gw, gr, floor_t, hist_max))
    fits = [lb for lb in len_buckets if lb <= k]
    sml = max(fits) if fits else min(len_buckets)
    shapes = [lb * d for lb in len_buckets if lb <= sml for d in depths if lb * d <= k]
    budget = max(shapes + [sml * min(depths)])
    return {"short_max_len": sml, "short_token_budget": budget, "fuse_budget": budget}


def fit(L, H, tc, tm):
    L, H, tc, tm = (np.asarray(a, np.float64) for a in (L, H, tc, tm))
    ab, *_ = np.linalg.lstsq(np.stack([L * (L + 2 * H), L], 1), tc, rcond=None)
    gg, *_ = np.linalg.lstsq(np.stack([L, H], 1), tm, rcond=None)
    return float(ab[0]), float(ab[1]), float(gg[0]), float(gg[1])
