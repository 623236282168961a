"""Oracle for the instance-pressure controller of spatial disaggregation.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

What the paper fixes (Algorithm 2; Section 3.2, spatial disaggregation): N instances in a SHORT pool (n_s) and a
LONG pool (n_l = N - n_s); every control period each instance k reports queue backlog q_k, SLA deviation e_k and
utilisation u_k, giving psi_k = alpha q_k + beta e_k - gamma u_k; a robust aggregate (P90) per pool, P_s and P_l;
during the cool-down after a migration nothing moves; otherwise one instance moves to the SHORT pool if
P_s > (1 + tau) P_l and n_l > n_min, else one to the LONG pool if P_l > (1 + tau) P_s and n_s > n_min.
Readings where the paper is silent: the P90 of a set is its nearest-rank quantile (the smallest member with at
least 90 % of the set at or below it); an empty pool has pressure 0; which instance of the donor pool moves is the
caller's choice.  Optional, off by default (not in the printed algorithm): no move unless the pressure of the pool
that would gain exceeds `min_pressure` - with the utilisation term both pressures can be negative, where a
ratio test flips sign and idle pools would trade instances forever.

Pins (tests/test_pool_ctrl.py): quantiles worked by hand, a hand-worked control sequence (hysteresis band,
cool-down, minimum allocation), and the invariants n_s + n_l = N, both >= n_min, at most one move per period.
"""
from __future__ import annotations

import math


def quantile_nearest_rank(values, q=0.9):
    if not values:
        return 0.0
    v = sorted(values)
    rank = max(1, math.ceil(q * len(v)))
    return v[rank - 1]


class Controller:
    def __init__(self, n_total, n_short, n_min=1, cool=0.0, tau=0.1, alpha=1.0, beta=1.0, gamma=1.0, q=0.9,
                 min_pressure=-math.inf):
        assert 0 <= n_short <= n_total
        self.N, self.n_s, self.n_l = n_total, n_short, n_total - n_short
        self.n_min, self.cool, self.tau = n_min, cool, tau
        self.alpha, self.beta, self.gamma, self.q = alpha, beta, gamma, q
        self.t_last = -math.inf
        self.min_pressure = min_pressure

    def step(self, now, short_signals, long_signals):
        """signals: lists of (q_k, e_k, u_k).  Returns (action, P_s, P_l); action +1 = one instance LONG -> SHORT,
        -1 = one SHORT -> LONG, 0 = none."""
        psi = lambda s: [self.alpha * qk + self.beta * ek - self.gamma * uk for qk, ek, uk in s]
        p_s = quantile_nearest_rank(psi(short_signals), self.q)
        p_l = quantile_nearest_rank(psi(long_signals), self.q)
        if now - self.t_last < self.cool:
            return 0, p_s, p_l
        if p_s > (1 + self.tau) * p_l and p_s > self.min_pressure and self.n_l > self.n_min:
            self.n_s, self.n_l, self.t_last = self.n_s + 1, self.n_l - 1, now
            return 1, p_s, p_l
        if p_l > (1 + self.tau) * p_s and p_l > self.min_pressure and self.n_s > self.n_min:
            self.n_l, self.n_s, self.t_last = self.n_l + 1, self.n_s - 1, now
            return -1, p_s, p_l
        return 0, p_s, p_l
