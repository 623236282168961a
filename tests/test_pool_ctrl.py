"""Instance-pressure controller (Algorithm 2): the oracle against hand-worked values, the library against the oracle."""
import math

import numpy as np
import pytest

from oracle import ctrl_oracle as CO
from paper_2601_11589_amd import api


def test_oracle_nearest_rank_quantile_by_hand():
    assert CO.quantile_nearest_rank([5.0]) == 5.0                       # ceil(0.9 * 1) = 1st
    assert CO.quantile_nearest_rank([3.0, 1.0]) == 3.0                  # ceil(1.8) = 2nd of (1, 3)
    assert CO.quantile_nearest_rank(list(range(1, 11))) == 9            # ceil(9.0) = 9th of 1..10
    assert CO.quantile_nearest_rank(list(range(1, 12))) == 10           # ceil(9.9) = 10th of 1..11
    assert CO.quantile_nearest_rank([4.0, 2.0, 8.0, 6.0], q=0.5) == 4.0  # ceil(2.0) = 2nd of (2, 4, 6, 8)
    assert CO.quantile_nearest_rank([]) == 0.0


def hand_sequence():
    """N = 4, two per pool, n_min = 1, cool-down 10, tau = 0.5, weights (1, 2, 0.5), P90.  Signals are (q, e, u).
    t=0 : short psi = (1*4 + 2*1 - 0.5*1, 1*2 + 0 - 0.5) = (5.5, 1.5) -> P_s = 5.5; long psi = (1.5, 0.5) -> P_l = 1.5;
          5.5 > 1.5 * 1.5 and n_l = 2 > 1 -> +1 (pools 3 / 1), t_last = 0.
    t=5 : same imbalance but 5 - 0 < 10 -> 0.
    t=10: short psi (3 instances) = (2, 2, 2) -> 2; long (1 instance) = (9,) -> 9; 9 > 1.5 * 2 and n_s = 3 > 1 -> -1 (2 / 2).
    t=20: short (1.0, 1.0), long (1.4, 0.2): P_l = 1.4 <= 1.5 * 1.0 and P_s = 1.0 <= 1.5 * 1.4 -> 0 (inside the band).
    t=30: short (8, 8), long (1, 1): -> +1 (3 / 1).   t=40: short (8, 8, 8), long (1,): n_l = 1 = n_min -> 0."""
    return [
        (0.0, [(4, 1, 1), (2, 0, 1)], [(2, 0, 1), (1, 0, 1)], (1, 5.5, 1.5)),
        (5.0, [(4, 1, 1), (2, 0, 1), (2, 0, 1)], [(1, 0, 1)], (0, 5.5, 0.5)),
        (10.0, [(2.5, 0, 1), (2.5, 0, 1), (2.5, 0, 1)], [(9.5, 0, 1)], (-1, 2.0, 9.0)),
        (20.0, [(1.5, 0, 1), (1.5, 0, 1)], [(1.9, 0, 1), (0.7, 0, 1)], (0, 1.0, 1.4)),
        (30.0, [(8.5, 0, 1), (8.5, 0, 1)], [(1.5, 0, 1), (1.5, 0, 1)], (1, 8.0, 1.0)),
        (40.0, [(8.5, 0, 1)] * 3, [(1.5, 0, 1)], (0, 8.0, 1.0)),
    ]


def test_oracle_hand_worked_sequence():
    c = CO.Controller(4, 2, n_min=1, cool=10.0, tau=0.5, alpha=1.0, beta=2.0, gamma=0.5)
    for now, ss, ls, want in hand_sequence():
        got = c.step(now, ss, ls)
        assert got[0] == want[0] and got[1] == pytest.approx(want[1]) and got[2] == pytest.approx(want[2]), (now, got)
    assert (c.n_s, c.n_l) == (3, 1)


def test_library_hand_worked_sequence():
    c = api.LapsCtrl(4, 2, n_min=1, cool_us=10.0, tau=0.5, w_q=1.0, w_e=2.0, w_u=0.5)
    for now, ss, ls, want in hand_sequence():
        got = c.laps_ctrl_step(now, ss, ls)
        assert got[0] == want[0] and got[1] == pytest.approx(want[1]) and got[2] == pytest.approx(want[2]), (now, got)
    assert c.n_short == 3
    c.close()


@pytest.mark.parametrize("seed", range(5))
def test_library_matches_oracle_on_random_signals(seed):
    rng = np.random.default_rng(300 + seed)
    N, n_min = int(rng.integers(2, 17)), int(rng.integers(0, 2))
    n_s = int(rng.integers(n_min, N - n_min + 1))
    kw = dict(cool=float(rng.choice([0.0, 3.0])), tau=float(rng.choice([0.0, 0.2, 1.0])))
    mp = float(rng.choice([-math.inf, 0.0, 4.0]))
    w = [float(x) for x in rng.uniform(0, 2, 3)]
    oc = CO.Controller(N, n_s, n_min=n_min, alpha=w[0], beta=w[1], gamma=w[2], min_pressure=mp, **kw)
    lc = api.LapsCtrl(N, n_s, n_min=n_min, cool_us=kw["cool"], tau=kw["tau"], w_q=w[0], w_e=w[1], w_u=w[2], min_pressure=mp)
    for step in range(200):
        ss = [tuple(rng.uniform(0, 10, 3)) for _ in range(oc.n_s)]
        ls = [tuple(rng.uniform(0, 10, 3)) for _ in range(oc.n_l)]
        want = oc.step(float(step), ss, ls)
        got = lc.laps_ctrl_step(float(step), ss, ls)
        assert got[0] == want[0] and got[1] == pytest.approx(want[1], rel=1e-12) and got[2] == pytest.approx(want[2], rel=1e-12)
        assert lc.n_short == oc.n_s and oc.n_s + oc.n_l == N
        assert oc.n_s >= min(n_min, n_s) and oc.n_l >= min(n_min, N - n_s)
    lc.close()


def test_min_pressure_by_hand():
    """P_s = -0.2, P_l = -0.4, tau = 0.25: as printed -0.2 > 1.25 * -0.4 = -0.5 moves an instance to the idle SHORT pool;
    with min_pressure = 0 nothing moves."""
    sig_s, sig_l = [(0.0, 0.0, 0.2)], [(0.0, 0.0, 0.4)]
    for make in (lambda **k: CO.Controller(2, 1, n_min=0, tau=0.25, **k),):
        assert make().step(0.0, sig_s, sig_l)[0] == 1
        assert make(min_pressure=0.0).step(0.0, sig_s, sig_l)[0] == 0
    assert api.LapsCtrl(2, 1, n_min=0, tau=0.25).laps_ctrl_step(0.0, sig_s, sig_l)[0] == 1
    assert api.LapsCtrl(2, 1, n_min=0, tau=0.25, min_pressure=0.0).laps_ctrl_step(0.0, sig_s, sig_l)[0] == 0


def test_library_ctrl_argument_errors():
    with pytest.raises(api.LapsError):
        api.LapsCtrl(4, 5)
    with pytest.raises(api.LapsError):
        api.LapsCtrl(4, 2, quantile=0.0)
    c = api.LapsCtrl(4, 2)
    with pytest.raises(api.LapsError):
        c.laps_ctrl_step(0.0, [(1, 1, 1)], [(1, 1, 1), (2, 2, 2)])       # 1 + 2 signals for pools of 2 + 2
    with pytest.raises(api.LapsError):
        c.laps_ctrl_step(0.0, [(1, 1, 1), (1, float("nan"), 1)], [(1, 1, 1), (2, 2, 2)])   # a NaN signal has no rank
    assert c.n_short == 2
    c.close()


def test_pool_simulation_controller_follows_a_workload_shift():
    """N = 8 virtual instances, service times of the order measured on the GPU for a 64-layer 32B model (short
    replay ~17-25 ms, 2048-token chunk ~145 ms).  Phase A loads the short pool, phase B the long pool; a static 4/4
    split overloads the long pool in phase B, the controller moves instances there."""
    from paper_2601_11589_amd import poolsim
    arr, ln, lg = poolsim.shifting_workload(7, 40e6, short_rate_a=900, long_rate_a=2, short_rate_b=150, long_rate_b=10)
    step = lambda d: 17_000.0 + 1_000.0 * d
    prm = poolsim.PoolSimParams()
    stat = poolsim.simulate(arr, ln, lg, step, 145_000.0, prm, controller=False)
    dyn = poolsim.simulate(arr, ln, lg, step, 145_000.0, prm, controller=True)
    print(stat)
    print(dyn)
    assert stat["migrations"] == 0 and dyn["migrations"] >= 1
    assert any(a == -1 for _, a in dyn["moves"])                         # instances went to the LONG pool in phase B
    assert dyn["slo_violation_frac"] < stat["slo_violation_frac"]
    assert dyn["long_latency_ms"]["p99"] < stat["long_latency_ms"]["p99"]
