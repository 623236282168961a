"""Fixed-window dispatch of the short queue (Section 3.1 waiting window and graph fusion, Section 3.2 two queues):
the oracle against hand-worked decisions and limits, the library (laps_window_poll) against the oracle."""
import math

import numpy as np
import pytest

from oracle import window_oracle as WO
from paper_2601_11589_amd import api

GRID = [16, 32, 64]


def test_oracle_hand_worked_decisions():
    # three requests of 10, 20, 60 tokens need 16 + 32 + 64 = 112 padded tokens; the oldest arrived at t = 100
    arr, lens = [100.0, 150.0, 180.0], [10, 20, 60]
    # window 500 not yet over at t = 400, budget 2048 not reached, a long request still waits: keep waiting until 600
    assert WO.poll(GRID, 500.0, 2048, 128, 400.0, arr, lens, False) == \
        {"dispatch": False, "fused_len_bucket": 0, "padded_tokens": 112, "wake_us": 600.0}
    # at t = 600 the oldest has waited exactly the window: leave; 112 < 128 padded tokens: all in the 64-token bucket
    assert WO.poll(GRID, 500.0, 2048, 128, 600.0, arr, lens, False) == \
        {"dispatch": True, "fused_len_bucket": 64, "padded_tokens": 112, "wake_us": math.inf}
    # budget 112 is filled at once, whatever the window; merge_below 112 is not undercut: no fusion
    assert WO.poll(GRID, 500.0, 112, 112, 200.0, arr, lens, False)["dispatch"] is True
    assert WO.poll(GRID, 500.0, 112, 112, 200.0, arr, lens, False)["fused_len_bucket"] == 0
    # nothing else to run: leave although neither window nor budget says so
    assert WO.poll(GRID, 500.0, 2048, 0, 200.0, arr, lens, True)["dispatch"] is True
    # an empty queue never dispatches
    assert WO.poll(GRID, 0.0, 1, 128, 5.0, [], [], True) == \
        {"dispatch": False, "fused_len_bucket": 0, "padded_tokens": 0, "wake_us": math.inf}
    # lengths on bucket edges: 16 -> 16, 17 -> 32, 64 -> 64
    assert WO.poll(GRID, 0.0, 10 ** 9, 0, 1.0, [0.0, 0.0, 0.0], [16, 17, 64], False)["padded_tokens"] == 112


def test_oracle_limits():
    rng = np.random.default_rng(3)
    for _ in range(50):
        n = int(rng.integers(1, 20))
        arr = np.sort(rng.uniform(0, 1000, n))
        lens = rng.integers(1, 65, n)
        now = float(arr[-1] + rng.uniform(0, 100))
        assert WO.poll(GRID, 0.0, 10 ** 9, 128, now, arr, lens, False)["dispatch"]            # W = 0: always
        never = WO.poll(GRID, math.inf, 10 ** 9, 128, now, arr, lens, False)                   # W = inf, huge budget
        assert not never["dispatch"] and never["wake_us"] == math.inf
        assert WO.poll(GRID, math.inf, 10 ** 9, 128, now, arr, lens, True)["dispatch"]         # ... unless nothing else


def test_library_matches_oracle_on_random_queues():
    rng = np.random.default_rng(2601_11589)
    grids = [GRID, [8, 16, 32, 64, 128, 256], [24, 40]]
    for _ in range(600):
        grid = grids[int(rng.integers(len(grids)))]
        n = int(rng.integers(0, 30))
        arr = np.sort(rng.uniform(0, 5000, n))
        lens = rng.integers(1, grid[-1] + 1, n)
        now = float((arr[-1] if n else 0.0) + rng.choice([0.0, 1.0, 300.0, 3000.0]))
        w = float(rng.choice([0.0, 100.0, 1000.0, 10000.0]))
        budget = int(rng.choice([1, 64, 128, 512, 2048]))
        merge = int(rng.choice([0, 64, 128, 200, 4096]))
        ne = bool(rng.integers(2))
        got = api.laps_window_poll(grid, w, budget, merge, now, arr, lens, ne)
        want = WO.poll(grid, w, budget, merge, now, list(arr), list(lens), ne)
        assert got == want, (grid, w, budget, merge, now, list(arr), list(lens), ne, got, want)


def test_library_rejects_bad_input():
    with pytest.raises(api.LapsError):
        api.laps_window_poll(GRID, 100.0, 128, 128, 10.0, [0.0], [65], False)          # longer than the largest bucket
    with pytest.raises(api.LapsError):
        api.laps_window_poll(GRID, 100.0, 128, 128, 10.0, [5.0, 1.0], [8, 8], False)   # arrivals out of order
    with pytest.raises(api.LapsError):
        api.laps_window_poll(GRID, 100.0, 128, 128, 10.0, [11.0], [8], False)          # arrival after now
    with pytest.raises(api.LapsError):
        api.laps_window_poll([32, 16], 100.0, 128, 128, 10.0, [1.0], [8], False)
    with pytest.raises(api.LapsError):
        api.laps_window_poll(GRID, -1.0, 128, 128, 10.0, [1.0], [8], False)
