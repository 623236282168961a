"""Pins for the brute-force plan oracle: hand-worked plans, the closed form on
power-of-two grids, structural invariants."""
import json
import os
import random

import pytest

from oracle import plan_oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "plan_cases.json")


def load_cases():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", load_cases(), ids=lambda c: c["name"])
def test_hand_worked_plans(case):
    p = case["params"]
    got = plan_oracle.plan_buckets(p["short_max_len"], p["len_buckets"], p["depths"], p["token_budget"],
                                   p["long_chunk"], case["new_len"], case["prefix_len"])
    assert got["cls"] == case["cls"]
    assert got["bucket"] == case["bucket"]
    assert got["batches"] == case["batches"]
    assert got["longs"] == case["longs"]


def random_case(rng, n_max=10):
    n_lb = rng.randint(1, 4)
    len_buckets = sorted(rng.sample([4, 8, 16, 32, 64], n_lb))
    depths = sorted(rng.sample([1, 2, 3, 4, 6, 8], rng.randint(1, 4)))
    short_max = rng.choice([len_buckets[-1], len_buckets[-1] - 1, len_buckets[0]])
    budget = rng.choice([8, 16, 32, 64, 100, 128, 256])
    chunk = rng.choice([16, 64, 100])
    n = rng.randint(0, n_max)
    new_len = [rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 31, 32, 33, 64, 65, 100, 129, 300]) for _ in range(n)]
    prefix = [rng.choice([0, 1, 15, 16, 17, 500]) for _ in range(n)]
    return dict(short_max_len=short_max, len_buckets=len_buckets, depths=depths, token_budget=budget,
                long_chunk=chunk, new_len=new_len, prefix_len=prefix)


def test_invariants_on_random_small_inputs():
    rng = random.Random(11589)
    for _ in range(150):
        c = random_case(rng)
        plan = plan_oracle.plan_buckets(**c)
        n = len(c["new_len"])
        seen = []
        for b in plan["batches"]:
            seen += b["req_ids"]
            assert b["req_ids"] == sorted(b["req_ids"])                 # arrival order kept
            assert 1 <= len(b["req_ids"]) <= b["depth"]
            for i in b["req_ids"]:
                assert c["new_len"][i] <= b["len_bucket"]
                smaller = [lb for lb in c["len_buckets"] if lb < b["len_bucket"]]
                assert all(lb < c["new_len"][i] for lb in smaller)      # minimal bucket
            if b["graph_ok"]:
                assert b["depth"] in c["depths"]
                assert b["depth"] * b["len_bucket"] <= c["token_budget"]
            else:
                assert all(d * b["len_bucket"] > c["token_budget"] for d in c["depths"])
                tot = sum(c["new_len"][i] for i in b["req_ids"])
                assert tot <= c["token_budget"] or len(b["req_ids"]) == 1
        for lg in plan["longs"]:
            seen.append(lg["req_id"])
            assert sum(lg["chunks"]) == c["new_len"][lg["req_id"]]
            assert all(x == c["long_chunk"] for x in lg["chunks"][:-1])
            assert 1 <= lg["chunks"][-1] <= c["long_chunk"]
            assert c["new_len"][lg["req_id"]] > c["short_max_len"]
        assert sorted(seen) == list(range(n))                           # each request exactly once
        assert [b["len_bucket"] for b in plan["batches"]] == sorted(b["len_bucket"] for b in plan["batches"])


def test_power_of_two_grid_closed_form():
    """floor(n/D) batches of the cap depth D plus one remainder batch at the smallest depth
    that holds it."""
    depths = [1, 2, 4, 8, 16]
    for lb, budget in [(16, 128), (32, 128), (64, 128), (16, 256), (8, 8)]:
        cap = max(b for b in depths if b * lb <= budget)
        for n in range(1, 12):
            plan = plan_oracle.plan_buckets(lb, [lb], depths, budget, 1024, [lb] * n, [0] * n)
            got = [b["depth"] for b in plan["batches"]]
            full, rem = divmod(n, cap)
            want = [cap] * full + ([min(b for b in depths if b >= rem)] if rem else [])
            assert got == want, (lb, budget, n)
            assert len(got) == -(-n // cap)                              # launches = ceil(n / D)


def test_padding_never_truncates_and_boundary_is_inclusive():
    plan = plan_oracle.plan_buckets(64, [16, 32, 64], [1, 2], 128, 2048, [64, 65, 17, 16], [0, 0, 5000, 5000])
    assert plan["cls"] == [0, 1, 0, 0]
    assert plan["bucket"] == [2, -1, 1, 0]            # 17 -> 32 (never rounded down to 16); prefix ignored
