"""Brute-force oracle for the length-aware bucket plan.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  Pure Python integers; exhaustive enumeration, so only for small inputs.

What the paper fixes (Section 3.1 "Graph capture and bucketization", "Graph-aware
memory-based batching", Algorithm 1; Section 3.2 "Mutual exclusion", deadline-free mode):
  * requests are classified by prompt length against a boundary into a short and a long queue;
  * a grid of (prompt length L, batch size B) shapes exists; a short request is padded up to
    a length bucket and grouped with requests of the same length bucket;
  * a batch is matched to a captured shape with depth >= the batch's depth and memory within
    the budget M, else it runs on the standard (un-captured) path;
  * the batching goals are fewer graph launches and more reuse of large-batch graphs;
  * a long request advances alone in fixed-size chunks C_l.
Readings taken where the paper is silent: length means NEW tokens; short iff
new_len <= short_max_len; bucket = smallest length bucket >= new_len; mem(G) = depth * L_b
padded tokens against token_budget; ties resolved as (fewest launches, fewest padded rows,
larger depths first); arrival order kept.

Pins (tests/test_plan_oracle.py): hand-worked plans stored under tests/golden/, the closed
form for power-of-two grids (floor(n/D) full batches plus one nearest-depth remainder),
and the structural invariants (every request exactly once, minimal bucket, budget respected,
chunk lengths sum to the prompt length).
"""
from __future__ import annotations

from itertools import combinations_with_replacement, product


def _best_depth_multiset(n_rows: int, allowed: list[int]) -> tuple[int, ...]:
    """Over every multiset of allowed depths with total >= n_rows, the one that minimises
    (number of launches, total padded rows) and, among those, is largest when written in
    descending order (larger depths first)."""
    best_key, best = None, None
    for count in range(1, n_rows + 1):
        for combo in combinations_with_replacement(sorted(allowed, reverse=True), count):
            total = sum(combo)
            if total < n_rows:
                continue
            key = (count, total, tuple(-d for d in combo))
            if best_key is None or key < best_key:
                best_key, best = key, combo
    return best


def _best_contiguous_split(lens: list[int], budget: int) -> list[int]:
    """Un-captured fallback: split requests (arrival order kept, contiguous groups) so that each
    group's un-padded token total is within budget (a single over-budget request forms its own
    group), using the fewest groups and, among those, the largest leading groups."""
    n = len(lens)
    best_key, best = None, None
    for cuts in product([0, 1], repeat=n - 1):
        sizes, cur = [], 1
        for c in cuts:
            if c:
                sizes.append(cur)
                cur = 1
            else:
                cur += 1
        sizes.append(cur)
        ok, o = True, 0
        for s in sizes:
            tot = sum(lens[o:o + s])
            if s > 1 and tot > budget:
                ok = False
                break
            o += s
        if not ok:
            continue
        key = (len(sizes), tuple(-s for s in sizes))
        if best_key is None or key < best_key:
            best_key, best = key, sizes
    return best


def plan_buckets(short_max_len: int, len_buckets: list[int], depths: list[int], token_budget: int,
                 long_chunk: int, new_len: list[int], prefix_len: list[int]) -> dict:
    n = len(new_len)
    assert len(prefix_len) == n
    cls = [0 if new_len[i] <= short_max_len else 1 for i in range(n)]
    bucket = [-1] * n
    for i in range(n):
        if cls[i] == 0:
            for j, lb in enumerate(len_buckets):
                if lb >= new_len[i]:
                    bucket[i] = j
                    break
            assert bucket[i] >= 0, "short_max_len must not exceed the largest length bucket"
    batches = []
    for j, lb in enumerate(len_buckets):
        reqs = [i for i in range(n) if cls[i] == 0 and bucket[i] == j]
        if not reqs:
            continue
        allowed = [b for b in depths if b * lb <= token_budget]
        if allowed:
            o = 0
            for d in _best_depth_multiset(len(reqs), allowed):
                take = reqs[o:o + d]
                o += len(take)
                batches.append({"len_bucket": lb, "depth": d, "graph_ok": 1, "req_ids": take})
        else:
            o = 0
            for s in _best_contiguous_split([new_len[i] for i in reqs], token_budget):
                batches.append({"len_bucket": lb, "depth": s, "graph_ok": 0, "req_ids": reqs[o:o + s]})
                o += s
    longs = []
    for i in range(n):
        if cls[i] == 1:
            full, rem = divmod(new_len[i], long_chunk)
            longs.append({"req_id": i, "chunks": [long_chunk] * full + ([rem] if rem else [])})
    return {"cls": cls, "bucket": bucket, "batches": batches, "longs": longs}
