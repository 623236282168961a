"""Oracle for the fixed-window dispatch rule of the short queue.  TEST INFRASTRUCTURE ONLY.

The paper keeps a short and a long queue, runs one class of prefill at a time (Section 3.2) and batches short
requests into captured shapes after a waiting window, fusing graphs where that pays (Section 3.1).  Read for one GPU
that alternates between the queues, the decision at an instant `now` over the waiting short requests is written
here directly from that reading, in plain Python: the queue leaves when the oldest request has waited the window,
when the padded tokens fill the graph budget, or when nothing else could use the GPU; below `merge_below` padded
tokens all requests share the widest bucket any of them needs.
Pins (tests/test_window_dispatch.py): hand-worked decisions, and the limits W = 0 (always dispatch) and W = infinity
with an unreachable budget (dispatch only when nothing else is left).
"""
from __future__ import annotations

import math


def need(len_buckets, n):
    for b in len_buckets:
        if b >= n:
            return b
    raise ValueError("length outside the grid")


def poll(len_buckets, window_us, token_budget, merge_below, now_us, arrival_us, new_len, nothing_else):
    needs = [need(len_buckets, n) for n in new_len]
    padded = sum(needs)
    if not needs:
        return {"dispatch": False, "fused_len_bucket": 0, "padded_tokens": 0, "wake_us": math.inf}
    waited = now_us - arrival_us[0]
    if waited >= window_us or padded >= token_budget or nothing_else:
        return {"dispatch": True, "fused_len_bucket": max(needs) if padded < merge_below else 0,
                "padded_tokens": padded, "wake_us": math.inf}
    return {"dispatch": False, "fused_len_bucket": 0, "padded_tokens": padded, "wake_us": arrival_us[0] + window_us}
