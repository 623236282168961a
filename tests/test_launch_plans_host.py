"""Host-only checks of the launch arithmetic behind the GEMM and attention kernels (laps_gemm_plan_info,
laps_attn_plan_info): whatever shape the layer driver asks for, the plan must satisfy what the kernels assume -
tiles that divide the matrix, K slices that are whole slabs and none of them empty, tables and partial-result
buffers large enough for every work item a batch of that shape can produce.  A violated assumption here is an
out-of-bounds access on the GPU, so these run on the CPU, over all model shapes and a sweep of row counts.
"""
import ctypes as C

import numpy as np
import pytest

from paper_2601_11589_amd import api

MODELS = {  # hidden, qkv width, intermediate
    "tiny": (256, 512, 512), "7B": (3584, 4608, 18944), "14B": (5120, 7168, 13824), "32B": (5120, 7168, 27648)}
ROWS = sorted(set(list(range(1, 131)) + [160, 192, 255, 256, 257, 384, 511, 512, 513, 1000, 1024, 2047, 2048, 2049, 4096,
                                         8192, 16384]))
PARTIAL, RESID, SWIGLU = 0, 1, 2


def gemm_plan(m, n, k, split=0, epi=PARTIAL):
    out = (C.c_int32 * 7)()
    rc = api.lib().laps_gemm_plan_info(C.c_int32(m), C.c_int32(n), C.c_int32(k), C.c_int32(split), C.c_int32(epi), out)
    assert rc == 0, api.lib().laps_last_error()
    return dict(zip(("bm", "bn", "split", "k_per", "epi", "ws", "wgs"), list(out)))


@pytest.mark.parametrize("model", sorted(MODELS))
def test_gemm_plans_satisfy_the_kernels_assumptions(model):
    d, qkv, inter = MODELS[model]
    projections = {"qkv": (qkv, d, PARTIAL), "o": (d, d, RESID), "gate_up": (2 * inter, d, SWIGLU), "down": (d, inter, RESID)}
    lib = api.lib()
    for name, (n, k, want) in projections.items():
        for m in ROWS:
            p = gemm_plan(m, n, k, 0, want)
            what = (model, name, m, p)
            assert p["bm"] in (128, 256) and n % p["bn"] == 0, what
            assert p["k_per"] % 64 == 0 and p["split"] >= 1, what
            slabs = p["k_per"] // 64
            assert p["ws"] in (1, 2) and slabs % p["ws"] == 0, what
            # every K slice holds work, the slices cover K, and the last one is a whole number of slab groups too
            assert (p["split"] - 1) * p["k_per"] < k <= p["split"] * p["k_per"], what
            last = (k - (p["split"] - 1) * p["k_per"]) // 64
            assert last >= p["ws"] and last % p["ws"] == 0, what
            # a fused epilogue only on an un-split K; SwiGLU only where a wave holds gate / up column pairs
            assert p["epi"] == (want if p["split"] == 1 else PARTIAL) or (want == SWIGLU and p["epi"] == PARTIAL), what
            if p["epi"] == SWIGLU:
                assert p["bn"] % 128 == 0, what
            assert p["wgs"] == -(-m // p["bm"]) * (n // p["bn"]) * p["split"], what
            if m <= 128:
                assert p["bm"] == 128 and p["wgs"] <= 256, what      # one streaming workgroup per compute unit at most
            # the workspace the public GEMM entry point asks for is the K slices' partial sums
            q = gemm_plan(m, n, k, 0, PARTIAL)
            need = lib.laps_gemm_workspace_bytes(C.c_int32(m), C.c_int32(n), C.c_int32(k), C.c_int32(0))
            assert need == (q["split"] * m * n * 4 if q["split"] > 1 else 0), what


def test_forced_k_splits_are_clamped_to_whole_slices():
    for n, k in ((7168, 5120), (5120, 27648), (512, 256)):
        for m in (1, 64, 128, 300, 2048):
            for split in (1, 2, 3, 5, 7, 8, 16, 64, 1000):
                p = gemm_plan(m, n, k, split, PARTIAL)
                assert 1 <= p["split"] <= k // 64
                assert (p["split"] - 1) * p["k_per"] < k <= p["split"] * p["k_per"]
                assert (p["k_per"] // 64) % p["ws"] == 0 and ((k - (p["split"] - 1) * p["k_per"]) // 64) % p["ws"] == 0


def test_plan_info_rejects_unsupported_shapes():
    lib = api.lib()
    out = (C.c_int32 * 7)()
    for m, n, k, s, e in ((0, 512, 256, 0, 0), (8, 100, 256, 0, 0), (8, 512, 100, 0, 0), (8, 512, 256, -1, 0), (8, 512, 256, 0, 3)):
        assert lib.laps_gemm_plan_info(C.c_int32(m), C.c_int32(n), C.c_int32(k), C.c_int32(s), C.c_int32(e), out) == -1
    assert lib.laps_gemm_plan_info(C.c_int32(8), C.c_int32(512), C.c_int32(256), C.c_int32(0), C.c_int32(0), None) == -1
    out6 = (C.c_int64 * 6)()
    for a in ((0, 8, 4, 2, 64, 4), (1, 0, 4, 2, 64, 4), (1, 8, 5, 2, 64, 4), (1, 8, 4, 2, 96, 4), (1, 8, 4, 2, 64, 0)):
        assert lib.laps_attn_plan_info(*[C.c_int32(v) for v in a], out6) == -1


def attn_plan(n_seq, n_tokens, n_q, n_kv, hd, max_pages):
    out = (C.c_int64 * 6)()
    rc = api.lib().laps_attn_plan_info(C.c_int32(n_seq), C.c_int32(n_tokens), C.c_int32(n_q), C.c_int32(n_kv),
                                       C.c_int32(hd), C.c_int32(max_pages), out)
    assert rc == 0, api.lib().laps_last_error()
    return dict(zip(("rows", "max_items", "n_split", "min_tiles", "table_bytes", "partial_bytes"), list(out)))


def test_attention_tables_and_partials_hold_every_work_item_of_a_batch_shape():
    """The grid, the work-item table and the key-split partial buffer are sized from the launch shape alone (a
    captured graph replays them for any lengths): every batch that fits the shape must fit them, and the key
    ranges the device derives per work item must tile [0, visible keys) without gaps."""
    KT, PAGE = 64, 16
    rng = np.random.default_rng(0)
    seen_split = seen_flat = 0
    for trial in range(6000):
        n_q, n_kv, hd = [(40, 8, 128), (28, 4, 128), (4, 2, 64)][rng.integers(3)]
        G = n_q // n_kv
        n_seq = int(rng.integers(1, 70))
        L = rng.integers(0, 65, n_seq) if rng.random() < 0.8 else rng.integers(0, 2100, n_seq)
        if rng.random() < 0.3:
            L[rng.integers(n_seq)] = int(rng.integers(1, 2049))
        H = np.where(rng.random(n_seq) < 0.3, 0, rng.integers(0, 8200, n_seq))
        n_tokens = int(L.sum()) + int(rng.integers(0, 40)) * int(rng.random() < 0.3)   # rows past the packed total: padding
        if n_tokens == 0:
            continue
        max_pages = int(max(1, ((H + L + PAGE - 1) // PAGE).max())) + int(rng.integers(0, 4))
        p = attn_plan(n_seq, n_tokens, n_q, n_kv, hd, max_pages)
        assert p["rows"] in (128, 256) and p["n_split"] >= 1
        items = (L * G + p["rows"] - 1) // p["rows"]
        assert items.sum() <= p["max_items"], (trial, p)
        assert (p["max_items"] + 1) * 4 <= p["table_bytes"], (trial, p)
        if p["n_split"] > 1:
            seen_split += 1
            assert p["rows"] == 128
            blocks = p["max_items"] * n_kv * p["n_split"]
            assert blocks * 128 * (hd + 2) * 4 <= p["partial_bytes"], (trial, p)
        else:
            seen_flat += 1
        for s in range(n_seq):
            n_rows, kv_len = int(L[s]) * G, int(H[s] + L[s])
            for q in range(int(items[s])):
                last = min((q + 1) * p["rows"], n_rows) - 1
                kv_end = int(H[s]) + last // G + 1
                assert 1 <= kv_end <= kv_len
                if p["n_split"] == 1:
                    continue
                nt = (kv_end + KT - 1) // KT
                eff = min(max(nt // p["min_tiles"], 1), p["n_split"])
                per = (nt + eff - 1) // eff
                wrote = [z for z in range(p["n_split"]) if z < eff and z * per * KT < kv_end]
                used = min((nt + per - 1) // per, eff)                # what the merge kernel expects to find
                assert wrote == list(range(used)), (trial, s, q)
                ranges = [(z * per * KT, min((z + 1) * per * KT, kv_end)) for z in wrote]
                assert ranges[0][0] == 0 and ranges[-1][1] == kv_end and all(a < b for a, b in ranges)
                assert all(ranges[i][1] == ranges[i + 1][0] for i in range(len(ranges) - 1))
    assert seen_split > 200 and seen_flat > 200


def test_a_workspace_sized_for_a_maximum_serves_every_smaller_batch():
    """laps_workspace_bytes(max_tokens, max_seqs) must cover every call with fewer rows and sequences (each call
    checks its own need against the buffer it is given): the K-split factor, and with it the partial-sum region,
    does not grow monotonically with the row count."""
    from paper_2601_11589_amd import inputs
    lib = api.lib()
    for cfgf in (inputs.tiny_cfg, inputs.qwen7b_cfg, inputs.qwen14b_cfg, inputs.qwen32b_cfg):
        cfg = cfgf(1)
        c = api._ModelCfg(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.intermediate, cfg.n_layers, 16,
                          int(getattr(cfg, "has_qkv_bias", 0)), 1e6, 1e-6)
        need = lambda m, s: lib.laps_workspace_bytes_for(C.byref(c), C.c_int32(m), C.c_int32(s))
        assert need(0, 1) == 0 and need(8, 0) == 0
        for cap, seqs in ((64, 4), (128, 8), (200, 8), (300, 16), (512, 8), (1000, 64), (2048, 1), (4096, 64)):
            total = need(cap, seqs)
            assert total > 0
            for m in sorted(set(list(range(1, min(cap, 300) + 1)) + list(range(300, cap + 1, 37)) + [cap])):
                assert need(m, min(seqs, m)) <= total, (cfgf.__name__, cap, m)
