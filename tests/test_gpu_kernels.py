"""GPU parity of the HIP path against the fp64 oracle, called through the C-ABI binding.
Sizes: small enough for the oracle to finish in seconds, large enough to span several tiles and a
ragged tail.  Full-size configurations live in test_gpu_configs.py."""
import math

import numpy as np
import pytest
import torch

from oracle import laps_oracle as O
from paper_2601_11589_amd import api, inputs

from gpu_harness import MAX_ABS_TOL, REL_L2_TOL, Case, errors

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tiny_ctx():
    ctx = api.LapsCtx(inputs.tiny_cfg(1), max_positions=4096)
    yield ctx
    ctx.close()


def rand_bf16(rng, shape, std=1.0):
    return inputs.f32_to_bf16_bits((rng.standard_normal(shape) * std).astype(np.float32))


# ----------------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("m,n,k,split", [
    (1, 128, 64, 0), (37, 256, 256, 0), (128, 512, 512, 0), (128, 512, 512, 1), (100, 256, 1024, 3),
    (129, 256, 256, 0), (300, 512, 512, 0), (515, 1024, 256, 1), (515, 1024, 1024, 2), (515, 384, 320, 0),
    (2048, 512, 2048, 0),
])
def test_gemm_matches_fp64_matmul(tiny_ctx, m, n, k, split):
    rng = np.random.default_rng(m * 1000003 + n * 101 + k)
    a, w = rand_bf16(rng, (m, k)), rand_bf16(rng, (n, k), 0.05)
    want = inputs.bf16_bits_to_f64(a) @ inputs.bf16_bits_to_f64(w).T          # library routine, fp64
    got = tiny_ctx.laps_gemm_bf16(api.bf16_tensor(a), api.bf16_tensor(w), split_k=split)
    torch.cuda.synchronize()
    rel, mx = errors(got.cpu().numpy(), want)
    assert rel < 2e-6 and mx < 1e-4 * math.sqrt(k), (rel, mx)      # fp32 accumulation of exact bf16 products


def test_gemm_tiny_explicit_triple_loop(tiny_ctx):
    rng = np.random.default_rng(5)
    m, n, k = 3, 128, 64
    a, w = rand_bf16(rng, (m, k)), rand_bf16(rng, (n, k))
    af, wf = inputs.bf16_bits_to_f64(a), inputs.bf16_bits_to_f64(w)
    got = tiny_ctx.laps_gemm_bf16(api.bf16_tensor(a), api.bf16_tensor(w)).cpu().numpy()
    for i in range(m):
        for j in (0, 1, 31, 32, 63, 64, 127):
            want = sum(af[i, t] * wf[j, t] for t in range(k))
            assert abs(got[i, j] - want) < 1e-4


def test_gemm_rejects_bad_shapes(tiny_ctx):
    a = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((128, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.LapsError):
        tiny_ctx.laps_gemm_bf16(a, w)                       # k % 64 != 0
    a = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((100, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.LapsError):
        tiny_ctx.laps_gemm_bf16(a, w)                       # n % 128 != 0


# ----------------------------------------------------------------------------------- attention
def attention_case(cfg, new_len, prefix_len, seed):
    """Random q and KV placed in poisoned pools; returns device inputs and the oracle's output."""
    rng = np.random.default_rng(seed)
    n = len(new_len)
    cu = np.concatenate([[0], np.cumsum(new_len)]).astype(np.int32)
    T = int(cu[-1])
    table, n_pages = inputs.make_page_table(seed, new_len, prefix_len)
    q = rand_bf16(rng, (T, cfg.n_q_heads, cfg.head_dim))
    tot = np.asarray(new_len) + np.asarray(prefix_len)
    kv_cu = np.concatenate([[0], np.cumsum(tot)]).astype(np.int32)
    k = rand_bf16(rng, (int(kv_cu[-1]), cfg.n_kv_heads, cfg.head_dim))
    v = rand_bf16(rng, (int(kv_cu[-1]), cfg.n_kv_heads, cfg.head_dim))
    want = np.empty((T, cfg.n_q_heads, cfg.head_dim))
    for i in range(n):
        want[cu[i]:cu[i + 1]] = O.attention_one(
            inputs.bf16_bits_to_f64(q[cu[i]:cu[i + 1]]), inputs.bf16_bits_to_f64(k[kv_cu[i]:kv_cu[i + 1]]),
            inputs.bf16_bits_to_f64(v[kv_cu[i]:kv_cu[i + 1]]), int(prefix_len[i]), 1 / math.sqrt(cfg.head_dim))
    return dict(cu=cu, T=T, table=table, n_pages=n_pages, q=q, k=k, v=v, kv_cu=kv_cu, want=want)


def run_attention(ctx, cfg, c, prefix_len):
    kp, vp = ctx.new_pools(c["n_pages"], 1)
    kp[0].view(torch.int16).fill_(0x7FC0)
    vp[0].view(torch.int16).fill_(0x7FC0)
    d_table = torch.from_numpy(c["table"]).cuda()
    d_kvcu = torch.from_numpy(c["kv_cu"]).cuda()
    zero = torch.zeros(len(prefix_len), dtype=torch.int32, device="cuda")
    ctx.laps_kv_scatter(d_kvcu, zero, d_table, api.bf16_tensor(c["k"]), api.bf16_tensor(c["v"]), kp[0], vp[0])
    out = ctx.laps_attention(torch.from_numpy(c["cu"]).cuda(), None, torch.from_numpy(np.asarray(prefix_len, np.int32)).cuda(),
                             d_table, kp[0], vp[0], api.bf16_tensor(c["q"].reshape(c["T"], -1)))
    torch.cuda.synchronize()
    return out.float().cpu().numpy().reshape(c["want"].shape)


@pytest.mark.parametrize("name,cfgf,new_len,prefix_len", [
    ("tiny_no_prefix", inputs.tiny_cfg, [1, 64, 17, 33, 2, 50], [0, 0, 0, 0, 0, 0]),
    ("tiny_prefix_midpage", inputs.tiny_cfg, [5, 1, 64, 31], [3, 16, 100, 257]),
    ("tiny_many_row_blocks", inputs.tiny_cfg, [200, 70], [0, 130]),
    ("hd128_group5", lambda: inputs.qwen32b_cfg(1), [1, 16, 64, 40, 130], [0, 515, 100, 1, 64]),
    ("hd128_group5_short", lambda: inputs.qwen32b_cfg(1), [1, 16, 20, 8], [0, 515, 100, 1]),
    # few query rows over long prefixes: the key range is split over workgroups and merged (5, 2, 4 and 1 splits)
    ("tiny_key_split", inputs.tiny_cfg, [5, 16, 1, 64], [3000, 1100, 2047, 0]),
    ("hd128_key_split", lambda: inputs.qwen32b_cfg(1), [16, 8, 33], [4100, 1500, 20]),
    # 73 key tiles in 9 splits: the last split is one diagonal tile in which the first 30 tokens see no key
    ("tiny_key_split_rows_without_keys", inputs.tiny_cfg, [64], [4578]),
    # more than 128 query rows per sequence (two or three row blocks walk the same split key range): an odd and an
    # even number of tiles per split, a last row block with few rows, a sequence too short to split
    ("hd128_wide_key_split", lambda: inputs.qwen32b_cfg(1), [40, 64, 30, 52], [4100, 1500, 700, 90]),
    ("tiny_wide_key_split", inputs.tiny_cfg, [150, 100, 129], [3000, 2047, 5]),
    ("hd128_wide_key_split_one_request", lambda: inputs.qwen32b_cfg(1), [64], [4032]),
])
def test_attention_matches_oracle(name, cfgf, new_len, prefix_len):
    cfg = cfgf()
    ctx = api.LapsCtx(cfg, max_positions=1024)
    c = attention_case(cfg, new_len, prefix_len, 11589 + len(name))
    got = run_attention(ctx, cfg, c, prefix_len)
    assert np.all(np.isfinite(got))
    rel, mx = errors(got, c["want"])
    # output and probabilities are bf16: relative error ~2^-9 per element
    assert rel < 4e-3 and mx < 3e-2, (rel, mx)
    ctx.close()


def test_attention_length_one_returns_v_exactly():
    cfg = inputs.tiny_cfg()
    ctx = api.LapsCtx(cfg, max_positions=64)
    c = attention_case(cfg, [1, 1, 1], [0, 0, 0], 3)
    got = run_attention(ctx, cfg, c, [0, 0, 0])
    v = inputs.bf16_bits_to_f64(c["v"])
    for i in range(3):
        for h in range(cfg.n_q_heads):
            assert np.array_equal(got[i, h], v[i, h // (cfg.n_q_heads // cfg.n_kv_heads)])
    ctx.close()


# ----------------------------------------------------------------------------------- layer / stack
def check_stack(case: Case, y_gpu, what=""):
    y, ks, vs, _ = case.oracle()
    rel, mx = errors(y_gpu, y)
    assert np.all(np.isfinite(y_gpu)), what
    assert rel < REL_L2_TOL and mx < MAX_ABS_TOL, (what, rel, mx)
    return y, ks, vs


def test_config1_tiny_layer_matches_oracle():
    """Configuration 1: tiny single layer, 8 new prompts with lengths in [1, 64], no prefix."""
    cfg = inputs.tiny_cfg(1)
    b = inputs.make_batch(1)
    case = Case(cfg, b.new_len, b.prefix_len, inputs.SEED_BASE + 1)
    ctx = api.LapsCtx(cfg, max_positions=256)
    case.to_device(ctx)
    y_gpu = case.run_stack()
    y, ks, vs = check_stack(case, y_gpu, "config1")
    # appended KV equals the oracle's new k, v up to bf16 storage
    kg, vg = case.gathered_new_kv(0)
    kw = np.concatenate(ks[0])
    vw = np.concatenate(vs[0])
    assert errors(kg, kw)[0] < 4e-3 and errors(vg, vw)[0] < 4e-3
    # same through laps_prefill_layer
    y1 = ctx.laps_prefill_layer(case.dev_layers[0], case.d_cu, None, case.d_prefix_len, case.d_page_table,
                                case.k_pools[0], case.v_pools[0], case.d_x)
    torch.cuda.synchronize()
    assert np.array_equal(y1.cpu().numpy(), y_gpu)
    ctx.close()


def test_tiny_stack_with_prefix_and_ragged_tail():
    cfg = inputs.tiny_cfg(3)
    case = Case(cfg, [64, 1, 37, 5, 130, 16], [0, 40, 300, 15, 33, 16], 777)
    ctx = api.LapsCtx(cfg, max_positions=1024)
    case.to_device(ctx)
    y_gpu = case.run_stack()
    check_stack(case, y_gpu, "tiny stack")
    ctx.close()


def test_tiny_stack_with_qkv_bias():
    """The q/k/v projection bias of the model family the paper serves (off in the benchmark configurations):
    a small batch (skinny GEMM path) and a 300-row one (wide tiles), with prefixes, against the oracle; the
    appended keys and values carry the bias too.  A context created without the flag rejects nothing but ignores
    the bias, so the two outputs must differ."""
    cfg = inputs.tiny_cfg(2)
    for lens, pres in (([7, 33, 1], [0, 20, 130]), ([200, 64, 36], [0, 17, 0])):
        case = Case(cfg, lens, pres, 909, qkv_bias=True)
        ctx = api.LapsCtx(cfg, max_positions=512, has_qkv_bias=True)
        case.to_device(ctx)
        y_gpu = case.run_stack()
        _, ks, vs = check_stack(case, y_gpu, "tiny stack with qkv bias")
        k_gpu, v_gpu = case.gathered_new_kv(1)
        k_want = np.concatenate(ks[1])
        v_want = np.concatenate(vs[1])
        assert errors(k_gpu, k_want)[0] < 6e-3 and errors(v_gpu, v_want)[0] < 6e-3
        ctx.close()
        ctx0 = api.LapsCtx(cfg, max_positions=512, has_qkv_bias=False)
        case.to_device(ctx0)
        y_nobias = case.run_stack()
        assert errors(y_nobias, y_gpu)[0] > 1e-2
        ctx0.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_ragged_batches_match_oracle(seed):
    """Seeded random batches at the tiny shape: 1-40 sequences, new lengths 1-150 (a few up to 600), prefixes 0-2500
    with page-boundary cases, so that skinny and wide GEMM tiles, 128- and 256-row attention blocks and the
    key-split path all occur; stack output and appended KV against the oracle."""
    rng = np.random.default_rng(8800 + seed)
    cfg = inputs.tiny_cfg(2)
    ctx = api.LapsCtx(cfg, max_positions=4096)
    for rep in range(4):
        n = int(rng.integers(1, 41)) if rep else 1
        new_len = rng.integers(1, 151, n)
        if rng.random() < 0.5:
            new_len[rng.integers(n)] = int(rng.integers(150, 601))
        prefix = np.where(rng.random(n) < 0.4, 0, rng.choice([1, 15, 16, 17, 63, 64, 65, 255, 256, 1000, 2500], n))
        if n <= 3:
            prefix[0] = int(rng.choice([0, 2047, 2500]))      # few rows over a long prefix: key-split attention
        case = Case(cfg, new_len, prefix, 5000 + 10 * seed + rep).to_device(ctx)
        y_gpu = case.run_stack()
        _, ks, vs = check_stack(case, y_gpu, f"random batch seed {seed} rep {rep}: lens {list(new_len)} prefixes {list(prefix)}")
        k_gpu, v_gpu = case.gathered_new_kv(1)
        assert errors(k_gpu, np.concatenate(ks[1]))[0] < 6e-3 and errors(v_gpu, np.concatenate(vs[1]))[0] < 6e-3
    ctx.close()


def test_cached_prefix_equals_full_prefill_on_device():
    """prefill(prefix || new) == prefill(prefix) followed by re-prefill(new) over the cache written by the first."""
    cfg = inputs.tiny_cfg(2)
    ctx = api.LapsCtx(cfg, max_positions=512)
    lens_full = [90, 33]
    split_at = [50, 16]
    full = Case(cfg, lens_full, [0, 0], 4242).to_device(ctx)
    y_full = full.run_stack()
    # turn 1 and turn 2 share weights, activations and the page table of `full`
    cu_full = full.cu
    x = full.x
    x1 = np.concatenate([x[cu_full[i]:cu_full[i] + split_at[i]] for i in range(2)])
    x2 = np.concatenate([x[cu_full[i] + split_at[i]:cu_full[i + 1]] for i in range(2)])
    kp, vp = ctx.new_pools(full.n_pages, 2)
    for p in kp + vp:
        p.view(torch.int16).fill_(0x7FC0)
    l1 = np.asarray(split_at, np.int32)
    l2 = np.asarray(lens_full, np.int32) - l1
    cu1 = torch.from_numpy(np.concatenate([[0], np.cumsum(l1)]).astype(np.int32)).cuda()
    cu2 = torch.from_numpy(np.concatenate([[0], np.cumsum(l2)]).astype(np.int32)).cuda()
    zero = torch.zeros(2, dtype=torch.int32, device="cuda")
    y1 = ctx.laps_prefill_stack(full.dev_layers, cu1, None, zero, full.d_page_table, kp, vp, torch.from_numpy(x1).cuda())
    y2 = ctx.laps_prefill_stack(full.dev_layers, cu2, None, torch.from_numpy(l1).cuda(), full.d_page_table, kp, vp,
                                torch.from_numpy(x2).cuda())
    torch.cuda.synchronize()
    y1, y2 = y1.cpu().numpy(), y2.cpu().numpy()
    got = np.concatenate([y1[:50], y2[:40], y1[50:], y2[40:]])
    rel, mx = errors(got, y_full)
    assert rel < 2e-3 and mx < MAX_ABS_TOL, (rel, mx)       # only bf16 cache / split-order effects
    y_or, _, _, _ = full.oracle()
    rel, mx = errors(got, y_or)
    assert rel < REL_L2_TOL and mx < MAX_ABS_TOL, (rel, mx)
    ctx.close()


def test_batch_order_and_padding_do_not_change_rows():
    cfg = inputs.tiny_cfg(2)
    ctx = api.LapsCtx(cfg, max_positions=512)
    case = Case(cfg, [13, 16, 7, 1], [20, 0, 37, 5], 99).to_device(ctx)
    y = case.run_stack()
    # padded bucket layout: every sequence owns 16 rows, only seq_len of them real; two extra empty slots
    Lb, depth = 16, 6
    xp = np.zeros((Lb * depth, cfg.hidden), np.float32)
    perm = [2, 0, 3, 1]
    seq_len = np.zeros(depth, np.int32)
    pre = np.zeros(depth, np.int32)
    table = np.zeros((depth, case.page_table.shape[1]), np.int32)
    for slot, i in enumerate(perm):
        xp[slot * Lb: slot * Lb + case.new_len[i]] = case.x[case.cu[i]:case.cu[i + 1]]
        seq_len[slot], pre[slot], table[slot] = case.new_len[i], case.prefix_len[i], case.page_table[i]
    fresh = Case(cfg, [13, 16, 7, 1], [20, 0, 37, 5], 99).to_device(ctx)     # same cache, untouched by the first run
    cu = torch.arange(0, (depth + 1) * Lb, Lb, dtype=torch.int32, device="cuda")
    yp = ctx.laps_prefill_stack(fresh.dev_layers, cu, torch.from_numpy(seq_len).cuda(), torch.from_numpy(pre).cuda(),
                                torch.from_numpy(table).cuda(), fresh.k_pools, fresh.v_pools, torch.from_numpy(xp).cuda())
    torch.cuda.synchronize()
    yp = yp.cpu().numpy()
    for slot, i in enumerate(perm):
        got = yp[slot * Lb: slot * Lb + case.new_len[i]]
        rel, mx = errors(got, y[case.cu[i]:case.cu[i + 1]])
        assert rel < 1e-3 and mx < 5e-3, (i, rel, mx)
    # the padded run appended the same KV
    k0, v0 = case.gathered_new_kv(1)
    k1, v1 = fresh.gathered_new_kv(1)
    assert errors(k1, k0)[0] < 1e-2 and errors(v1, v0)[0] < 1e-2
    ctx.close()


@pytest.mark.parametrize("prefixes", [[0, 33, 100, 7, 16, 250, 0], [0, 2033, 100, 700, 16, 2500, 0]],
                         ids=["short_prefixes", "long_prefixes_key_split"])
def test_graph_replays_match_uncaptured_path(prefixes):
    """Replays of one captured (16, 4) graph with different slot fillings (rows packed, as the graph holds them) are
    bit-equal to the un-captured path run on a padded layout of the same 64 rows.  With the long prefixes the page table is wide enough for the key-split attention: its
    grid is fixed at capture, how many splits a slot uses changes from replay to replay."""
    cfg = inputs.tiny_cfg(2)
    ctx = api.LapsCtx(cfg, max_positions=4096)
    Lb, depth = 16, 4
    case = Case(cfg, [16, 3, 9, 12, 1, 16, 5], prefixes, 1234).to_device(ctx)
    max_pages = case.page_table.shape[1]
    stream = torch.cuda.Stream()
    graph = ctx.laps_graph_capture(case.dev_layers, Lb, depth, max_pages, case.k_pools, case.v_pools, stream)
    assert graph.laps_graph_device_bytes() > 0
    groups = [[0, 1, 2, 3], [4, 5], [6], [3, 2, 1, 0], [5]]
    cu = torch.arange(0, (depth + 1) * Lb, Lb, dtype=torch.int32, device="cuda")
    for rep, ids in enumerate(groups):
        n_real = len(ids)
        xp = np.zeros((depth * Lb, cfg.hidden), np.float32)
        seq_len = np.zeros(depth, np.int32)
        pre = np.zeros(depth, np.int32)
        table = np.zeros((depth, max_pages), np.int32)
        for slot, i in enumerate(ids):
            xp[slot * Lb: slot * Lb + case.new_len[i]] = case.x[case.cu[i]:case.cu[i + 1]]
            seq_len[slot], pre[slot], table[slot] = case.new_len[i], case.prefix_len[i], case.page_table[i]
        d_x = torch.from_numpy(xp).cuda()
        d_sl, d_pre, d_tab = (torch.from_numpy(a).cuda() for a in (seq_len, pre, table))
        # eager result on the same padded layout (program's own work between replays)
        want = ctx.laps_prefill_stack(case.dev_layers, cu, d_sl, d_pre, d_tab, case.k_pools, case.v_pools, d_x)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            packed = torch.cat([d_x[slot * Lb: slot * Lb + int(case.new_len[i])] for slot, i in enumerate(ids)])
            graph.laps_graph_stage(n_real, d_sl[:n_real].contiguous(), d_pre[:n_real].contiguous(),
                                   d_tab[:n_real].contiguous(), packed, stream)
            graph.laps_graph_replay(stream)
            got = torch.empty((packed.shape[0], cfg.hidden), dtype=torch.float32, device="cuda")
            graph.laps_graph_read_output(packed.shape[0], got, stream)
        stream.synchronize()
        row = 0
        for slot, i in enumerate(ids):
            n = int(case.new_len[i])
            a = got[row: row + n].cpu().numpy()
            b = want[slot * Lb: slot * Lb + n].cpu().numpy()
            assert np.array_equal(a, b), (rep, slot)
            row += n
    graph.close()
    ctx.close()


def test_graph_stage_clamps_lengths_to_the_bucket():
    """A staged length above the graph's length bucket is cut to the bucket on the device: rows stay inside the
    graph's buffers, and the result is that of the cut lengths."""
    cfg = inputs.tiny_cfg(1)
    ctx = api.LapsCtx(cfg, max_positions=256)
    case = Case(cfg, [16, 7], [3, 20], 77).to_device(ctx)
    want = case.run_stack()
    stream = torch.cuda.Stream()
    g = ctx.laps_graph_capture(case.dev_layers, 16, 2, case.page_table.shape[1], case.k_pools, case.v_pools, stream)
    too_long = torch.tensor([40, 7], dtype=torch.int32, device="cuda")
    got = torch.empty((23, cfg.hidden), dtype=torch.float32, device="cuda")
    with torch.cuda.stream(stream):
        g.laps_graph_stage(2, too_long, case.d_prefix_len, case.d_page_table, case.d_x, stream)
        g.laps_graph_replay(stream)
        g.laps_graph_read_output(23, got, stream)
    stream.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)
    g.close()
    ctx.close()


def test_prefill_argument_errors(tiny_ctx):
    cfg = inputs.tiny_cfg(1)
    case = Case(cfg, [4], [0], 1).to_device(tiny_ctx)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    import ctypes as C
    arr = tiny_ctx._weights_array(case.dev_layers)
    rc = api.lib().laps_prefill_layer(tiny_ctx._h, arr, C.c_int32(1), C.c_int32(4), api._p(case.d_cu), None,
                                      api._p(case.d_prefix_len), api._p(case.d_page_table), C.c_int32(1),
                                      api._p(case.k_pools[0]), api._p(case.v_pools[0]), api._p(case.d_x), api._p(case.d_x),
                                      api._p(small), C.c_size_t(256), None)
    assert rc == -2 and b"workspace too small" in api.lib().laps_last_error()
    rc = api.lib().laps_prefill_layer(tiny_ctx._h, arr, C.c_int32(0), C.c_int32(4), api._p(case.d_cu), None,
                                      api._p(case.d_prefix_len), api._p(case.d_page_table), C.c_int32(1),
                                      api._p(case.k_pools[0]), api._p(case.v_pools[0]), api._p(case.d_x), api._p(case.d_x),
                                      api._p(small), C.c_size_t(256), None)
    assert rc == -1
    with pytest.raises(api.LapsError):
        api.LapsCtx(inputs.ModelCfg(250, 4, 2, 64, 512, 1), 16)        # hidden not a multiple of 128


def test_many_single_token_sequences_and_scan_over_256():
    """300 sequences of 1-3 tokens: the query-block table is built by a scan that loops over 256-entry
    chunks; length-1 rows without prefix must return v of their kv head through the whole layer."""
    cfg = inputs.tiny_cfg(1)
    rng = np.random.default_rng(17)
    new_len = rng.integers(1, 4, 300)
    prefix = np.where(rng.random(300) < 0.5, 0, rng.integers(1, 40, 300))
    case = Case(cfg, new_len, prefix, 4711)
    ctx = api.LapsCtx(cfg, max_positions=128)
    case.to_device(ctx)
    y_gpu = case.run_stack()
    check_stack(case, y_gpu, "300 tiny sequences")
    ctx.close()


def test_stack_is_deterministic_bit_for_bit():
    """Split-K sums are reduced in slice order and nothing uses atomics: two runs on fresh caches agree bitwise."""
    cfg = inputs.tiny_cfg(2)
    ctx = api.LapsCtx(cfg, max_positions=512)
    a = Case(cfg, [64, 3, 128, 17], [5, 100, 0, 31], 2024).to_device(ctx)
    ya = a.run_stack()
    b = Case(cfg, [64, 3, 128, 17], [5, 100, 0, 31], 2024).to_device(ctx)
    yb = b.run_stack()
    assert np.array_equal(ya, yb)
    ka, va = a.gathered_new_kv(1)
    kb, vb = b.gathered_new_kv(1)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    ctx.close()


def test_graph_stage_rejects_too_many_slots_and_empty_replay_is_harmless():
    cfg = inputs.tiny_cfg(1)
    ctx = api.LapsCtx(cfg, max_positions=64)
    case = Case(cfg, [4, 4], [0, 0], 9).to_device(ctx)
    stream = torch.cuda.Stream()
    g = ctx.laps_graph_capture(case.dev_layers, 16, 2, case.page_table.shape[1], case.k_pools, case.v_pools, stream)
    three = torch.zeros(3, dtype=torch.int32, device="cuda")
    tab = torch.zeros((3, case.page_table.shape[1]), dtype=torch.int32, device="cuda")
    with pytest.raises(api.LapsError):
        g.laps_graph_stage(3, three, three, tab, None, stream)
    with pytest.raises(api.LapsError):                          # more input rows than the graph holds
        g.laps_graph_stage(2, three[:2], three[:2], tab[:2], torch.zeros((33, cfg.hidden), device="cuda"), stream)
    g.laps_graph_stage(0, None, None, None, None, stream)      # all slots empty
    g.laps_graph_replay(stream)
    stream.synchronize()
    kp = case.k_pools[0].view(torch.int16)
    assert bool((kp == 0x7FC0).all())                           # nothing was appended to the poisoned cache
    g.close()
    ctx.close()
