"""Full-size parity: the benchmark configurations at the 32B layer shape, in the launch
configurations bench.py times (captured bucket graphs for short batches, 2048-token chunks for
long prompts), checked against the fp64 oracle on sampled sequences.  A sequence's output depends
only on its own tokens and its own cached prefix (pinned for the oracle in test_oracle_layer.py),
so the oracle can check any subset one by one.

Tolerance.  The stated bar is relative L2 <= 5e-3 and max-abs <= 2e-2 against the pure fp64 oracle.
At the 32B shape that bar cannot be met by ANY arithmetic that keeps the declared bf16 storage
points (normed rows, q, k, v, attention output, MLP activation - the MFMA operands and the cache):
the fp64 oracle with only those roundings applied already deviates from the pure oracle by ~5.7e-3
relative L2 per layer (max-abs ~0.13), because each bf16 rounding injects ~1.6e-3 relative noise and
the MLP branch (std ~4.3) amplifies it.  So here the tests (a) always print the error against the
pure oracle and say whether the stated bar is met, and (b) hold the device error to the deviation that
the declared storage points alone produce in fp64 arithmetic on the same inputs, at three grains:
relative L2 of the sample and of every sequence within 1.1x, the error norm of every row within 1.25x,
and every single element within 7.5 standard deviations of its row's noise (assert_parity) - i.e. the
kernels add nothing beyond the bf16 operand format, and one wrong value of a few tenths fails.  The
stages themselves (every projection at its real tiles, the fused epilogues, attention of a 2048-row
chunk over 6144 cached keys, the appended K/V) meet fp64 without such a floor in test_gpu_stages_32b.py
and assert_new_kv.  The tiny configuration meets the stated bar outright (test_gpu_kernels.py).
"""
import os

import numpy as np
import pytest
import torch

from paper_2601_11589_amd import api, inputs, runner

from gpu_harness import MAX_ABS_TOL, REL_L2_TOL, Case, errors

pytestmark = pytest.mark.gpu

LEN_BUCKETS = [16, 32, 64]
DEPTHS = [1, 2, 4, 8, 16, 32, 64]


# Measured on MI355X over all configurations: a row's error norm is 1.00-1.12 x its floor (median 1.005), a
# sequence's 1.00-1.01 x, and the largest single deviation is 5.3-6.2 standard deviations of its row's noise (the
# extreme of ~2e7 Gaussian-like values).  The factors below leave a small margin over that.
ROW_FACTOR = 1.25    # a row's error norm may exceed the noise floor of that row by this factor
SEQ_FACTOR = 1.1     # a sequence's (and the whole sample's) relative L2 error, likewise
ELEM_SIGMAS = 7.5    # no element may be off by more than this many standard deviations of its row's noise


def assert_parity(tag, got, case, seqs, oracle_cache=None):
    """Returns (rel, max_abs, rel_floor): device-vs-pure errors and the storage-point noise floor.
    oracle_cache: dict reused when several device runs are checked against the same oracle outputs.

    Checked against the pure fp64 oracle y, with the deviation of the fp64 oracle that applies the declared bf16
    storage points (ys) as the noise floor of the operand format:
      * the whole sample and every sequence: relative L2 <= max(stated bar, SEQ_FACTOR x floor of that sequence);
      * every row: error norm <= ROW_FACTOR x the floor's error norm of that row (or the stated bar);
      * every element: |error| <= ELEM_SIGMAS x the per-element noise of its row (floor error norm / sqrt(d)), or the
        stated max-abs bar - so a single wrong value of a few tenths fails, where a pooled max-abs bound of twice
        the floor's extreme value would let it pass."""
    if oracle_cache is not None and "y" in oracle_cache:
        y, ys = oracle_cache["y"], oracle_cache["ys"]
    else:
        y, ks, vs, rows = case.oracle(seqs=seqs)
        ys, _, _, _ = case.oracle(storage_rounding=True, seqs=seqs)
        if oracle_cache is not None:
            oracle_cache.update(y=y, ys=ys, ks=ks, vs=vs)
    got = np.asarray(got, np.float64)
    rel, mx = errors(got, y)
    rel_f, mx_f = errors(ys, y)
    strict = rel < REL_L2_TOL and mx < MAX_ABS_TOL
    assert np.all(np.isfinite(got))
    d = y.shape[1]
    err_row = np.linalg.norm(got - y, axis=1)
    flo_row = np.linalg.norm(ys - y, axis=1)
    ref_row = np.linalg.norm(y, axis=1)
    row_ratio = err_row / np.maximum(flo_row, 1e-300)
    sigma = np.maximum(flo_row, err_row * 0) / np.sqrt(d)
    z = np.abs(got - y) / np.maximum(sigma[:, None], 1e-300)
    print(f"[parity] {tag}: device vs fp64 oracle rel_l2={rel:.3e} max_abs={mx:.3e} | bf16 storage points alone "
          f"(fp64 arithmetic) rel_l2={rel_f:.3e} max_abs={mx_f:.3e} | stated bar (5e-3, 2e-2) "
          f"{'MET' if strict else 'NOT met (bf16 operand noise)'} | per row: error / floor max {row_ratio.max():.3f} "
          f"median {np.median(row_ratio):.3f}; per element: max {z.max():.2f} sigma of its row's noise", flush=True)
    assert rel < max(REL_L2_TOL, SEQ_FACTOR * rel_f), (tag, rel, rel_f)
    ids = list(range(case.n)) if seqs is None else list(seqs)
    o = 0
    for i in ids:
        n = int(case.new_len[i])
        r_s, _ = errors(got[o:o + n], y[o:o + n])
        f_s, _ = errors(ys[o:o + n], y[o:o + n])
        assert r_s < max(REL_L2_TOL, SEQ_FACTOR * f_s), (tag, "sequence", i, r_s, f_s)
        o += n
    assert o == got.shape[0]
    bad_rows = err_row > np.maximum(ROW_FACTOR * flo_row, REL_L2_TOL * ref_row)
    assert not bad_rows.any(), (tag, "rows", np.nonzero(bad_rows)[0][:8], row_ratio[bad_rows][:8])
    bad = np.abs(got - y) > np.maximum(ELEM_SIGMAS * sigma[:, None], MAX_ABS_TOL)
    assert not bad.any(), (tag, "elements", int(bad.sum()), float(z.max()))
    return rel, mx, rel_f


def assert_new_kv(tag, case, layer, seqs, ks, vs):
    """Appended K and V of `layer` for the sampled sequences against the oracle's: at layer 0 two roundings (the normed
    row, the stored value) separate them, deeper layers inherit the noise of the residual stream."""
    k_gpu, v_gpu = case.gathered_new_kv(layer)
    for what, g, want in (("k", k_gpu, ks), ("v", v_gpu, vs)):
        got = np.concatenate([g[case.cu[i]:case.cu[i + 1]] for i in seqs])
        rel, mx = errors(got, np.concatenate(want))
        print(f"[parity] {tag}: appended {what} of layer {layer}: rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
        assert rel < 4e-3, (tag, what, rel)
        # element by element: one bf16 half-ulp of the stored value plus the propagated rounding of the normed row
        w = np.concatenate(want)
        assert np.all(np.abs(got - w) <= np.abs(w) * 2.0 ** -8 + 0.03), (tag, what, float(np.max(np.abs(got - w))))


@pytest.fixture(scope="module")
def model():
    """4 layers at the 32B shape (seeded), uploaded once for the whole module."""
    cfg = inputs.qwen32b_cfg(4)
    ctx = api.LapsCtx(cfg, max_positions=8192 + 64)
    seed = inputs.SEED_BASE + 2
    host_layers = [inputs.make_layer_weights(cfg, seed, l, threads=min(16, os.cpu_count() or 8)) for l in range(4)]
    dev_layers = [ctx.upload_layer(w) for w in host_layers]
    yield cfg, ctx, host_layers, dev_layers
    ctx.close()


class SharedCase(Case):
    """A Case that reuses the module's weights instead of drawing its own."""

    def __init__(self, cfg, new_len, prefix_len, seed, host_layers, dev_layers, prefix_for=None):
        self.cfg, self.n_layers = cfg, cfg.n_layers
        self.new_len = np.asarray(new_len, np.int32)
        self.prefix_len = np.asarray(prefix_len, np.int32)
        self.seed, self.n = seed, len(new_len)
        self.cu = np.concatenate([[0], np.cumsum(self.new_len)]).astype(np.int32)
        self.T = int(self.cu[-1])
        self.page_table, self.n_pages = inputs.make_page_table(seed, self.new_len, self.prefix_len)
        self.host_layers, self.dev_layers = host_layers, dev_layers
        self.x = inputs.make_activations(cfg, seed, self.T)
        self.prefix = [[inputs.make_prefix_kv(cfg, seed, l, i, int(h)) if h > 0 else None
                        for i, h in enumerate(self.prefix_len)] for l in range(self.n_layers)]

    def to_device(self, ctx):
        dl = self.dev_layers
        self.upload = None
        # Case.to_device re-uploads weights; skip that part
        self.ctx = ctx
        self.k_pools, self.v_pools = ctx.new_pools(self.n_pages, self.n_layers)
        for p in self.k_pools + self.v_pools:
            p.view(torch.int16).fill_(0x7FC0)
        self.d_cu = torch.from_numpy(self.cu).cuda()
        self.d_prefix_len = torch.from_numpy(self.prefix_len).cuda()
        self.d_page_table = torch.from_numpy(self.page_table).cuda()
        self.d_x = torch.from_numpy(self.x).cuda()
        pcu = np.concatenate([[0], np.cumsum(self.prefix_len)]).astype(np.int32)
        if pcu[-1] > 0:
            d_pcu = torch.from_numpy(pcu).cuda()
            d_zero = torch.zeros(self.n, dtype=torch.int32, device="cuda")
            for l in range(self.n_layers):
                kk = np.concatenate([self.prefix[l][i][0] for i in range(self.n) if self.prefix[l][i] is not None])
                vv = np.concatenate([self.prefix[l][i][1] for i in range(self.n) if self.prefix[l][i] is not None])
                ctx.laps_kv_scatter(d_pcu, d_zero, self.d_page_table, api.bf16_tensor(kk), api.bf16_tensor(vv),
                                    self.k_pools[l], self.v_pools[l])
        self.dev_layers = dl
        torch.cuda.synchronize()
        return self


def run_planned_short(case, cfg, ctx, token_budget, len_buckets=LEN_BUCKETS):
    """Plan -> stage -> replay every short batch as a captured graph; returns y per request."""
    plan = api.laps_plan_buckets(len_buckets[-1], len_buckets, DEPTHS, token_budget, 2048, case.new_len, case.prefix_len)
    assert not plan["longs"]
    staged = runner.stage_short_batches(plan, case.new_len, case.prefix_len, case.page_table, case.cu, case.d_x, cfg.hidden)
    stream = torch.cuda.Stream()
    sr = runner.ShortRunner(ctx, case.dev_layers, case.k_pools, case.v_pools, case.page_table.shape[1], stream)
    ys = {}
    for sb in staged:
        out = torch.empty((sb.real_tokens, cfg.hidden), dtype=torch.float32, device="cuda")
        sr.run(sb, out)
        stream.synchronize()
        o = out.cpu().numpy()
        row = 0
        for i in sb.req_ids:
            ys[i] = o[row: row + int(case.new_len[i])]
            row += int(case.new_len[i])
    sr.close()
    return ys, plan


def test_config2_short_buckets_as_graphs(model):
    """256 new prompts U[8,64] in buckets {16,32,64}, token_budget 128, one graph per shape."""
    cfg, ctx, host_layers, dev_layers = model
    b = inputs.make_batch(2)
    case = SharedCase(cfg, b.new_len, b.prefix_len, inputs.SEED_BASE + 2, host_layers, dev_layers).to_device(ctx)
    ys, plan = run_planned_short(case, cfg, ctx, 128)
    assert sorted(ys) == list(range(256))
    assert all(np.all(np.isfinite(v)) for v in ys.values())
    order = np.argsort(b.new_len)
    # 36 of the 256 requests: the shortest and longest, every 8th in arrival order, and the first and last
    sample = sorted({int(order[0]), int(order[-1]), int(order[128]), 0, 255, 100} | set(range(3, 256, 8)))
    assert len(sample) >= 32
    got = np.concatenate([ys[i] for i in sample])
    cache = {}
    _, _, floor = assert_parity(f"config2 ({len(sample)} sampled requests, graphs, budget 128)", got, case, sample, cache)
    _, ks, vs, _ = case.oracle(seqs=sample[:8])
    assert_new_kv("config2", case, 0, sample[:8], ks[0], vs[0])
    # token-max variant (large depths): same requests, same answers up to split-order effects
    case2 = SharedCase(cfg, b.new_len, b.prefix_len, inputs.SEED_BASE + 2, host_layers, dev_layers).to_device(ctx)
    ys2, _ = run_planned_short(case2, cfg, ctx, 4096)
    got2 = np.concatenate([ys2[i] for i in sample])
    assert_parity(f"config2 ({len(sample)} sampled requests, graphs, budget 4096)", got2, case2, sample, cache)
    rel, mx = errors(got2, got)      # two valid bf16 evaluations differ by about sqrt(2) x the noise floor
    print(f"[parity] config2 budget 4096 vs budget 128 on device: rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert rel < 2.0 * floor, (rel, floor)


def test_config3_reprefill_over_paged_prefix(model):
    """Multi-turn re-prefill: cached bf16 prefix U[512,4096] in 16-token pages + new tokens U[16,64].
    A seeded subset of the 128 requests keeps host time and memory bounded; the page pool is still
    one random permutation so pages interleave across requests."""
    cfg, ctx, host_layers, dev_layers = model
    b = inputs.make_batch(3)
    keep = [0, 17, 41, 63, 77, 90, 101, 127]
    shortest, longest = int(np.argmin(b.prefix_len)), int(np.argmax(b.prefix_len))
    keep = sorted(set(keep + [shortest, longest]))
    case = SharedCase(cfg, b.new_len[keep], b.prefix_len[keep], inputs.SEED_BASE + 3, host_layers, dev_layers).to_device(ctx)
    # (a) one packed varlen batch, un-captured
    y = case.run_stack()
    cache = {}
    assert_parity(f"config3 varlen batch (all {len(keep)} kept requests)", y, case, None, cache)
    _, ks, vs, _ = case.oracle(seqs=[0, len(keep) - 1])
    assert_new_kv("config3", case, 0, [0, len(keep) - 1], ks[0], vs[0])
    # (b) the same requests through captured bucket graphs
    case_g = SharedCase(cfg, b.new_len[keep], b.prefix_len[keep], inputs.SEED_BASE + 3, host_layers, dev_layers).to_device(ctx)
    ys, _ = run_planned_short(case_g, cfg, ctx, 128)
    got = np.concatenate([ys[i] for i in range(len(keep))])
    assert_parity(f"config3 bucket graphs (all {len(keep)} kept requests)", got, case_g, None, cache)


def test_prefix_cache_equivalence_at_full_shape(model):
    """prefill(prefix || new) == prefill(prefix) then re-prefill(new) over the cache the first pass wrote."""
    cfg, ctx, host_layers, dev_layers = model
    H, L = 530, 45
    full = SharedCase(cfg, [H + L], [0], 31337, host_layers, dev_layers).to_device(ctx)
    y_full = full.run_stack()
    two = SharedCase(cfg, [H + L], [0], 31337, host_layers, dev_layers).to_device(ctx)
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    cu1 = torch.tensor([0, H], dtype=torch.int32, device="cuda")
    cu2 = torch.tensor([0, L], dtype=torch.int32, device="cuda")
    y1 = ctx.laps_prefill_stack(dev_layers, cu1, None, zero, two.d_page_table, two.k_pools, two.v_pools, two.d_x[:H].contiguous())
    y2 = ctx.laps_prefill_stack(dev_layers, cu2, None, torch.tensor([H], dtype=torch.int32, device="cuda"), two.d_page_table,
                                two.k_pools, two.v_pools, two.d_x[H:].contiguous())
    torch.cuda.synchronize()
    got = np.concatenate([y1.cpu().numpy(), y2.cpu().numpy()])
    rel, mx = errors(got, y_full)
    print(f"[parity] prefix-cache equivalence on device: rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
    _, _, floor = assert_parity("full prefill of prefix||new (575 tokens)", y_full, full, [0])
    assert rel < 2.0 * floor, (rel, floor)


def test_config4_long_prefill_in_chunks(model):
    """8 prompts U[1024,8192] in 2048-token chunks; the oracle (unchunked) checks the shortest prompt (one chunk)
    and the 3251-token one (two chunks: 1203 rows attending to 2048 cached keys that the first chunk appended),
    the others are checked for finiteness and against an unchunked device pass of a mid-size prompt.  Attention
    over longer cached ranges (2048 rows over 6144 keys) meets the oracle in test_gpu_stages_32b.py."""
    cfg, ctx, host_layers, dev_layers = model
    b = inputs.make_batch(4)
    case = SharedCase(cfg, b.new_len, b.prefix_len, inputs.SEED_BASE + 4, host_layers, dev_layers).to_device(ctx)
    plan = api.laps_plan_buckets(64, LEN_BUCKETS, DEPTHS, 128, 2048, case.new_len, case.prefix_len)
    assert len(plan["longs"]) == 8
    stream = torch.cuda.Stream()
    out = torch.empty_like(case.d_x)
    ctx.workspace(int(case.new_len.max()), 1)
    keep = []
    for lg in plan["longs"]:
        i = lg["req_id"]
        assert sum(lg["chunks"]) == case.new_len[i] and all(c == 2048 for c in lg["chunks"][:-1])
        keep += runner.run_long_chunks(ctx, dev_layers, case.k_pools, case.v_pools, case.d_x[case.cu[i]:case.cu[i + 1]], 0,
                               case.d_page_table[i:i + 1], lg["chunks"], stream, out[case.cu[i]:case.cu[i + 1]])
    stream.synchronize()
    y = out.cpu().numpy()
    assert np.all(np.isfinite(y))
    i0 = int(np.argmin(case.new_len))
    _, _, floor = assert_parity(f"config4 shortest prompt ({case.new_len[i0]} tokens, chunked)",
                                y[case.cu[i0]:case.cu[i0 + 1]], case, [i0])
    # appended K/V of the shortest prompt (1090 rows: the 256-row projection tiles, one K slice, then RoPE + append)
    _, ks, vs, _ = case.oracle(seqs=[i0])
    assert_new_kv("config4", case, 0, [i0], ks[0], vs[0])
    i1 = int(np.argsort(case.new_len)[1])
    assert case.new_len[i1] > 2048
    assert_parity(f"config4 second shortest prompt ({case.new_len[i1]} tokens in 2 chunks) vs the unchunked oracle",
                  y[case.cu[i1]:case.cu[i1 + 1]], case, [i1])
    # chunked == unchunked on the device for the same prompt
    solo = SharedCase(cfg, [case.new_len[i1]], [0], inputs.SEED_BASE + 4, host_layers, dev_layers)
    solo.x = case.x[case.cu[i1]:case.cu[i1 + 1]]
    solo.to_device(ctx)
    y_un = solo.run_stack()
    rel, mx = errors(y[case.cu[i1]:case.cu[i1 + 1]], y_un)
    print(f"[parity] config4 chunked vs unchunked on device ({case.new_len[i1]} tokens): rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert rel < 2.0 * floor, (rel, floor)


def test_config4_longest_prompt_in_four_chunks_through_the_stack(model):
    """The longest prompt of the configuration (7991 tokens) in four chunks through all four layers, against the
    unchunked oracle: the last chunk's 1847 rows attend to 6144 keys that the three chunks before it appended, at
    every layer, in the launch shapes of the long-prefill workload.  The fp64 side (the pure oracle and the one with
    the bf16 storage points) takes a few minutes of host time; it is the only check of this depth at this length."""
    cfg, ctx, host_layers, dev_layers = model
    b = inputs.make_batch(4)
    i = int(np.argmax(b.new_len))
    n = int(b.new_len[i])
    assert n > 3 * 2048
    case = SharedCase(cfg, [n], [0], inputs.SEED_BASE + 4, host_layers, dev_layers).to_device(ctx)
    plan = api.laps_plan_buckets(64, LEN_BUCKETS, DEPTHS, 128, 2048, case.new_len, case.prefix_len)
    chunks = plan["longs"][0]["chunks"]
    assert len(chunks) == 4 and sum(chunks) == n
    stream = torch.cuda.Stream()
    out = torch.empty_like(case.d_x)
    ctx.workspace(2048, 1)
    keep = runner.run_long_chunks(ctx, dev_layers, case.k_pools, case.v_pools, case.d_x, 0, case.d_page_table[0:1],
                                  chunks, stream, out)
    stream.synchronize()
    cache = {}
    assert_parity(f"config4 longest prompt ({n} tokens in 4 chunks, {cfg.n_layers} layers) vs the unchunked oracle",
                  out.cpu().numpy(), case, [0], cache)
    assert_new_kv("config4 longest prompt", case, 0, [0], cache["ks"][0], cache["vs"][0])
    del keep


@pytest.mark.parametrize("name,cfgf", [("7B", inputs.qwen7b_cfg), ("14B", inputs.qwen14b_cfg)])
def test_wider_bucket_grid_on_smaller_model_shapes(name, cfgf):
    """The length grid the paper gives as an example (8 ... 256, Section 3.1) on the 7B- and 14B-shaped layers it
    also serves (Numerical Results): every request of a mixed new-prompt / re-prefill set runs in a captured
    (bucket, depth) graph and is checked against the oracle.  The 7B shape has 7 query heads per kv head."""
    cfg = cfgf(2)
    ctx = api.LapsCtx(cfg, max_positions=4096 + 256)
    seed = inputs.SEED_BASE + 40 + len(name)
    host_layers = [inputs.make_layer_weights(cfg, seed, l, threads=min(16, os.cpu_count() or 8)) for l in range(2)]
    dev_layers = [ctx.upload_layer(w) for w in host_layers]
    rng = np.random.default_rng(seed)
    new_len = np.array([1, 8, 9, 100, 128, 129, 255, 256, 33, 64, 17, 200], np.int32)
    prefix_len = np.array([0, 0, 700, 0, 15, 2049, 0, 1, 3000, 16, 0, 640], np.int32)
    case = SharedCase(cfg, new_len, prefix_len, seed, host_layers, dev_layers).to_device(ctx)
    ys, plan = run_planned_short(case, cfg, ctx, 512, len_buckets=[8, 16, 32, 64, 128, 256])
    assert sorted(i for b in plan["batches"] for i in b["req_ids"]) == list(range(case.n))
    assert {b["len_bucket"] for b in plan["batches"]} == {8, 16, 32, 64, 128, 256}
    got = np.concatenate([ys[i] for i in range(case.n)])
    assert_parity(f"{name} shape, buckets 8..256, {len(plan['batches'])} graphs", got, case, None)
    ctx.close()


@pytest.fixture(scope="module")
def model8():
    """8 layers at the 32B shape for the mixed dual-queue configuration."""
    cfg = inputs.qwen32b_cfg(8)
    ctx = api.LapsCtx(cfg, max_positions=8192 + 64)
    seed = inputs.SEED_BASE + 5
    host_layers = [inputs.make_layer_weights(cfg, seed, l, threads=min(16, os.cpu_count() or 8)) for l in range(8)]
    dev_layers = [ctx.upload_layer(w) for w in host_layers]
    yield cfg, ctx, host_layers, dev_layers
    ctx.close()


class Config5State:
    pass


@pytest.fixture(scope="module")
def config5(model8):
    """configs[4] resident in HBM: 4 long prompts + 512 short / re-prefill requests on the 8-layer stack, with
    nine sampled requests (2 fresh short prompts, 6 re-prefills from the shortest to the longest cached prefix, and
    the shortest long prompt) whose prefix KV is seeded from the host so that the oracle can follow them."""
    from paper_2601_11589_amd import dualqueue
    cfg, ctx, host_layers, dev_layers = model8
    st = Config5State()
    seed = inputs.SEED_BASE + 5
    b = inputs.make_batch(5)
    x = inputs.make_activations(cfg, seed, b.n_tokens)
    d_x = torch.from_numpy(x).cuda()
    k_pools, v_pools = ctx.new_pools(b.n_pages, 8)
    gen = torch.Generator(device="cuda").manual_seed(seed)
    for p in k_pools + v_pools:                    # un-sampled requests: any finite cache content will do
        p.copy_(torch.randn(p.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16))
    is_long = b.new_len > 64
    shorts = np.nonzero(~is_long)[0]
    fresh = [int(i) for i in shorts if b.prefix_len[i] == 0][:2]
    with_pre = sorted((int(i) for i in shorts if b.prefix_len[i] > 0), key=lambda i: int(b.prefix_len[i]))
    spread = [with_pre[int(q * (len(with_pre) - 1))] for q in (0.0, 0.2, 0.4, 0.6, 0.8, 1.0)]   # shortest .. longest prefix
    sample = fresh + spread + [int(min(np.nonzero(is_long)[0], key=lambda i: b.new_len[i]))]
    assert len(set(sample)) == len(sample) == 9
    # the sampled requests get seeded host-side prefix KV, written into their pages of the big pools
    sub = SharedCase(cfg, b.new_len[sample], b.prefix_len[sample], seed, host_layers, dev_layers)
    cu_all = b.cu_seqlens
    sub.x = np.concatenate([x[cu_all[i]:cu_all[i + 1]] for i in sample])
    pcu = np.concatenate([[0], np.cumsum(sub.prefix_len)]).astype(np.int32)
    d_pt_sample = torch.from_numpy(np.ascontiguousarray(b.page_table[sample])).cuda()
    for l in range(8):
        kk = np.concatenate([sub.prefix[l][j][0] for j in range(len(sample)) if sub.prefix[l][j] is not None])
        vv = np.concatenate([sub.prefix[l][j][1] for j in range(len(sample)) if sub.prefix[l][j] is not None])
        ctx.laps_kv_scatter(torch.from_numpy(pcu).cuda(), torch.zeros(len(sample), dtype=torch.int32, device="cuda"),
                            d_pt_sample, api.bf16_tensor(kk), api.bf16_tensor(vv), k_pools[l], v_pools[l])
    torch.cuda.synchronize()
    st.dq = dualqueue.DualQueue(ctx, dev_layers, b.new_len, b.prefix_len, b.page_table, d_x, k_pools, v_pools,
                                dualqueue.DQParams(), keep_outputs=True)
    st.b, st.is_long, st.sub, st.seed, st.cache, st.unified_makespan_us = b, is_long, sub, seed, {}, None
    st.sampled_rows = lambda: np.concatenate([st.dq.out[cu_all[i]:cu_all[i + 1]].cpu().numpy() for i in sample])
    yield st
    st.dq.close()


def test_config5_dual_queue_step_loop(config5):
    """Temporal disaggregation (short buckets as graphs, long chunks) and the unified mixed-batch baseline both
    reproduce the oracle on sampled requests; every request completes exactly once."""
    st, dq, b, is_long = config5, config5.dq, config5.b, config5.is_long
    zeros = np.zeros(b.n)
    rd = dq.run_disaggregated(zeros, window_us=0.0)
    assert_parity("config5 disaggregated (8 short + shortest long)", st.sampled_rows(), st.sub, None, st.cache)
    dq.out.zero_()
    ru = dq.run_unified(zeros)
    assert_parity("config5 unified mixed batches (same requests)", st.sampled_rows(), st.sub, None, st.cache)
    # memory-based batching that takes long prompts whole (Section 2.3): batches of up to 16384 rows, a 2K-8K prompt
    # and hundreds of short sequences in one launch
    dq.out.zero_()
    rv = dq.run_unified(zeros, budget=16384)
    assert_parity("config5 unified, long prompts whole (same requests)", st.sampled_rows(), st.sub, None, st.cache)
    assert rv.n_steps < ru.n_steps
    for r in (rd, ru, rv):
        assert np.all(r.finish_us > 0) and np.all(r.latency_us > 0)
        print("[config5]", r.summary(b.new_len, is_long), flush=True)
    assert rd.step_kinds["long_chunk"] == int(sum(-(-int(l) // 2048) for l in b.new_len[is_long]))
    st.unified_makespan_us = ru.makespan_us
    # Poisson arrivals at 0.7 of the unified back-to-back service rate: both policies still finish everything
    arr = inputs.poisson_arrivals_us(st.seed, b.n, 0.7 * b.n / (ru.makespan_us * 1e-6)).astype(np.float64)
    rd2 = dq.run_disaggregated(arr, window_us=1000.0)
    ru2 = dq.run_unified(arr)
    for r in (rd2, ru2):
        assert np.all(r.finish_us >= arr) and r.makespan_us >= arr.max()
        print("[config5 poisson]", r.summary(b.new_len, is_long), flush=True)


def test_config5_awd_policy(config5):
    """The short queue batched by the library's Adaptive-Wait-Depth state (Algorithm 1): one captured graph per
    dispatch, mixed buckets padded to the largest one; sampled outputs reproduce the oracle, every request
    completes once, and under Poisson arrivals with deadlines the SLA trigger fires before the deadline passes."""
    st, dq, b, is_long = config5, config5.dq, config5.b, config5.is_long
    dq.out.zero_()
    ra = dq.run_awd(np.zeros(b.n))
    assert_parity("config5 AWD deadline-free (8 short + shortest long)", st.sampled_rows(), st.sub, None, st.cache)
    assert np.all(ra.finish_us > 0)
    assert ra.step_kinds["long_chunk"] == int(sum(-(-int(l) // 2048) for l in b.new_len[is_long]))
    assert ra.step_kinds["dispatch_reasons"].get("depth", 0) >= 1          # all waiting at t=0: rounds fill D at once
    print("[config5 awd]", ra.summary(b.new_len, is_long), flush=True)
    base = st.unified_makespan_us or ra.makespan_us
    arr = inputs.poisson_arrivals_us(st.seed, b.n, 0.7 * b.n / (base * 1e-6)).astype(np.float64)
    ddl = arr + 60_000.0
    for sla_window in (False, True):
        r = dq.run_awd(arr, ddl_us=ddl, s_hat_us=3000.0, sigma_us=1000.0, w_min_us=200.0, w_max_us=10_000.0,
                       t_max_us=30_000.0, delta_us=500.0, sla_window=sla_window)
        assert np.all(r.finish_us >= arr) and r.makespan_us >= arr.max()
        assert 200.0 <= r.step_kinds["final_W_us"] <= 10_000.0 and r.step_kinds["final_D"] >= 1
        print("[config5 awd poisson]", r.summary(b.new_len, is_long), flush=True)
