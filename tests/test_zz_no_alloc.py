"""The entry point for callers that cannot allocate (laps_prefill_stack_static): same kernels as laps_prefill_stack
with the library's static device array as workspace.  Two calls in a row, the second on a smaller batch, each
bit-equal to the existing entry point on the same inputs and fresh caches; a batch whose workspace exceeds the array
is rejected."""
import numpy as np
import pytest
import torch

from paper_2601_11589_amd import api, inputs

from gpu_harness import MAX_ABS_TOL, REL_L2_TOL, Case, errors

pytestmark = pytest.mark.gpu


def run_both(ctx, cfg, new_len, prefix_len, seed):
    ref = Case(cfg, new_len, prefix_len, seed).to_device(ctx)
    want = ref.run_stack()                               # laps_prefill_stack, caller-owned workspace
    k_ref, v_ref = ref.gathered_new_kv(cfg.n_layers - 1)
    st = Case(cfg, new_len, prefix_len, seed).to_device(ctx)   # same inputs, caches untouched by the first run
    out = torch.full_like(st.d_x, float("nan"))
    torch.cuda.synchronize()
    ctx.laps_prefill_stack_static(st.dev_layers, st.d_cu, None, st.d_prefix_len, st.d_page_table, st.k_pools, st.v_pools,
                                  st.d_x, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    k_st, v_st = st.gathered_new_kv(cfg.n_layers - 1)
    return ref, want, got, (k_ref, v_ref), (k_st, v_st)


def test_static_scratch_entry_point_matches_prefill_stack_twice():
    cfg = inputs.tiny_cfg(2)
    ctx = api.LapsCtx(cfg, max_positions=4096)
    assert api.lib().laps_static_scratch_bytes() == 128 << 20
    # first call: 300 rows (wide GEMM tiles, split-K partial sums in the scratch, un-split attention);
    # second call, smaller: 25 rows over long prefixes (skinny tiles, key-split attention partials in the scratch)
    for new_len, prefix_len, seed in (([130, 64, 7, 99], [0, 40, 300, 15], 4401), ([16, 8, 1], [2100, 0, 1500], 4402)):
        ref, want, got, kv_ref, kv_st = run_both(ctx, cfg, new_len, prefix_len, seed)
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, want), errors(got, want)          # same kernels, same launch plan: bit-equal
        assert np.array_equal(kv_st[0], kv_ref[0]) and np.array_equal(kv_st[1], kv_ref[1])
        y, _, _, _ = ref.oracle()
        rel, mx = errors(got, y)
        assert rel < REL_L2_TOL and mx < MAX_ABS_TOL, (rel, mx)
    ctx.close()


def test_static_scratch_entry_point_rejects_batches_beyond_the_array():
    cfg = inputs.qwen32b_cfg(1)
    ctx = api.LapsCtx(cfg, max_positions=64)
    n_tok = 4096                                          # its workspace is far beyond 128 MiB at this shape
    assert ctx.laps_workspace_bytes(n_tok, 1) > api.lib().laps_static_scratch_bytes()
    x = torch.zeros((n_tok, cfg.hidden), dtype=torch.float32, device="cuda")
    cu = torch.tensor([0, n_tok], dtype=torch.int32, device="cuda")
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    pt = torch.zeros((1, n_tok // 16), dtype=torch.int32, device="cuda")
    kp, vp = ctx.new_pools(n_tok // 16, 1, zero=True)
    w = {k: torch.zeros(1, dtype=torch.bfloat16, device="cuda") for k in ("ln1", "w_qkv", "w_o", "ln2", "w_gate_up", "w_down")}
    with pytest.raises(api.LapsError, match="static scratch"):
        ctx.laps_prefill_stack_static([w], cu, None, zero, pt, kp, vp, x, x)
    ctx.close()
