"""Stage-level parity at the real 32B layer shapes: every projection of the layer on the tiles, K splits and
epilogues the layer driver uses for 96 / 128-row short batches and for 2048-row chunks, and the attention of
a 2048-row chunk over 6144 cached keys, each against fp64 evaluated on the same bf16 inputs.

The stack tests at this shape can only be held to the noise floor of the bf16 operand format (see
test_gpu_configs.py); a stage whose inputs are exact bf16 values has no such floor: a GEMM is fp32
accumulation of exact products (relative L2 ~1e-6), the SwiGLU and attention outputs add one bf16 rounding."""
import math

import numpy as np
import pytest
import torch

from oracle import laps_oracle as O
from paper_2601_11589_amd import api, inputs

from gpu_harness import errors

pytestmark = pytest.mark.gpu

D, QD, QKV, INTER = 5120, 5120, 7168, 27648
SHAPES = {"qkv": (QKV, D), "o": (D, QD), "gate_up": (2 * INTER, D), "down": (D, INTER)}


@pytest.fixture(scope="module")
def ctx32():
    ctx = api.LapsCtx(inputs.qwen32b_cfg(1), max_positions=8192 + 64)
    yield ctx
    ctx.close()


def draw(seed, shape, std):
    """bf16 bit patterns of N(0, std^2) values, drawn in float32 in parallel chunks."""
    rng = np.random.default_rng(seed)
    return inputs.f32_to_bf16_bits((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)))


_W = {}


def weight(name):
    """One seeded weight matrix per projection, shared by the row counts (device tensor, fp64 copy)."""
    if name not in _W:
        n, k = SHAPES[name]
        bits = draw(700 + len(name), (n, k), 0.02)
        _W.clear()                        # one fp64 matrix at a time (the widest is 2.3 GB)
        _W[name] = (api.bf16_tensor(bits), inputs.bf16_bits_to_f64(bits))
    return _W[name]


@pytest.mark.parametrize("m", [96, 128, 2048])          # the row counts vary fastest: one weight matrix at a time
@pytest.mark.parametrize("name", ["qkv", "o", "gate_up", "down"])
def test_projection_at_real_shape_matches_fp64_matmul(ctx32, name, m):
    n, k = SHAPES[name]
    info = ctx32.laps_gemm_plan_info(m, n, k, 0, 0)
    print(f"[stage] {name} m={m}: tile {info['bm']}x{info['bn']}, {info['split']} K slices of {info['k_per_split']}, "
          f"{info['ws']} slabs in flight, {info['workgroups']} workgroups", flush=True)
    if m <= 128:      # the streaming tiles: 256 columns for the wide / long-K projections, 128 for the narrow ones
        assert info["bm"] == 128 and info["bn"] == (256 if name in ("gate_up", "down") else 128) and info["ws"] == 2
    else:
        assert info["bm"] == 256 and info["bn"] == {"qkv": 224, "o": 160, "gate_up": 256, "down": 160}[name]
    w_dev, w64 = weight(name)
    a = draw(m * 31 + len(name), (m, k), 1.0)
    got = ctx32.laps_gemm_bf16(api.bf16_tensor(a), w_dev)
    torch.cuda.synchronize()
    want = inputs.bf16_bits_to_f64(a) @ w64.T
    rel, mx = errors(got.cpu().numpy(), want)
    print(f"[stage] {name} m={m}: rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert rel < 2e-6 and mx < 1e-4 * math.sqrt(k) * 0.02 * 4, (rel, mx)


@pytest.mark.parametrize("m", [100, 128, 300, 2048])
def test_fused_residual_epilogue_at_real_shape(ctx32, m):
    """o and down projections with the residual add: fused into the 256x160 tile for chunks, K-slice sums plus the row
    kernel for short batches."""
    for name in ("o", "down"):
        n, k = SHAPES[name]
        info = ctx32.laps_gemm_plan_info(m, n, k, 0, 1)
        assert (info["epi"] == 1) == (info["split"] == 1)
        w_dev, w64 = weight(name)
        a = draw(m * 17 + len(name), (m, k), 1.0)
        resid = np.random.default_rng(m + len(name)).standard_normal((m, n), dtype=np.float32) * 4
        got = ctx32.laps_gemm_epilogue_bf16(api.bf16_tensor(a), w_dev, 1, resid=torch.from_numpy(resid).cuda())
        torch.cuda.synchronize()
        want = resid.astype(np.float64) + inputs.bf16_bits_to_f64(a) @ w64.T
        rel, mx = errors(got.cpu().numpy(), want)
        print(f"[stage] {name}+resid m={m} (tile {info['bm']}x{info['bn']}, split {info['split']}, fused={info['epi'] == 1}): "
              f"rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
        assert rel < 2e-6, (name, m, rel, mx)


@pytest.mark.parametrize("m", [100, 128, 300, 2048])
def test_fused_swiglu_epilogue_at_real_shape(ctx32, m):
    """gate/up projection with the SwiGLU epilogue on packed (32-row interleaved) weights: the streaming 128x256 tile
    and the 256x256 tile both fuse it; the result is one bf16 rounding away from fp64."""
    n, k = SHAPES["gate_up"]
    info = ctx32.laps_gemm_plan_info(m, n, k, 0, 2)
    assert info["epi"] == 2 and info["split"] == 1 and info["bn"] == 256
    rng_seed = 4242
    wg = draw(rng_seed, (INTER, D), 0.02)
    wu = draw(rng_seed + 1, (INTER, D), 0.02)
    packed = ctx32.laps_pack_gate_up(api.bf16_tensor(wg), api.bf16_tensor(wu))
    a = draw(m * 13, (m, k), 1.0)
    got = ctx32.laps_gemm_epilogue_bf16(api.bf16_tensor(a), packed, 2)
    torch.cuda.synchronize()
    a64 = inputs.bf16_bits_to_f64(a)
    want = O.silu(a64 @ inputs.bf16_bits_to_f64(wg).T) * (a64 @ inputs.bf16_bits_to_f64(wu).T)
    g = got.float().cpu().numpy().astype(np.float64)
    rel, mx = errors(g, want)
    print(f"[stage] gate/up+swiglu m={m} (tile {info['bm']}x{info['bn']}): rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert rel < 2.5e-3, (m, rel)                      # bf16 output: 2^-9 / sqrt(3) relative per element
    # element by element: within one bf16 half-ulp of the fp64 value (+ fp32 accumulation slack)
    bound = np.abs(want) * 2.0 ** -8 + 1e-4
    assert np.all(np.abs(g - want) <= bound), float(np.max(np.abs(g - want) - bound))


def test_attention_of_a_2048_row_chunk_over_6144_cached_keys(ctx32):
    """The last chunk of an 8K prompt: 2048 new tokens (256-row query blocks, 5 query heads per kv head packed into
    the rows) over 6144 cached keys in 16-token pages - 128 key tiles per block, the diagonal ones masked."""
    from test_gpu_kernels import attention_case, run_attention
    cfg = inputs.qwen32b_cfg(1)
    new_len, prefix_len = [2048], [6144]
    c = attention_case(cfg, new_len, prefix_len, 11589 + 64)
    got = run_attention(ctx32, cfg, c, prefix_len)
    assert np.all(np.isfinite(got))
    rel, mx = errors(got, c["want"])
    print(f"[stage] attention L=2048 H=6144 hd=128 G=5: rel_l2={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert rel < 4e-3 and mx < 3e-2, (rel, mx)
    # per row: no row may be off by more than the bf16 probability / output rounding explains
    err_row = np.linalg.norm((got - c["want"]).reshape(2048, -1), axis=1)
    ref_row = np.linalg.norm(c["want"].reshape(2048, -1), axis=1)
    assert np.all(err_row <= 8e-3 * ref_row), float(np.max(err_row / ref_row))
