"""Seeded synthetic inputs for the ragged-prefill hot path.

This module serves both the CPU oracle's tests and the HIP path's tests and bench.
It holds none of the layer arithmetic: only random draws, bf16 storage conversion
of those draws, length mixes and page-table shuffles.  The workloads stand in for
the multi-turn chat traces the paper evaluates on (Experiments, "Our evaluations
focus on multi-turn conversational workloads"): most prompts short, re-prefills
over a cached history, a few long prompts (Introduction, dataset length figure).

Every tensor has its own PCG64 stream keyed by (seed, layer, tensor id) so that
tensors can be drawn in parallel and any single one can be re-drawn alone.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 11589 * 10  # per-config seed = SEED_BASE + config index (1..5)
PAGE = 16


# --------------------------------------------------------------------------- bf16 storage
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even.  Inputs are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------- model shapes
@dataclass(frozen=True)
class ModelCfg:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    n_layers: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    page_size: int = PAGE

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def params_per_layer(self) -> int:
        d, i = self.hidden, self.intermediate
        return d * self.qkv_dim + self.q_dim * d + 3 * d * i


def tiny_cfg(n_layers: int = 1) -> ModelCfg:
    return ModelCfg(256, 4, 2, 64, 512, n_layers)


def qwen32b_cfg(n_layers: int = 4) -> ModelCfg:
    """Layer shape of the largest model the paper serves (Numerical Results: 7/14/32B)."""
    return ModelCfg(5120, 40, 8, 128, 27648, n_layers)


def qwen14b_cfg(n_layers: int = 4) -> ModelCfg:
    """Layer shape of the 14B model of the same family (Numerical Results)."""
    return ModelCfg(5120, 40, 8, 128, 13824, n_layers)


def qwen7b_cfg(n_layers: int = 4) -> ModelCfg:
    """Layer shape of the 7B model of the same family (Numerical Results): 28 query heads over 4 kv heads."""
    return ModelCfg(3584, 28, 4, 128, 18944, n_layers)


# --------------------------------------------------------------------------- random tensors
_TENSOR_IDS = {"ln1": 0, "w_qkv": 1, "w_o": 2, "ln2": 3, "w_gate": 4, "w_up": 5, "w_down": 6,
               "x": 7, "lens": 8, "prefix_k": 9, "prefix_v": 10, "pages": 11, "arrivals": 12, "b_qkv": 13}


def _rng(seed: int, layer: int, name: str, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, layer, _TENSOR_IDS[name], extra])))


def _normal_bf16(seed, layer, name, shape, std, mean=0.0, extra=0) -> np.ndarray:
    g = _rng(seed, layer, name, extra)
    a = g.standard_normal(int(np.prod(shape)), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return f32_to_bf16_bits(a).reshape(shape)


def layer_weight_shapes(cfg: ModelCfg) -> dict:
    d, i = cfg.hidden, cfg.intermediate
    return {"ln1": (d,), "w_qkv": (cfg.qkv_dim, d), "w_o": (d, cfg.q_dim), "ln2": (d,),
            "w_gate": (i, d), "w_up": (i, d), "w_down": (d, i)}


def make_layer_weights(cfg: ModelCfg, seed: int, layer: int, threads: int = 8) -> dict:
    """bf16 bit patterns (uint16).  Projections N(0, 0.02^2) in [out, in] row-major order
    (w_qkv rows: all q heads, then all k heads, then all v heads); norm gains 1 + N(0, 0.02^2)."""
    shapes = layer_weight_shapes(cfg)

    def one(name):
        if name in ("ln1", "ln2"):
            return name, _normal_bf16(seed, layer, name, shapes[name], 0.02, mean=1.0)
        return name, _normal_bf16(seed, layer, name, shapes[name], 0.02)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        return dict(ex.map(one, shapes.keys()))


def make_qkv_bias(cfg: ModelCfg, seed: int, layer: int) -> np.ndarray:
    """bf16 bit pattern of a q/k/v projection bias, [qkv_dim], N(0, 0.5^2) (the model family the paper serves has one;
    the benchmark configurations leave it off)."""
    return _normal_bf16(seed, layer, "b_qkv", (cfg.qkv_dim,), 0.5)


def make_activations(cfg: ModelCfg, seed: int, n_tokens: int) -> np.ndarray:
    """fp32 N(0,1) hidden states for the packed new tokens, [n_tokens, hidden]."""
    return _rng(seed, 0, "x").standard_normal((n_tokens, cfg.hidden), dtype=np.float32)


def make_prefix_kv(cfg: ModelCfg, seed: int, layer: int, req: int, h: int):
    """Cached K and V of one request in one layer, bf16 bits, [h, n_kv, head_dim] each.
    K is regarded as already rotated."""
    shp = (h, cfg.n_kv_heads, cfg.head_dim)
    k = _normal_bf16(seed, layer, "prefix_k", shp, 1.0, extra=req)
    v = _normal_bf16(seed, layer, "prefix_v", shp, 1.0, extra=req)
    return k, v


# --------------------------------------------------------------------------- batches
@dataclass
class Batch:
    """A ragged batch: request i brings new_len[i] new tokens on top of prefix_len[i] cached ones."""
    new_len: np.ndarray                      # int32 [n]
    prefix_len: np.ndarray                   # int32 [n]
    page_table: np.ndarray                   # int32 [n, max_pages], -1 where unused
    n_pages: int                             # pool size the table indexes into
    arrival_us: np.ndarray | None = None     # int64 [n] virtual arrival times (config 5)
    extra: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(self.new_len.shape[0])

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.new_len)]).astype(np.int32)

    @property
    def n_tokens(self) -> int:
        return int(self.new_len.sum())


def make_page_table(seed: int, new_len, prefix_len, spare_pages: int = 3):
    """Pages for prefix + new tokens of every request, drawn as a random permutation of the pool
    so that no request's pages are contiguous.  `spare_pages` pool pages stay unreferenced."""
    tot = np.asarray(new_len, np.int64) + np.asarray(prefix_len, np.int64)
    need = (tot + PAGE - 1) // PAGE
    n_pages = int(need.sum()) + spare_pages
    perm = _rng(seed, 0, "pages").permutation(n_pages).astype(np.int32)
    max_pages = int(need.max()) if len(need) else 1
    table = np.full((len(need), max(max_pages, 1)), -1, np.int32)
    o = 0
    for i, c in enumerate(need):
        table[i, :c] = perm[o:o + c]
        o += int(c)
    return table, n_pages


def make_batch(config: int, n_req: int | None = None) -> Batch:
    """Length mixes of the five benchmark configurations (1-based index)."""
    seed = SEED_BASE + config
    g = _rng(seed, 0, "lens")
    if config == 1:
        n = n_req or 8
        new = g.integers(1, 65, n)
        pre = np.zeros(n, np.int64)
    elif config == 2:
        n = n_req or 256
        new = g.integers(8, 65, n)
        pre = np.zeros(n, np.int64)
    elif config == 3:
        n = n_req or 128
        pre = g.integers(512, 4097, n)
        new = g.integers(16, 65, n)
    elif config == 4:
        n = n_req or 8
        new = g.integers(1024, 8193, n)
        pre = np.zeros(n, np.int64)
    elif config == 5:
        n_long, n_short = 4, (n_req or 512)
        long_new = g.integers(2048, 8193, n_long)
        short_new = g.integers(1, 65, n_short)
        fresh = g.random(n_short) < 0.25
        short_pre = np.where(fresh, 0, g.integers(1, 4097, n_short))
        new = np.concatenate([long_new, short_new])
        pre = np.concatenate([np.zeros(n_long, np.int64), short_pre])
    else:
        raise ValueError(f"config {config}")
    new = new.astype(np.int32)
    pre = pre.astype(np.int32)
    table, n_pages = make_page_table(seed, new, pre)
    return Batch(new, pre, table, n_pages)


def poisson_arrivals_us(seed: int, n: int, rate_per_s: float) -> np.ndarray:
    """Virtual arrival timestamps in integer microseconds: exponential gaps at `rate_per_s`."""
    gaps = _rng(seed, 0, "arrivals").exponential(1.0 / rate_per_s, n)
    return np.floor(np.cumsum(gaps) * 1e6).astype(np.int64)
