"""CPU oracle for the ragged prefill layer stack.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module; the product path never does.  It shares no code with the HIP path.

What it is.  The paper (LAPS) defines the scheduling around the prefill forward and says
of the forward itself only that it is "incremental causal attention and FFN" over L new
tokens and H historical tokens whose KV is cached (Background, latency model
T_comp = alpha*L*(L+2H) + beta*L; Introduction, definition of re-prefill), on Qwen2.5
models (Numerical Results).  The layer below is therefore the plain textbook definition
of one such decoder layer (pre-RMSNorm, grouped-query attention with rotate-half RoPE,
SwiGLU MLP), written out in float64 numpy with no tiling, no fusion and no intermediate
rounding.  Dense products use numpy.matmul as a library step.

Parity pins (tests/test_oracle_*.py): length-1 attention returns V; cached-prefix prefill
equals full prefill of the concatenation; chunked equals unchunked; order / padding
independence; softmax rows sum to one; equal-keys closed form; RoPE relative-position
invariance; GQA == MHA with repeated heads; zero-weight reductions; explicit triple-loop
matmul; torch scaled_dot_product_attention (float64, CPU) for the no-prefix case.
The conventions the paper does not state (eps, rotate-half pairing, contiguous GQA groups,
1/sqrt(head_dim) scale) are pinned only by declaration: parity unpinned by the paper.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- pieces
def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise x * w / sqrt(mean(x^2) + eps)."""
    x = np.asarray(x, np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * np.asarray(w, np.float64) / np.sqrt(ms + eps)


def rope(u: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate-half rotary embedding.  u: [T, heads, hd]; pos: [T] absolute positions.
    Pair (j, j + hd/2) is rotated by angle pos * theta^(-2j/hd)."""
    u = np.asarray(u, np.float64)
    hd = u.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / hd)
    ang = np.asarray(pos, np.float64)[:, None] * inv_freq[None, :]      # [T, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (ties to even) of each float64 entry, returned as float64.
    Used only by the storage_rounding variant of the layer, which applies the declared
    storage points of the device path (q, k, v, normed rows, attention output, MLP
    activation kept in bf16) while all arithmetic stays float64."""
    a = np.asarray(a, np.float64)
    m, e = np.frexp(a)                      # a = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0          # 8 significant bits; rint is ties-to-even
    return np.ldexp(q, e)


def attention_one(q, k_all, v_all, h_prefix: int, scale: float, return_probs: bool = False):
    """Causal attention of one sequence.  q: [L, n_q, hd]; k_all, v_all: [H+L, n_kv, hd].
    New token t (absolute position H+t) sees keys 0..H+t.  Query head h uses kv head
    h // (n_q / n_kv)."""
    L, n_q, hd = q.shape
    n_kv = k_all.shape[1]
    group = n_q // n_kv
    S_len = k_all.shape[0]
    key_idx = np.arange(S_len)[None, :]
    limit = (h_prefix + np.arange(L))[:, None]
    visible = key_idx <= limit                                          # [L, H+L]
    out = np.empty((L, n_q, hd), np.float64)
    probs = [] if return_probs else None
    for h in range(n_q):
        g = h // group
        s = (q[:, h, :] @ k_all[:, g, :].T) * scale
        s = np.where(visible, s, -np.inf)
        s = s - np.max(s, axis=1, keepdims=True)
        p = np.exp(s)
        p = p / np.sum(p, axis=1, keepdims=True)
        out[:, h, :] = p @ v_all[:, g, :]
        if return_probs:
            probs.append(p)
    return (out, probs) if return_probs else out


# ----------------------------------------------------------------------------- one layer
def layer_forward(cfg, w: dict, x: np.ndarray, new_len, prefix_k, prefix_v,
                  storage_rounding: bool = False, return_probs: bool = False):
    """One decoder layer over a packed ragged batch.

    cfg: object with hidden, n_q_heads, n_kv_heads, head_dim, intermediate, rope_theta, rms_eps.
    w: float64 arrays ln1 [d], w_qkv [(n_q+2 n_kv) hd, d], w_o [d, n_q hd], ln2 [d],
       w_gate [I, d], w_up [I, d], w_down [d, I]; optional b_qkv.
    x: [T, d] packed new tokens, sequence i occupying rows cu[i]:cu[i+1].
    new_len: [n] new-token counts.  prefix_k / prefix_v: per sequence, [H_i, n_kv, hd]
    (already-rotated K) or None for H_i = 0.
    Returns y [T, d], list of new k [L_i, n_kv, hd], list of new v, (optional) probabilities.
    """
    x = np.asarray(x, np.float64)
    n_q, n_kv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    rnd = round_to_bf16 if storage_rounding else (lambda a: a)
    cu = np.concatenate([[0], np.cumsum(np.asarray(new_len, np.int64))])
    assert cu[-1] == x.shape[0]

    r = rnd(rmsnorm(x, w["ln1"], cfg.rms_eps))
    qkv = r @ w["w_qkv"].T
    if w.get("b_qkv") is not None:
        qkv = qkv + w["b_qkv"]
    qd, kd = n_q * hd, n_kv * hd
    attn = np.empty((x.shape[0], qd), np.float64)
    new_k, new_v, all_probs = [], [], []
    scale = 1.0 / np.sqrt(hd)
    for i in range(len(new_len)):
        a, b = int(cu[i]), int(cu[i + 1])
        L = b - a
        pk = None if prefix_k is None else prefix_k[i]
        pv = None if prefix_v is None else prefix_v[i]
        H = 0 if pk is None else int(pk.shape[0])
        pos = H + np.arange(L)
        q = rnd(rope(qkv[a:b, :qd].reshape(L, n_q, hd), pos, cfg.rope_theta))
        k = rnd(rope(qkv[a:b, qd:qd + kd].reshape(L, n_kv, hd), pos, cfg.rope_theta))
        v = rnd(qkv[a:b, qd + kd:].reshape(L, n_kv, hd))
        if H > 0:
            k_all = np.concatenate([np.asarray(pk, np.float64), k], axis=0)
            v_all = np.concatenate([np.asarray(pv, np.float64), v], axis=0)
        else:
            k_all, v_all = k, v
        res = attention_one(q, k_all, v_all, H, scale, return_probs)
        if return_probs:
            o, p = res
            all_probs.append(p)
        else:
            o = res
        attn[a:b] = o.reshape(L, qd)
        new_k.append(k)
        new_v.append(v)
    x1 = x + rnd(attn) @ w["w_o"].T
    r2 = rnd(rmsnorm(x1, w["ln2"], cfg.rms_eps))
    act = rnd(silu(r2 @ w["w_gate"].T) * (r2 @ w["w_up"].T))
    y = x1 + act @ w["w_down"].T
    if return_probs:
        return y, new_k, new_v, all_probs
    return y, new_k, new_v


# ----------------------------------------------------------------------------- stack
def stack_forward(cfg, layers, x, new_len, prefix_k=None, prefix_v=None, storage_rounding=False):
    """Repeat layer_forward over `layers` (any indexable of weight dicts, length n_layers).
    prefix_k / prefix_v: per layer, per sequence arrays (or None).  No embedding, final norm
    or LM head.  Returns y and per-layer lists of appended k, v."""
    ks, vs = [], []
    y = np.asarray(x, np.float64)
    for l in range(len(layers)):
        pk = None if prefix_k is None else prefix_k[l]
        pv = None if prefix_v is None else prefix_v[l]
        y, nk, nv = layer_forward(cfg, layers[l], y, new_len, pk, pv, storage_rounding)
        ks.append(nk)
        vs.append(nv)
    return y, ks, vs


def chunked_stack_forward(cfg, layers, x, chunk: int, prefix_k=None, prefix_v=None,
                          storage_rounding=False):
    """One long request advanced by fixed-size chunks (SLA-constrained mode, last sentence:
    long-prefill dispatch advances a single request by chunks C_l).  Chunk c is a re-prefill
    whose history is the cached prefix plus chunks < c.  x: [L, d]; prefix_k/v: per layer
    [H, n_kv, hd] or None.  Returns y [L, d] and per-layer appended k, v [L, n_kv, hd]."""
    L = x.shape[0]
    n_layers = len(layers)
    hist_k = [None if prefix_k is None else prefix_k[l] for l in range(n_layers)]
    hist_v = [None if prefix_v is None else prefix_v[l] for l in range(n_layers)]
    h0 = [0 if hk is None else hk.shape[0] for hk in hist_k]
    ys = []
    for s in range(0, L, chunk):
        e = min(L, s + chunk)
        y, nk, nv = stack_forward(cfg, layers, x[s:e], [e - s],
                                  [[hk] for hk in hist_k], [[hv] for hv in hist_v], storage_rounding)
        ys.append(y)
        for l in range(n_layers):
            hist_k[l] = nk[l][0] if hist_k[l] is None else np.concatenate([hist_k[l], nk[l][0]], 0)
            hist_v[l] = nv[l][0] if hist_v[l] is None else np.concatenate([hist_v[l], nv[l][0]], 0)
    return (np.concatenate(ys, 0),
            [hist_k[l][h0[l]:] for l in range(n_layers)],
            [hist_v[l][h0[l]:] for l in range(n_layers)])
