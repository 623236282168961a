"""Pins for the fp64 layer oracle against facts fixed outside it: closed forms, invariants,
special cases that reduce to a library routine, and an index-by-index scalar evaluation of
a tiny layer."""
import math
import types

import numpy as np
import pytest
import torch

from oracle import laps_oracle as O


def cfg_of(d, n_q, n_kv, hd, inter, theta=1.0e6, eps=1.0e-6):
    return types.SimpleNamespace(hidden=d, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=hd,
                                 intermediate=inter, rope_theta=theta, rms_eps=eps)


def rand_weights(cfg, rng, scale=0.2):
    d, i = cfg.hidden, cfg.intermediate
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    return {"ln1": 1 + 0.1 * rng.standard_normal(d), "w_qkv": scale * rng.standard_normal((qd + 2 * kd, d)),
            "w_o": scale * rng.standard_normal((d, qd)), "ln2": 1 + 0.1 * rng.standard_normal(d),
            "w_gate": scale * rng.standard_normal((i, d)), "w_up": scale * rng.standard_normal((i, d)),
            "w_down": scale * rng.standard_normal((d, i))}


# ------------------------------------------------------------------------------- RMSNorm
def test_rmsnorm_hand_values_and_invariants():
    got = O.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 1.0]), 0.0)
    assert np.allclose(got, [[3 / math.sqrt(12.5), 4 / math.sqrt(12.5)]], atol=1e-15)
    got = O.rmsnorm(np.array([[3.0, 4.0]]), np.array([2.0, 0.5]), 0.0)
    assert np.allclose(got, [[6 / math.sqrt(12.5), 2 / math.sqrt(12.5)]], atol=1e-15)
    got = O.rmsnorm(np.array([[1.0, 1.0]]), np.array([1.0, 1.0]), 3.0)        # 1 / sqrt(1 + 3)
    assert np.allclose(got, [[0.5, 0.5]], atol=1e-15)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    y = O.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=1)), 1.0, atol=1e-13)
    assert np.allclose(O.rmsnorm(7.5 * x, np.ones(64), 0.0), y, atol=1e-13)


# ------------------------------------------------------------------------------- RoPE
def test_rope_hand_rotation_pairs_and_frequencies():
    # hd = 4, theta = 10000: pair (0,2) turns by pos*1, pair (1,3) by pos*10000^(-2/4) = pos*0.01
    u = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    got = O.rope(u, np.array([3]), 10000.0)[0, 0]
    a0, a1 = 3.0, 3.0 * 0.01
    want = [1 * math.cos(a0) - 3 * math.sin(a0), 2 * math.cos(a1) - 4 * math.sin(a1),
            3 * math.cos(a0) + 1 * math.sin(a0), 4 * math.cos(a1) + 2 * math.sin(a1)]
    assert np.allclose(got, want, atol=1e-14)


def test_rope_identity_norm_and_relative_position():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((6, 3, 16))
    k = rng.standard_normal((6, 3, 16))
    assert np.array_equal(O.rope(q, np.zeros(6), 1e6), q)                    # position 0 is identity
    pos = np.array([0, 1, 5, 17, 100, 8000])
    rq = O.rope(q, pos, 1e6)
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), atol=1e-12)
    s0 = np.einsum("thd,shd->hts", O.rope(q, pos, 1e6), O.rope(k, pos, 1e6))
    s1 = np.einsum("thd,shd->hts", O.rope(q, pos + 1234, 1e6), O.rope(k, pos + 1234, 1e6))
    assert np.allclose(s0, s1, atol=1e-9)                                    # scores see only p - p'


# ------------------------------------------------------------------------------- attention
def test_length_one_sequence_returns_v():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 4, 8))
    k = rng.standard_normal((1, 2, 8))
    v = rng.standard_normal((1, 2, 8))
    out = O.attention_one(q, k, v, 0, 1 / math.sqrt(8))
    for h in range(4):
        assert np.array_equal(out[0, h], v[0, h // 2])


def test_softmax_rows_sum_to_one_and_mask():
    rng = np.random.default_rng(3)
    L, H = 5, 7
    q = rng.standard_normal((L, 4, 8))
    k = rng.standard_normal((H + L, 2, 8))
    v = rng.standard_normal((H + L, 2, 8))
    _, probs = O.attention_one(q, k, v, H, 1 / math.sqrt(8), return_probs=True)
    for p in probs:
        assert p.shape == (L, H + L)
        assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
        for t in range(L):
            assert np.all(p[t, H + t + 1:] == 0.0)
            assert np.all(p[t, :H + t + 1] > 0.0)


def test_equal_keys_give_running_mean_of_v():
    rng = np.random.default_rng(4)
    L, H = 6, 3
    q = rng.standard_normal((L, 2, 4))
    k = np.tile(rng.standard_normal((1, 1, 4)), (H + L, 1, 1))
    v = rng.standard_normal((H + L, 1, 4))
    out = O.attention_one(q, k, v, H, 0.5)
    for t in range(L):
        want = v[:H + t + 1, 0].mean(axis=0)
        assert np.allclose(out[t, 0], want, atol=1e-14) and np.allclose(out[t, 1], want, atol=1e-14)


def _sdpa(q, k, v, H):
    """torch float64 library attention with an explicit visibility mask; heads already expanded."""
    L, S = q.shape[0], k.shape[0]
    mask = torch.arange(S)[None, :] <= (H + torch.arange(L))[:, None]
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a.transpose(1, 0, 2))) for a in (q, k, v))
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).numpy().transpose(1, 0, 2)


def test_mha_matches_library_attention_and_gqa_is_repeated_mha():
    rng = np.random.default_rng(5)
    L, H, hd = 9, 11, 16
    q = rng.standard_normal((L, 6, hd))
    k = rng.standard_normal((H + L, 6, hd))
    v = rng.standard_normal((H + L, 6, hd))
    got = O.attention_one(q, k, v, H, 1 / math.sqrt(hd))
    assert np.allclose(got, _sdpa(q, k, v, H), atol=1e-12)
    # grouped: 6 query heads over 2 kv heads == MHA with each kv head repeated 3 times, contiguously
    kg, vg = k[:, :2], v[:, :2]
    got = O.attention_one(q, kg, vg, H, 1 / math.sqrt(hd))
    want = _sdpa(q, np.repeat(kg, 3, axis=1), np.repeat(vg, 3, axis=1), H)
    assert np.allclose(got, want, atol=1e-12)


# ------------------------------------------------------------------------------- whole layer
def scalar_layer(cfg, w, x, H, pk, pv):
    """Index-by-index evaluation of one layer for one sequence, python floats only."""
    d, nq, nkv, hd, I = cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.intermediate
    L, half, grp = len(x), cfg.head_dim // 2, cfg.n_q_heads // cfg.n_kv_heads

    def norm(row, g):
        ms = sum(v * v for v in row) / d
        return [row[c] * g[c] / math.sqrt(ms + cfg.rms_eps) for c in range(d)]

    def rot(vec, p):
        out = list(vec)
        for j in range(half):
            ang = p * cfg.rope_theta ** (-2.0 * j / hd)
            out[j] = vec[j] * math.cos(ang) - vec[j + half] * math.sin(ang)
            out[j + half] = vec[j + half] * math.cos(ang) + vec[j] * math.sin(ang)
        return out

    K = [[list(pk[s][g]) for g in range(nkv)] for s in range(H)]
    V = [[list(pv[s][g]) for g in range(nkv)] for s in range(H)]
    Q = []
    for t in range(L):
        r = norm(x[t], w["ln1"])
        proj = [sum(r[c] * w["w_qkv"][o][c] for c in range(d)) for o in range((nq + 2 * nkv) * hd)]
        Q.append([rot(proj[h * hd:(h + 1) * hd], H + t) for h in range(nq)])
        K.append([rot(proj[nq * hd + g * hd: nq * hd + (g + 1) * hd], H + t) for g in range(nkv)])
        V.append([proj[(nq + nkv) * hd + g * hd:(nq + nkv) * hd + (g + 1) * hd] for g in range(nkv)])
    y = []
    for t in range(L):
        att = []
        for h in range(nq):
            g = h // grp
            sc = [sum(Q[t][h][e] * K[s][g][e] for e in range(hd)) / math.sqrt(hd) for s in range(H + t + 1)]
            m = max(sc)
            ex = [math.exp(v - m) for v in sc]
            z = sum(ex)
            att += [sum(ex[s] / z * V[s][g][e] for s in range(H + t + 1)) for e in range(hd)]
        x1 = [x[t][c] + sum(att[o] * w["w_o"][c][o] for o in range(nq * hd)) for c in range(d)]
        r2 = norm(x1, w["ln2"])
        gate = [sum(r2[c] * w["w_gate"][i][c] for c in range(d)) for i in range(I)]
        up = [sum(r2[c] * w["w_up"][i][c] for c in range(d)) for i in range(I)]
        act = [gate[i] / (1 + math.exp(-gate[i])) * up[i] for i in range(I)]
        y.append([x1[c] + sum(act[i] * w["w_down"][c][i] for i in range(I)) for c in range(d)])
    return y, [K[H + t] for t in range(L)], [V[H + t] for t in range(L)]


def test_layer_matches_scalar_evaluation():
    rng = np.random.default_rng(6)
    cfg = cfg_of(8, 4, 2, 2, 5, theta=100.0)        # q_dim == hidden, as in the real shapes
    w = rand_weights(cfg, rng, 0.5)
    L, H = 3, 2
    x = rng.standard_normal((L, 8))
    pk = rng.standard_normal((H, 2, 2))
    pv = rng.standard_normal((H, 2, 2))
    y, nk, nv = O.layer_forward(cfg, w, x, [L], [pk], [pv])
    wl = {k: v.tolist() for k, v in w.items()}
    ys, ks, vs = scalar_layer(cfg, wl, x.tolist(), H, pk.tolist(), pv.tolist())
    assert np.allclose(y, np.array(ys), atol=1e-12)
    assert np.allclose(nk[0], np.array(ks), atol=1e-13)
    assert np.allclose(nv[0], np.array(vs), atol=1e-13)


def test_zero_weight_reductions_and_length_one_layer():
    rng = np.random.default_rng(7)
    cfg = cfg_of(16, 4, 2, 4, 12)
    w = rand_weights(cfg, rng)
    x = rng.standard_normal((7, 16))
    lens = [3, 1, 3]
    w0 = dict(w, w_gate=np.zeros_like(w["w_gate"]), w_o=np.zeros_like(w["w_o"]))
    y, _, _ = O.layer_forward(cfg, w0, x, lens, None, None)
    assert np.array_equal(y, x)                                   # both branches vanish
    # w_o = identity, no MLP: the length-1 sequence (row 3) gets x + v of its kv head per q head
    w1 = dict(w, w_gate=np.zeros_like(w["w_gate"]), w_o=np.eye(16))
    y, nk, nv = O.layer_forward(cfg, w1, x, lens, None, None)
    v_row = nv[1][0]                                              # [n_kv, hd]
    want = x[3] + np.repeat(v_row, 2, axis=0).reshape(-1)
    assert np.allclose(y[3], want, atol=1e-14)
    # and that v is the plain projection of the normed row
    r = O.rmsnorm(x[3:4], w["ln1"], cfg.rms_eps)
    assert np.allclose(v_row.reshape(-1), (r @ w["w_qkv"][24:].T)[0], atol=1e-14)


def _split_kv(k_list, v_list):
    return [[k] for k in k_list], [[v] for v in v_list]


def test_cached_prefix_equals_full_prefill_and_chunking():
    rng = np.random.default_rng(8)
    cfg = cfg_of(32, 4, 2, 8, 24)
    layers = [rand_weights(cfg, rng) for _ in range(3)]
    Ltot, H = 23, 9
    x = rng.standard_normal((Ltot, 32))
    y_full, k_full, v_full = O.stack_forward(cfg, layers, x, [Ltot])
    # turn 1 = first H tokens, turn 2 = the rest on top of turn 1's cache
    y1, k1, v1 = O.stack_forward(cfg, layers, x[:H], [H])
    pk, pv = _split_kv([k1[l][0] for l in range(3)], [v1[l][0] for l in range(3)])
    y2, k2, v2 = O.stack_forward(cfg, layers, x[H:], [Ltot - H], pk, pv)
    assert np.allclose(y_full[:H], y1, atol=1e-12) and np.allclose(y_full[H:], y2, atol=1e-12)
    for l in range(3):
        assert np.allclose(k_full[l][0][H:], k2[l][0], atol=1e-12)
        assert np.allclose(v_full[l][0][H:], v2[l][0], atol=1e-12)
    for chunk in (4, 7, 23, 100):
        yc, kc, vc = O.chunked_stack_forward(cfg, layers, x, chunk)
        assert np.allclose(yc, y_full, atol=1e-12)
        assert np.allclose(kc[2], k_full[2][0], atol=1e-12) and np.allclose(vc[0], v_full[0][0], atol=1e-12)


def test_batch_order_and_neighbours_do_not_matter():
    rng = np.random.default_rng(9)
    cfg = cfg_of(32, 4, 2, 8, 24)
    layers = [rand_weights(cfg, rng) for _ in range(2)]
    lens = [5, 1, 9, 3]
    Hs = [0, 4, 6, 0]
    xs = [rng.standard_normal((l, 32)) for l in lens]
    pk = [[None if h == 0 else rng.standard_normal((h, 2, 8)) for h in Hs] for _ in range(2)]
    pv = [[None if h == 0 else rng.standard_normal((h, 2, 8)) for h in Hs] for _ in range(2)]
    y, _, _ = O.stack_forward(cfg, layers, np.concatenate(xs), lens, pk, pv)
    cu = np.concatenate([[0], np.cumsum(lens)])
    perm = [2, 0, 3, 1]
    yp, _, _ = O.stack_forward(cfg, layers, np.concatenate([xs[i] for i in perm]), [lens[i] for i in perm],
                               [[pk[l][i] for i in perm] for l in range(2)],
                               [[pv[l][i] for i in perm] for l in range(2)])
    cup = np.concatenate([[0], np.cumsum([lens[i] for i in perm])])
    for slot, i in enumerate(perm):
        assert np.allclose(yp[cup[slot]:cup[slot + 1]], y[cu[i]:cu[i + 1]], atol=1e-12)
    # a sequence alone gives the same rows as inside the batch
    for i in range(4):
        yi, _, _ = O.stack_forward(cfg, layers, xs[i], [lens[i]],
                                   [[pk[l][i]] for l in range(2)], [[pv[l][i]] for l in range(2)])
        assert np.allclose(yi, y[cu[i]:cu[i + 1]], atol=1e-12)


def test_round_to_bf16_matches_bit_twiddled_rounding():
    from paper_2601_11589_amd.inputs import bf16_bits_to_f32, f32_to_bf16_bits
    rng = np.random.default_rng(11)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-8, 8, 20000))).astype(np.float32)
    a = np.concatenate([a, np.float32([1.0, 1.00390625, 1.01171875, 0.0, -3.0])])  # includes exact ties
    want = bf16_bits_to_f32(f32_to_bf16_bits(a)).astype(np.float64)
    assert np.array_equal(O.round_to_bf16(a.astype(np.float64)), want)


def test_storage_rounding_variant_is_close_to_exact():
    rng = np.random.default_rng(12)
    cfg = cfg_of(64, 4, 2, 16, 96)
    w = rand_weights(cfg, rng, 0.1)
    x = rng.standard_normal((10, 64))
    y0, _, _ = O.layer_forward(cfg, w, x, [4, 6], None, None)
    y1, _, _ = O.layer_forward(cfg, w, x, [4, 6], None, None, storage_rounding=True)
    rel = np.linalg.norm(y1 - y0) / np.linalg.norm(y0)
    assert 0 < rel < 5e-3


def test_qkv_bias_closed_form():
    """With a zero q/k/v matrix every token's q, k, v is the bias itself: all value rows of a kv head are equal,
    so attention returns that row whatever the probabilities, and with a zero down projection the layer output is
    x + W_o a, where a repeats the value bias of each kv head over its group of query heads.  Catches a bias that
    is dropped, added to the wrong segment, or a wrong head-to-group mapping."""
    cfg = cfg_of(32, 6, 2, 8, 48)
    rng = np.random.default_rng(5)
    w = rand_weights(cfg, rng)
    w["w_qkv"] = np.zeros_like(w["w_qkv"])
    w["w_down"] = np.zeros_like(w["w_down"])
    q_dim, kv_dim = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    w["b_qkv"] = rng.standard_normal(q_dim + 2 * kv_dim)
    new_len = [3, 7]
    x = rng.standard_normal((10, cfg.hidden))
    y, new_k, new_v = O.layer_forward(cfg, w, x, new_len, [None, None], [None, None])[:3]
    hd, G = cfg.head_dim, cfg.n_q_heads // cfg.n_kv_heads
    b_v = w["b_qkv"][q_dim + kv_dim:].reshape(cfg.n_kv_heads, hd)
    a = np.concatenate([b_v[h // G] for h in range(cfg.n_q_heads)])
    assert np.allclose(y, x + w["w_o"] @ a, rtol=0, atol=1e-12)
    for i, L in enumerate(new_len):
        assert np.array_equal(new_v[i], np.broadcast_to(b_v, (L, cfg.n_kv_heads, hd)))
        # position 0 is not rotated: the first new key of a fresh prompt is the key bias
        assert np.allclose(new_k[i][0], w["b_qkv"][q_dim:q_dim + kv_dim].reshape(cfg.n_kv_heads, hd), atol=1e-14)
