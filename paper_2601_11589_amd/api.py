"""Thin ctypes binding over liblaps.so: same names as include/laps.h, argument marshalling only.

PyTorch is used for device memory (tensors -> raw pointers) and streams; every step of the
path runs inside the library's HIP kernels.  There is no CPU or eager fallback: if the shared
library is missing or fails to load, the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblaps.so")

K_NAMES = ["prep", "rmsnorm", "gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "epi_qkv", "epi_resid",
           "epi_swiglu", "attn"]


class LapsError(RuntimeError):
    pass


class _ModelCfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("intermediate", C.c_int32), ("n_layers", C.c_int32), ("page_size", C.c_int32),
                ("has_qkv_bias", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ln1_w", "w_qkv", "b_qkv", "w_o", "ln2_w", "w_gate_up", "w_down")]


class _PlanParams(C.Structure):
    _fields_ = [("short_max_len", C.c_int32), ("n_len_buckets", C.c_int32), ("len_buckets", C.POINTER(C.c_int32)),
                ("n_depths", C.c_int32), ("depths", C.POINTER(C.c_int32)), ("token_budget", C.c_int32),
                ("long_chunk", C.c_int32)]


_lib = None


def lib():
    """Loads liblaps.so (built in-tree by paper_2601_11589_amd.build).  Fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LapsError(f"{LIB_PATH} not found: run `python -m paper_2601_11589_amd.build` (no fallback path exists)")
        L = C.CDLL(LIB_PATH)
        L.laps_last_error.restype = C.c_char_p
        L.laps_version.restype = C.c_char_p
        L.laps_workspace_bytes.restype = C.c_size_t
        L.laps_workspace_bytes_for.restype = C.c_size_t
        L.laps_gemm_workspace_bytes.restype = C.c_size_t
        L.laps_static_scratch_bytes.restype = C.c_size_t
        L.laps_graph_device_bytes.restype = C.c_size_t
        L.laps_graph_output.restype = C.c_void_p
        L.laps_graph_input.restype = C.c_void_p
        for name in ("req_class", "req_bucket", "req_batch", "req_row", "batch_len_bucket", "batch_depth",
                     "batch_graph_ok", "batch_req_offset", "batch_req_ids", "long_req", "long_chunk_offset",
                     "long_chunk_len"):
            getattr(L, "laps_plan_" + name).restype = C.POINTER(C.c_int32)
            getattr(L, "laps_plan_" + name).argtypes = [C.c_void_p]
        for name in ("n_requests", "n_batches", "n_long"):
            getattr(L, "laps_plan_" + name).argtypes = [C.c_void_p]
        L.laps_lm_boundary_prefill.restype = C.c_double
        L.laps_lm_boundary_prefill.argtypes = [C.c_double] * 3
        L.laps_lm_boundary_reprefill.restype = C.c_double
        L.laps_lm_boundary_reprefill.argtypes = [C.c_double] * 5
        L.laps_lm_knee.restype = C.c_double
        L.laps_lm_knee.argtypes = [C.c_double] * 6
        L.laps_awd_window_us.restype = C.c_double
        L.laps_awd_window_us.argtypes = [C.c_void_p]
        L.laps_awd_target_depth.restype = C.c_int32
        L.laps_awd_target_depth.argtypes = [C.c_void_p]
        L.laps_awd_destroy.restype = None
        L.laps_awd_destroy.argtypes = [C.c_void_p]
        L.laps_awd_begin_round.argtypes = [C.c_void_p, C.c_double]
        L.laps_ctrl_destroy.restype = None
        L.laps_ctrl_destroy.argtypes = [C.c_void_p]
        L.laps_ctrl_n_short.argtypes = [C.c_void_p]
        L.laps_plan_free.argtypes = [C.c_void_p]
        L.laps_ctx_destroy.argtypes = [C.c_void_p]
        L.laps_graph_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise LapsError(f"liblaps error {rc}: {lib().laps_last_error().decode()}")


def _p(t):
    """Raw device (or host) address of a tensor, None -> NULL."""
    if t is None:
        return C.c_void_p(0)
    assert t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _after_current(stream):
    """Orders `stream` behind torch's current stream.  What a wrapper allocates (outputs, workspace) and what the
    caller has just filled (page tables, lengths, inputs) belongs to the current stream; the library enqueues on
    `stream`, which does not wait for another stream by itself - a page table read before it is written steers the
    K/V append to wherever the stale entries point.  One event record + wait, nothing when the two are the same."""
    if stream is None:
        return
    cur = torch.cuda.current_stream()
    if cur.cuda_stream != stream.cuda_stream:
        stream.wait_stream(cur)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


# --------------------------------------------------------------------------- plan
def laps_plan_buckets(short_max_len, len_buckets, depths, token_budget, long_chunk, new_len, prefix_len) -> dict:
    """Returns the plan as plain Python lists in the same structure the brute-force oracle uses."""
    L = lib()
    lb, lbp = _i32(len_buckets)
    dp, dpp = _i32(depths)
    nl, nlp = _i32(new_len)
    pl, plp = _i32(prefix_len)
    params = _PlanParams(short_max_len, len(lb), lbp, len(dp), dpp, token_budget, long_chunk)
    h = C.c_void_p()
    _check(L.laps_plan_buckets(C.byref(params), C.c_int32(len(nl)), nlp, plp, C.byref(h)))
    try:
        n, nb, nlong = L.laps_plan_n_requests(h), L.laps_plan_n_batches(h), L.laps_plan_n_long(h)

        def arr(name, cnt):
            ptr = getattr(L, "laps_plan_" + name)(h)
            return [int(ptr[i]) for i in range(cnt)]

        off = arr("batch_req_offset", nb + 1)
        ids = arr("batch_req_ids", off[-1] if nb else 0)
        lbk, dep, ok = arr("batch_len_bucket", nb), arr("batch_depth", nb), arr("batch_graph_ok", nb)
        batches = [{"len_bucket": lbk[b], "depth": dep[b], "graph_ok": ok[b], "req_ids": ids[off[b]:off[b + 1]]}
                   for b in range(nb)]
        coff = arr("long_chunk_offset", nlong + 1)
        clen = arr("long_chunk_len", coff[-1] if nlong else 0)
        lreq = arr("long_req", nlong)
        longs = [{"req_id": lreq[i], "chunks": clen[coff[i]:coff[i + 1]]} for i in range(nlong)]
        return {"cls": arr("req_class", n), "bucket": arr("req_bucket", n), "batches": batches, "longs": longs,
                "req_batch": arr("req_batch", n), "req_row": arr("req_row", n)}
    finally:
        L.laps_plan_free(h)


# --------------------------------------------------------------------------- latency model
def laps_lm_boundary_prefill(alpha, beta, gamma_w) -> float:
    return float(lib().laps_lm_boundary_prefill(alpha, beta, gamma_w))


def laps_lm_boundary_reprefill(alpha, beta, gamma_w, gamma_r, hist_len) -> float:
    return float(lib().laps_lm_boundary_reprefill(alpha, beta, gamma_w, gamma_r, hist_len))


def laps_lm_knee(alpha, beta, gamma_w, gamma_r, floor_t, hist_len) -> float:
    return float(lib().laps_lm_knee(alpha, beta, gamma_w, gamma_r, floor_t, hist_len))


class _LmParams(C.Structure):
    _fields_ = [("short_max_len", C.c_int32), ("short_token_budget", C.c_int32), ("fuse_budget", C.c_int32),
                ("knee_fresh", C.c_double), ("knee_hist", C.c_double)]


def laps_lm_derive_params(coef, floor_t, hist_max, len_buckets, depths) -> dict:
    """coef = (alpha, beta, gamma_w, gamma_r).  Returns the scheduling parameters that follow from the fit."""
    c = (C.c_double * 4)(*[float(v) for v in coef])
    (lb, lb_p), (dp, dp_p) = _i32(len_buckets), _i32(depths)
    out = _LmParams()
    _check(lib().laps_lm_derive_params(c, C.c_double(floor_t), C.c_double(hist_max), C.c_int32(len(lb)), lb_p,
                                       C.c_int32(len(dp)), dp_p, C.byref(out)))
    return {"short_max_len": out.short_max_len, "short_token_budget": out.short_token_budget,
            "fuse_budget": out.fuse_budget, "knee_fresh": out.knee_fresh, "knee_hist": out.knee_hist}


def laps_lm_fit(new_len, hist_len, t_comp=None, t_mem=None):
    """Returns (alpha, beta, gamma_w, gamma_r); the pair whose time array is None comes back as NaN."""
    arrs = [None if a is None else np.ascontiguousarray(a, dtype=np.float64) for a in (new_len, hist_len, t_comp, t_mem)]
    n = len(arrs[0])
    assert all(a is None or len(a) == n for a in arrs)
    out = (C.c_double * 4)(*([float("nan")] * 4))
    ptrs = [None if a is None else a.ctypes.data_as(C.POINTER(C.c_double)) for a in arrs]
    _check(lib().laps_lm_fit(C.c_int32(n), *ptrs, out))
    return tuple(float(v) for v in out)


# --------------------------------------------------------------------------- adaptive wait-depth batching
class _AwdParams(C.Structure):
    _fields_ = [("n_len_buckets", C.c_int32), ("len_buckets", C.POINTER(C.c_int32)), ("n_depths", C.c_int32),
                ("depths", C.POINTER(C.c_int32)), ("mem_budget", C.c_int64), ("fuse_budget", C.c_int64),
                ("sigma_us", C.c_double),
                ("w_min_us", C.c_double), ("w_max_us", C.c_double), ("s_hat_us", C.c_double), ("t_max_us", C.c_double),
                ("delta_us", C.c_double), ("rate_eps", C.c_double), ("sla_window", C.c_int32), ("d_regrow", C.c_int32)]


AWD_REASONS = ("none", "depth", "sla", "tmax", "window")


class LapsAwd:
    """Handle of the host-side AWD state (laps_awd_*): marshalling only."""

    def __init__(self, len_buckets, depths, mem_budget, sigma_us=0.0, w_min_us=0.0, w_max_us=10_000.0, s_hat_us=1_000.0,
                 t_max_us=float("inf"), delta_us=0.0, rate_eps=1e-9, sla_window=False, d_regrow=False,
                 first_slack_us=float("inf"), fuse_budget=-1):
        L = lib()
        (lb, lb_p), (dp, dp_p) = _i32(len_buckets), _i32(depths)
        prm = _AwdParams(len(lb), lb_p, len(dp), dp_p, int(mem_budget), int(fuse_budget), sigma_us, w_min_us, w_max_us, s_hat_us, t_max_us, delta_us, rate_eps,
                         int(sla_window), int(d_regrow))
        self._h = C.c_void_p()
        self._grid = (len(lb), len(dp))
        _check(L.laps_awd_create(C.byref(prm), C.c_double(first_slack_us), C.byref(self._h)))

    @property
    def window_us(self) -> float:
        return float(lib().laps_awd_window_us(self._h))

    @property
    def target_depth(self) -> int:
        return int(lib().laps_awd_target_depth(self._h))

    def laps_awd_set_service_table(self, table):
        """table: float array [n_len_buckets, n_depths] (NaN = no entry) or None."""
        if table is None:
            _check(lib().laps_awd_set_service_table(self._h, None))
            return
        t = np.ascontiguousarray(table, dtype=np.float64)
        assert t.shape == self._grid
        _check(lib().laps_awd_set_service_table(self._h, t.ctypes.data_as(C.POINTER(C.c_double))))

    def laps_awd_begin_round(self, free_at_us: float):
        _check(lib().laps_awd_begin_round(self._h, C.c_double(free_at_us)))

    def laps_awd_poll(self, now_us, arrival_us, ddl_us, new_len, rate_hat=0.0) -> dict:
        arr = np.ascontiguousarray(arrival_us, dtype=np.float64)
        ddl = np.ascontiguousarray(ddl_us, dtype=np.float64)
        nl, nl_p = _i32(new_len)
        n = len(arr)
        assert len(ddl) == n and len(nl) == n
        take = np.zeros(max(n, 1), np.int32)
        action, n_take, lb, depth, reason = (C.c_int32() for _ in range(5))
        wake = C.c_double()
        dp = lambda a: a.ctypes.data_as(C.POINTER(C.c_double))
        _check(lib().laps_awd_poll(self._h, C.c_double(now_us), C.c_double(rate_hat), C.c_int32(n), dp(arr), dp(ddl), nl_p,
                                   C.byref(action), C.byref(n_take), take.ctypes.data_as(C.POINTER(C.c_int32)),
                                   C.byref(lb), C.byref(depth),
                                   C.byref(reason), C.byref(wake)))
        return {"dispatch": action.value == 1, "take": [int(i) for i in take[:n_take.value]], "len_bucket": lb.value,
                "depth": depth.value, "reason": AWD_REASONS[reason.value], "wake_us": wake.value}

    def close(self):
        if self._h:
            lib().laps_awd_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# --------------------------------------------------------------------------- fixed-window dispatch
class _WindowParams(C.Structure):
    _fields_ = [("n_len_buckets", C.c_int32), ("len_buckets", C.POINTER(C.c_int32)), ("window_us", C.c_double),
                ("token_budget", C.c_int64), ("merge_below", C.c_int64)]


def laps_window_poll(len_buckets, window_us, token_budget, merge_below, now_us, arrival_us, new_len, nothing_else) -> dict:
    lb, lb_p = _i32(len_buckets)
    arr = np.ascontiguousarray(arrival_us, dtype=np.float64)
    nl, nl_p = _i32(new_len)
    assert len(arr) == len(nl)
    prm = _WindowParams(len(lb), lb_p, float(window_us), int(token_budget), int(merge_below))
    action, fused = C.c_int32(), C.c_int32()
    padded, wake = C.c_int64(), C.c_double()
    _check(lib().laps_window_poll(C.byref(prm), C.c_double(now_us), C.c_int32(len(arr)),
                                  arr.ctypes.data_as(C.POINTER(C.c_double)), nl_p, C.c_int32(int(bool(nothing_else))),
                                  C.byref(action), C.byref(fused), C.byref(padded), C.byref(wake)))
    return {"dispatch": action.value == 1, "fused_len_bucket": fused.value, "padded_tokens": padded.value,
            "wake_us": wake.value}


# --------------------------------------------------------------------------- instance-pressure controller
class _CtrlParams(C.Structure):
    _fields_ = [("n_total", C.c_int32), ("n_min", C.c_int32), ("cool_us", C.c_double), ("tau", C.c_double),
                ("w_q", C.c_double), ("w_e", C.c_double), ("w_u", C.c_double), ("quantile", C.c_double),
                ("min_pressure", C.c_double)]


class LapsCtrl:
    """Handle of the host-side pool controller (laps_ctrl_*): marshalling only."""

    def __init__(self, n_total, n_short, n_min=1, cool_us=0.0, tau=0.1, w_q=1.0, w_e=1.0, w_u=1.0, quantile=0.9,
                 min_pressure=float("-inf")):
        L = lib()
        prm = _CtrlParams(n_total, n_min, cool_us, tau, w_q, w_e, w_u, quantile, min_pressure)
        self._h = C.c_void_p()
        self.n_total = n_total
        _check(L.laps_ctrl_create(C.byref(prm), C.c_int32(n_short), C.byref(self._h)))

    @property
    def n_short(self) -> int:
        return int(lib().laps_ctrl_n_short(self._h))

    def laps_ctrl_step(self, now_us, short_signals, long_signals):
        """signals: sequences of (q, e, u) per instance.  Returns (action, P_s, P_l)."""
        def cols(sig):
            a = np.ascontiguousarray(np.asarray(sig, np.float64).reshape(-1, 3).T)
            return a, [a[i].ctypes.data_as(C.POINTER(C.c_double)) for i in range(3)]
        a_s, p_s = cols(short_signals)
        a_l, p_l = cols(long_signals)
        action, ps, pl = C.c_int32(), C.c_double(), C.c_double()
        _check(lib().laps_ctrl_step(self._h, C.c_double(now_us), C.c_int32(a_s.shape[1]), *p_s, C.c_int32(a_l.shape[1]),
                                    *p_l, C.byref(action), C.byref(ps), C.byref(pl)))
        return action.value, ps.value, pl.value

    def close(self):
        if self._h:
            lib().laps_ctrl_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# --------------------------------------------------------------------------- context
def bf16_tensor(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns (host) -> torch.bfloat16 tensor on the device."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class LapsCtx:
    def __init__(self, cfg, max_positions: int, has_qkv_bias: bool = False):
        self.cfg = cfg
        self._c = _ModelCfg(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.intermediate, cfg.n_layers,
                            cfg.page_size, int(has_qkv_bias), cfg.rope_theta, cfg.rms_eps)
        self._h = C.c_void_p()
        _check(lib().laps_ctx_create(C.byref(self._c), C.c_int32(max_positions), C.byref(self._h)))
        self._ws = None

    def close(self):
        if self._h:
            lib().laps_ctx_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- scratch
    def laps_workspace_bytes(self, max_tokens: int, max_seqs: int) -> int:
        return int(lib().laps_workspace_bytes(self._h, C.c_int32(max_tokens), C.c_int32(max_seqs)))

    def _guard_pools(self, pool: torch.Tensor):
        """Tells the library how many pages the pools of the next call hold, so that a page id outside them (a stale
        or corrupted table) is ignored instead of addressing memory outside the pools."""
        _check(lib().laps_ctx_set_pool_pages(self._h, C.c_int32(int(pool.shape[0]))))

    def workspace(self, max_tokens: int, max_seqs: int) -> torch.Tensor:
        need = self.laps_workspace_bytes(max_tokens, max_seqs)
        if need == 0:
            raise LapsError("laps_workspace_bytes returned 0 (bad arguments)")
        if self._ws is None or self._ws.numel() < need:
            # kernels launched through the library on other streams may still use the old buffer, and torch's allocator
            # knows nothing of them: let them finish before the block goes back to it
            torch.cuda.synchronize()
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    # ---- weights
    def laps_pack_gate_up(self, w_gate: torch.Tensor, w_up: torch.Tensor, stream=None) -> torch.Tensor:
        dst = torch.empty((2 * self.cfg.intermediate, self.cfg.hidden), dtype=torch.bfloat16, device=w_gate.device)
        _after_current(stream)
        _check(lib().laps_pack_gate_up(self._h, _p(w_gate), _p(w_up), _p(dst), _stream(stream)))
        return dst

    def upload_layer(self, w: dict) -> dict:
        """Host bf16 bit arrays (inputs.make_layer_weights) -> device tensors + the packed gate/up matrix."""
        dev = {k: bf16_tensor(v) for k, v in w.items()}
        dev["w_gate_up"] = self.laps_pack_gate_up(dev.pop("w_gate"), dev.pop("w_up"))
        torch.cuda.synchronize()
        return dev

    def _weights_array(self, layers):
        arr = (_LayerWeights * len(layers))()
        for i, w in enumerate(layers):
            b = w.get("b_qkv")
            arr[i] = _LayerWeights(w["ln1"].data_ptr(), w["w_qkv"].data_ptr(), b.data_ptr() if b is not None else 0,
                                   w["w_o"].data_ptr(), w["ln2"].data_ptr(), w["w_gate_up"].data_ptr(),
                                   w["w_down"].data_ptr())
        return arr

    # ---- KV pools
    def new_pools(self, n_pages: int, n_layers: int | None = None, zero: bool = False):
        n_layers = n_layers or self.cfg.n_layers
        mk = torch.zeros if zero else torch.empty
        shape_k = (n_pages, self.cfg.n_kv_heads, 16, self.cfg.head_dim)
        shape_v = (n_pages, self.cfg.n_kv_heads, self.cfg.head_dim, 16)
        return ([mk(shape_k, dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)],
                [mk(shape_v, dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)])

    def laps_kv_scatter(self, cu, start_pos, page_table, k_src, v_src, k_pool, v_pool, stream=None):
        n_seq, n_tok = cu.numel() - 1, k_src.shape[0]
        self._guard_pools(k_pool)
        _after_current(stream)
        _check(lib().laps_kv_scatter(self._h, C.c_int32(n_seq), C.c_int32(n_tok), _p(cu), _p(start_pos), _p(page_table),
                                     C.c_int32(page_table.shape[1]), _p(k_src), _p(v_src), _p(k_pool), _p(v_pool),
                                     _stream(stream)))

    def laps_kv_gather(self, cu, start_pos, page_table, k_pool, v_pool, n_tokens, stream=None):
        n_seq = cu.numel() - 1
        shp = (n_tokens, self.cfg.n_kv_heads, self.cfg.head_dim)
        k = torch.empty(shp, dtype=torch.bfloat16, device="cuda")
        v = torch.empty(shp, dtype=torch.bfloat16, device="cuda")
        self._guard_pools(k_pool)
        _after_current(stream)
        _check(lib().laps_kv_gather(self._h, C.c_int32(n_seq), C.c_int32(n_tokens), _p(cu), _p(start_pos), _p(page_table),
                                    C.c_int32(page_table.shape[1]), _p(k_pool), _p(v_pool), _p(k), _p(v), _stream(stream)))
        return k, v

    # ---- forward
    def laps_prefill_layer(self, w: dict, cu, seq_len, prefix_len, page_table, k_pool, v_pool, x_in, x_out=None,
                           stream=None):
        n_seq, n_tok = cu.numel() - 1, x_in.shape[0]
        x_out = torch.empty_like(x_in) if x_out is None else x_out
        ws = self.workspace(n_tok, n_seq)
        arr = self._weights_array([w])
        self._guard_pools(k_pool)
        _after_current(stream)
        _check(lib().laps_prefill_layer(self._h, arr, C.c_int32(n_seq), C.c_int32(n_tok), _p(cu), _p(seq_len), _p(prefix_len),
                                        _p(page_table), C.c_int32(page_table.shape[1]), _p(k_pool), _p(v_pool), _p(x_in),
                                        _p(x_out), _p(ws), C.c_size_t(ws.numel()), _stream(stream)))
        return x_out

    def laps_prefill_stack(self, layers, cu, seq_len, prefix_len, page_table, k_pools, v_pools, x_in, x_out=None,
                           stream=None):
        n_seq, n_tok = cu.numel() - 1, x_in.shape[0]
        x_out = torch.empty_like(x_in) if x_out is None else x_out
        ws = self.workspace(n_tok, n_seq)
        arr = self._weights_array(layers)
        kp = (C.c_void_p * len(layers))(*[t.data_ptr() for t in k_pools])
        vp = (C.c_void_p * len(layers))(*[t.data_ptr() for t in v_pools])
        self._guard_pools(k_pools[0])
        _after_current(stream)
        _check(lib().laps_prefill_stack(self._h, arr, C.c_int32(n_seq), C.c_int32(n_tok), _p(cu), _p(seq_len), _p(prefix_len),
                                        _p(page_table), C.c_int32(page_table.shape[1]), kp, vp, _p(x_in), _p(x_out), _p(ws),
                                        C.c_size_t(ws.numel()), _stream(stream)))
        return x_out

    def laps_prefill_stack_static(self, layers, cu, seq_len, prefix_len, page_table, k_pools, v_pools, x_in, x_out,
                                  stream=None):
        """laps_prefill_stack on the library's static scratch array: the caller passes the output tensor too, so
        that neither the binding nor the library allocates device memory in this call."""
        n_seq, n_tok = cu.numel() - 1, x_in.shape[0]
        arr = self._weights_array(layers)
        kp = (C.c_void_p * len(layers))(*[t.data_ptr() for t in k_pools])
        vp = (C.c_void_p * len(layers))(*[t.data_ptr() for t in v_pools])
        self._guard_pools(k_pools[0])
        _after_current(stream)
        _check(lib().laps_prefill_stack_static(self._h, arr, C.c_int32(n_seq), C.c_int32(n_tok), _p(cu), _p(seq_len),
                                               _p(prefix_len), _p(page_table), C.c_int32(page_table.shape[1]), kp, vp,
                                               _p(x_in), _p(x_out), _stream(stream)))
        return x_out

    # ---- single kernels
    def laps_gemm_bf16(self, a, w, split_k: int = 0, stream=None):
        m, k = a.shape
        n = w.shape[0]
        out = torch.empty((m, n), dtype=torch.float32, device=a.device)
        need = int(lib().laps_gemm_workspace_bytes(C.c_int32(m), C.c_int32(n), C.c_int32(k), C.c_int32(split_k)))
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=a.device)
        _after_current(stream)
        _check(lib().laps_gemm_bf16(self._h, _p(a), _p(w), _p(out), C.c_int32(m), C.c_int32(n), C.c_int32(k),
                                    C.c_int32(split_k), _p(ws), C.c_size_t(ws.numel()), _stream(stream)))
        return out

    def laps_gemm_plan_info(self, m, n, k, split_k=0, epilogue=0) -> dict:
        out = (C.c_int32 * 7)()
        _check(lib().laps_gemm_plan_info(C.c_int32(m), C.c_int32(n), C.c_int32(k), C.c_int32(split_k), C.c_int32(epilogue), out))
        return dict(zip(("bm", "bn", "split", "k_per_split", "epi", "ws", "workgroups"), (int(v) for v in out)))

    def laps_gemm_epilogue_bf16(self, a, w, epilogue: int, resid=None, stream=None):
        """epilogue 1: returns fp32 resid + a w^T; epilogue 2: returns bf16 silu(gate) * up (w packed by laps_pack_gate_up)."""
        m, k = a.shape
        n = w.shape[0]
        info = self.laps_gemm_plan_info(m, n, k, 0, epilogue)
        need = info["split"] * m * n * 4 if info["split"] > 1 else 0
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=a.device)
        out_f32 = torch.empty((m, n), dtype=torch.float32, device=a.device) if epilogue == 1 else None
        out_bf16 = torch.empty((m, n // 2), dtype=torch.bfloat16, device=a.device) if epilogue == 2 else None
        _after_current(stream)
        _check(lib().laps_gemm_epilogue_bf16(self._h, _p(a), _p(w), C.c_int32(m), C.c_int32(n), C.c_int32(k),
                                             C.c_int32(epilogue), _p(resid), _p(out_f32), _p(out_bf16), _p(ws),
                                             C.c_size_t(ws.numel()), _stream(stream)))
        return out_f32 if epilogue == 1 else out_bf16

    def laps_attention(self, cu, seq_len, prefix_len, page_table, k_pool, v_pool, q, stream=None):
        n_seq, n_tok = cu.numel() - 1, q.shape[0]
        out = torch.zeros_like(q)
        ws = self.workspace(n_tok, n_seq)
        self._guard_pools(k_pool)
        _after_current(stream)
        _check(lib().laps_attention(self._h, C.c_int32(n_seq), C.c_int32(n_tok), _p(cu), _p(seq_len), _p(prefix_len),
                                    _p(page_table), C.c_int32(page_table.shape[1]), _p(k_pool), _p(v_pool), _p(q), _p(out),
                                    _p(ws), C.c_size_t(ws.numel()), _stream(stream)))
        return out

    # ---- timing
    def laps_prof_enable(self, on: bool):
        _check(lib().laps_prof_enable(self._h, C.c_int32(int(on))))

    def laps_prof_read(self) -> dict:
        ms = (C.c_double * len(K_NAMES))()
        cnt = (C.c_int64 * len(K_NAMES))()
        _check(lib().laps_prof_read(self._h, ms, cnt))
        return {K_NAMES[i]: (float(ms[i]), int(cnt[i])) for i in range(len(K_NAMES))}

    # ---- graphs
    def laps_graph_capture(self, layers, len_bucket: int, depth: int, max_pages: int, k_pools, v_pools, stream):
        return LapsGraph(self, layers, len_bucket, depth, max_pages, k_pools, v_pools, stream)


class LapsGraph:
    """One captured (length bucket, depth) shape of the whole stack."""

    def __init__(self, ctx: LapsCtx, layers, len_bucket, depth, max_pages, k_pools, v_pools, stream):
        self.ctx, self.len_bucket, self.depth, self.max_pages = ctx, len_bucket, depth, max_pages
        self._keep = (layers, k_pools, v_pools)  # the graph holds raw pointers into these
        arr = ctx._weights_array(layers)
        kp = (C.c_void_p * len(layers))(*[t.data_ptr() for t in k_pools])
        vp = (C.c_void_p * len(layers))(*[t.data_ptr() for t in v_pools])
        self._h = C.c_void_p()
        ctx._guard_pools(k_pools[0])
        _after_current(stream)
        _check(lib().laps_graph_capture(ctx._h, arr, C.c_int32(len_bucket), C.c_int32(depth), C.c_int32(max_pages), kp, vp,
                                        C.c_void_p(stream.cuda_stream), C.byref(self._h)))

    def laps_graph_stage(self, n_real, seq_len, prefix_len, page_table, x_rows, stream=None):
        """x_rows: fp32 [sum of the lengths, hidden] on the device, the sequences packed in slot order (or None)."""
        assert page_table is None or page_table.shape[1] == self.max_pages
        n_rows = 0 if x_rows is None else int(x_rows.shape[0])
        _after_current(stream)       # the staged arrays may have been filled on the current stream
        _check(lib().laps_graph_stage(self._h, C.c_int32(n_real), _p(seq_len), _p(prefix_len), _p(page_table), _p(x_rows),
                                      C.c_int32(n_rows), _stream(stream)))

    def laps_graph_replay(self, stream=None):
        _check(lib().laps_graph_replay(self._h, _stream(stream)))

    def laps_graph_read_output(self, n_rows: int, dst: torch.Tensor, stream=None):
        _after_current(stream)       # dst may be a fresh allocation of the current stream
        _check(lib().laps_graph_read_output(self._h, C.c_int32(n_rows), _p(dst), _stream(stream)))
        return dst

    def laps_graph_device_bytes(self) -> int:
        return int(lib().laps_graph_device_bytes(self._h))

    def close(self):
        if self._h:
            lib().laps_graph_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
