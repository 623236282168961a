"""Shared plumbing of the GPU parity tests: builds a seeded case on the host, runs it through the
C-ABI binding on the device and through the fp64 oracle on the CPU, and measures the difference."""
from __future__ import annotations

import os
import time

import numpy as np
import torch

from oracle import laps_oracle as O
from paper_2601_11589_amd import api, inputs

REL_L2_TOL = 5e-3   # spec tolerance for layer / stack outputs vs the fp64 oracle
MAX_ABS_TOL = 2e-2


_PROGRESS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "gpu_tests_progress.log")


def progress(msg: str):
    """One line per finished step of a long test (an fp64 pass of the oracle takes up to a minute or two of host time),
    printed and appended to a log file: pytest holds the printed text back until the test ends, and a harness that
    watches for output would otherwise see nothing for the length of the longest test."""
    line = f"{time.strftime('%H:%M:%S')} {msg}"
    print(line, flush=True)
    try:
        os.makedirs(os.path.dirname(_PROGRESS), exist_ok=True)
        with open(_PROGRESS, "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def widen_layer(w_bits: dict) -> dict:
    return {k: inputs.bf16_bits_to_f64(v) for k, v in w_bits.items()}


class LazyWideLayers:
    """Indexable of fp64 weight dicts that widens one layer at a time (full-size layers are ~4 GB in fp64)."""

    def __init__(self, host_layers):
        self.host_layers = host_layers

    def __len__(self):
        return len(self.host_layers)

    def __getitem__(self, i):
        return widen_layer(self.host_layers[i])


def errors(got: np.ndarray, want: np.ndarray):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    rel = float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))
    mx = float(np.max(np.abs(got - want))) if got.size else 0.0
    return rel, mx


class Case:
    """One ragged batch with weights, activations and cached prefix KV, all seeded."""

    def __init__(self, cfg, new_len, prefix_len, seed, n_layers=None, spare_pages=3, qkv_bias=False):
        self.cfg = cfg
        self.n_layers = n_layers or cfg.n_layers
        self.new_len = np.asarray(new_len, np.int32)
        self.prefix_len = np.asarray(prefix_len, np.int32)
        self.seed = seed
        self.n = len(self.new_len)
        self.cu = np.concatenate([[0], np.cumsum(self.new_len)]).astype(np.int32)
        self.T = int(self.cu[-1])
        self.page_table, self.n_pages = inputs.make_page_table(seed, self.new_len, self.prefix_len, spare_pages)
        self.host_layers = [inputs.make_layer_weights(cfg, seed, l) for l in range(self.n_layers)]
        if qkv_bias:
            for l, w in enumerate(self.host_layers):
                w["b_qkv"] = inputs.make_qkv_bias(cfg, seed, l)
        self.x = inputs.make_activations(cfg, seed, self.T)
        # prefix KV bits: [layer][seq] -> (k, v) or None
        self.prefix = [[inputs.make_prefix_kv(cfg, seed, l, i, int(h)) if h > 0 else None
                        for i, h in enumerate(self.prefix_len)] for l in range(self.n_layers)]

    # ---- oracle side
    def oracle(self, storage_rounding=False, seqs=None):
        """fp64 stack output.  `seqs` restricts to a subset of sequences (outputs are per-sequence independent)."""
        ids = list(range(self.n)) if seqs is None else list(seqs)
        rows = np.concatenate([np.arange(self.cu[i], self.cu[i + 1]) for i in ids]) if ids else np.zeros(0, int)
        pk = [[None if self.prefix[l][i] is None else inputs.bf16_bits_to_f64(self.prefix[l][i][0]) for i in ids]
              for l in range(self.n_layers)]
        pv = [[None if self.prefix[l][i] is None else inputs.bf16_bits_to_f64(self.prefix[l][i][1]) for i in ids]
              for l in range(self.n_layers)]
        t0 = time.perf_counter()
        y, ks, vs = O.stack_forward(self.cfg, LazyWideLayers(self.host_layers), self.x[rows].astype(np.float64),
                                    [int(self.new_len[i]) for i in ids], pk, pv, storage_rounding)
        progress(f"oracle pass done: {len(ids)} sequences, {len(rows)} rows, {self.n_layers} layers, "
                 f"storage_rounding={storage_rounding}, {time.perf_counter() - t0:.1f} s")
        return y, ks, vs, rows

    # ---- device side
    def to_device(self, ctx: api.LapsCtx):
        self.ctx = ctx
        self.dev_layers = [ctx.upload_layer(w) for w in self.host_layers]
        self.k_pools, self.v_pools = ctx.new_pools(self.n_pages, self.n_layers)
        for p in self.k_pools + self.v_pools:      # poison: unwritten slots must never reach an output
            p.view(torch.int16).fill_(0x7FC0)      # bf16 NaN
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
        torch.cuda.synchronize()
        return self

    def run_stack(self):
        y = self.ctx.laps_prefill_stack(self.dev_layers, self.d_cu, None, self.d_prefix_len, self.d_page_table,
                                        self.k_pools, self.v_pools, self.d_x)
        torch.cuda.synchronize()
        return y.cpu().numpy()

    def gathered_new_kv(self, layer: int):
        """Appended K/V of every sequence read back from the pools, token-major float arrays."""
        k, v = self.ctx.laps_kv_gather(self.d_cu, self.d_prefix_len, self.d_page_table, self.k_pools[layer],
                                       self.v_pools[layer], self.T)
        torch.cuda.synchronize()
        return k.float().cpu().numpy(), v.float().cpu().numpy()
