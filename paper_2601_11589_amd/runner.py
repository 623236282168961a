"""Host harness over the C-ABI binding: runs a planned set of requests the way the paper's
single-instance temporal disaggregation does (Section 3.2): every GPU step is homogeneous -
either one short bucket batch replayed as a captured graph (Section 3.1) or one chunk of one
long request on the un-captured path.  Only sequencing and input placement live here; all
arithmetic is inside liblaps.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from . import api


@dataclass
class StagedBatch:
    """Device-resident inputs of one planned short batch: the requests' rows packed one after the other."""
    len_bucket: int
    depth: int
    graph_ok: int
    req_ids: list
    n_real: int
    seq_len: torch.Tensor      # int32 [n_real]
    prefix_len: torch.Tensor   # int32 [n_real]
    page_table: torch.Tensor   # int32 [n_real, max_pages]
    x_rows: torch.Tensor       # fp32 [real_tokens, hidden], packed
    cu: torch.Tensor           # int32 [n_real + 1] packed cu_seqlens (used by the un-captured path)
    real_tokens: int


def stage_short_batches(plan: dict, new_len, prefix_len, page_table, cu, d_x: torch.Tensor, hidden: int):
    """Places every planned short batch's inputs in HBM (outside any timed region).
    new_len/prefix_len/page_table/cu are host arrays; d_x is the packed fp32 [T, hidden] on the device."""
    out = []
    for b in plan["batches"]:
        ids = b["req_ids"]
        lb, n_real = b["len_bucket"], len(ids)
        sl = torch.tensor([int(new_len[i]) for i in ids], dtype=torch.int32, device="cuda")
        pl = torch.tensor([int(prefix_len[i]) for i in ids], dtype=torch.int32, device="cuda")
        pt = torch.from_numpy(np.ascontiguousarray(page_table[ids])).cuda()
        x = torch.cat([d_x[int(cu[i]):int(cu[i + 1])] for i in ids])
        c = torch.tensor(np.concatenate([[0], np.cumsum([int(new_len[i]) for i in ids])]), dtype=torch.int32,
                         device="cuda")
        out.append(StagedBatch(lb, b["depth"], b["graph_ok"], ids, n_real, sl, pl, pt, x, c,
                               int(sum(int(new_len[i]) for i in ids))))
    # the tensors were filled on torch's current stream; the runner launches on a stream of its own, which does not
    # wait for that one by itself
    torch.cuda.current_stream().synchronize()
    return out


class ShortRunner:
    """Captures one graph per (length bucket, depth) shape on first use and replays staged batches."""

    def __init__(self, ctx: api.LapsCtx, layers, k_pools, v_pools, max_pages: int, stream: torch.cuda.Stream):
        self.ctx, self.layers, self.k_pools, self.v_pools = ctx, layers, k_pools, v_pools
        self.max_pages, self.stream = max_pages, stream
        self.graphs = {}
        self.capture_s = {}

    def graph_for(self, len_bucket: int, depth: int) -> api.LapsGraph:
        key = (len_bucket, depth)
        if key not in self.graphs:
            import time
            t0 = time.perf_counter()
            self.graphs[key] = self.ctx.laps_graph_capture(self.layers, len_bucket, depth, self.max_pages,
                                                           self.k_pools, self.v_pools, self.stream)
            self.capture_s[key] = time.perf_counter() - t0
        return self.graphs[key]

    def run(self, sb: StagedBatch, out: torch.Tensor | None = None):
        """Enqueues stage + replay (or the un-captured path) on the runner's stream."""
        if sb.graph_ok:
            g = self.graph_for(sb.len_bucket, sb.depth)
            g.laps_graph_stage(sb.n_real, sb.seq_len, sb.prefix_len, sb.page_table, sb.x_rows, self.stream)
            g.laps_graph_replay(self.stream)
            if out is not None:
                g.laps_graph_read_output(sb.real_tokens, out, self.stream)
            return out
        with torch.cuda.stream(self.stream):
            return self.ctx.laps_prefill_stack(self.layers, sb.cu, None, sb.prefix_len, sb.page_table, self.k_pools,
                                               self.v_pools, sb.x_rows, out, self.stream)

    def close(self):
        for g in self.graphs.values():
            g.close()
        self.graphs = {}


def run_long_chunks(ctx: api.LapsCtx, layers, k_pools, v_pools, x_req: torch.Tensor, prefix_len: int,
                    page_table_row: torch.Tensor, chunks, stream: torch.cuda.Stream, out: torch.Tensor):
    """Advances one long request chunk by chunk (each chunk is a re-prefill over everything before it).
    x_req: fp32 [L, hidden] on the device; page_table_row: int32 [1, max_pages]; out: fp32 [L, hidden].

    The per-chunk length / prefix arrays are read by kernels that run asynchronously, so they are
    allocated on `stream` (their memory is then only recycled in that stream's order) and returned so
    that the caller can keep them alive until it synchronises."""
    keep = []
    done = 0
    with torch.cuda.stream(stream):
        for c in chunks:
            cu = torch.tensor([0, c], dtype=torch.int32, device="cuda")
            pre = torch.tensor([prefix_len + done], dtype=torch.int32, device="cuda")
            keep.append((cu, pre))
            ctx.laps_prefill_stack(layers, cu, None, pre, page_table_row, k_pools, v_pools, x_req[done:done + c],
                                   out[done:done + c], stream)
            done += c
    return keep
