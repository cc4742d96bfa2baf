"""Sub-part ping-pong on one GPU (the paper's Sec. III-B/III-C mechanism on a single device).

The vertex table of a source block lives in pinned host memory, split into k row ranges (sub-parts);
the context table stays on the device.  Three device buffers rotate: while sub-part s trains on the
compute stream, sub-part s+1 is copied host-to-device on a second stream and sub-part s-1 device-to-host
on a third.  Pairs must be grouped by sub-part of their source id.  This module only moves memory and
orders streams (torch tensors, streams, events); all arithmetic is the library's ne_train_block.
"""
from __future__ import annotations

import torch

from . import ne_set_vertex_window, ne_train_block


class SubpartTrainer:
    def __init__(self, tables, vertex_host: torch.Tensor, first_row: int, k: int):
        """vertex_host: pinned CPU fp32 [rows][dim] holding vertex rows first_row .. first_row+rows."""
        assert vertex_host.is_pinned() and vertex_host.dtype == torch.float32 and vertex_host.dim() == 2
        self.tables, self.host, self.first_row, self.k = tables, vertex_host, first_row, k
        rows = vertex_host.shape[0]
        self.bounds = [rows * i // k for i in range(k + 1)]
        cap = max(self.bounds[i + 1] - self.bounds[i] for i in range(k))
        dev = tables.context.device
        self.buffers = [torch.empty((cap, vertex_host.shape[1]), dtype=torch.float32, device=dev) for _ in range(3)]
        self.s_in, self.s_train, self.s_out = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()

    def subpart_of(self, src_ids: torch.Tensor) -> torch.Tensor:
        """Index of the sub-part each (absolute) source id belongs to."""
        local = src_ids.long() - self.first_row
        edges = torch.tensor(self.bounds[1:-1], device=local.device, dtype=local.dtype)
        return torch.bucketize(local, edges, right=True)

    def run(self, alias, pairs_by_subpart, B: int, K: int, lrs_by_subpart, sample_bases):
        """pairs_by_subpart[s]: CUDA int32 [n_s][2] whose sources all lie in sub-part s (absolute ids)."""
        k = self.k
        # Everything the caller has enqueued on its current stream (workspace clearing and table init of
        # ne_create_tables, the pair tensors, the context table) must be done before the private streams
        # start; and the caller's stream must see the result afterwards.
        cur = torch.cuda.current_stream()
        for st in (self.s_in, self.s_train, self.s_out):
            st.wait_stream(cur)
        loaded = [torch.cuda.Event() for _ in range(k)]
        trained = [torch.cuda.Event() for _ in range(k)]
        stored = [torch.cuda.Event() for _ in range(k)]
        for s in range(k):
            lo, hi = self.bounds[s], self.bounds[s + 1]
            buf = self.buffers[s % 3][: hi - lo]
            # host -> device: the buffer must have been written back by its previous user (s - 3)
            if s >= 3:
                self.s_in.wait_event(stored[s - 3])
            with torch.cuda.stream(self.s_in):
                buf.copy_(self.host[lo:hi], non_blocking=True)
            loaded[s].record(self.s_in)
            # train
            self.s_train.wait_event(loaded[s])
            ne_set_vertex_window(self.tables, buf, self.first_row + lo)
            p = pairs_by_subpart[s]
            if p.shape[0] > 0:
                ne_train_block(self.tables, alias, p, B, K, lrs_by_subpart[s], sample_bases[s], stream=self.s_train)
            trained[s].record(self.s_train)
            # device -> host
            self.s_out.wait_event(trained[s])
            with torch.cuda.stream(self.s_out):
                self.host[lo:hi].copy_(buf, non_blocking=True)
            stored[s].record(self.s_out)
        cur.wait_stream(self.s_train)      # the context table's updates
        cur.wait_stream(self.s_out)        # the vertex rows' way back to the host
        for ev in stored:                  # the host copy is complete when run() returns
            ev.synchronize()
