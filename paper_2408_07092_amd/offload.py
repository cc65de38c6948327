"""Offload arrangement of Double Sparsity (Sec. 5.1): the label cache lives on the
GPU, the full K/V caches in pinned host memory, and only the k selected rows of
a layer cross the host link, into one half of a double buffer, while the
previous layer's rows are being attended.

This module only sequences the library's calls on two streams; every step runs
in the library's kernels:
    select stream : ds_select(l)            -> idx[l % 2]
    copy stream   : ds_gather_rows_host(l)  -> rows[l % 2]   (reads pinned host memory)
    main stream   : ds_attend_rows(l)       -> out[l]
Row fetch of layer l+1 overlaps the attention of layer l.  The paper obtains
layer l+1's query early by pushing layer l's embedding through W_q of layer l+1
(Sec. 5.1); with `predict` the select stream does exactly that
(ds_predict_query) and selects with the approximate query, while the attention
uses the layer's real query.  Without it the given queries select, which
exercises the same transport.
"""
from __future__ import annotations

import torch

from . import binding as ds


class OffloadDecoder:
    def __init__(self, shp: ds.DsShape, device="cuda"):
        self.shp = shp
        self.dev = torch.device(device)
        B, Hq, Hkv, d, k = shp.B, shp.Hq, shp.Hkv, shp.d, shp.k
        self.idx = [torch.empty((B, Hkv, k), dtype=torch.int32, device=self.dev) for _ in range(2)]
        self.rows = [torch.empty((B, Hkv, k, 2, d), dtype=torch.float16, device=self.dev) for _ in range(2)]
        # select and attend run concurrently on different streams: one workspace each
        self.ws_sel = [ds.ds_workspace_alloc(shp, self.dev) for _ in range(2)]
        self.ws_att = ds.ds_workspace_alloc(shp, self.dev)
        self.s_sel = torch.cuda.Stream(device=self.dev)
        self.s_copy = torch.cuda.Stream(device=self.dev)
        self.ev_sel = [torch.cuda.Event() for _ in range(2)]
        self.ev_rows = [torch.cuda.Event() for _ in range(2)]
        self.ev_free = [torch.cuda.Event() for _ in range(2)]

    def decode(self, layers, outs, predict=None):
        """layers: list of (q, label, channels, K_pinned, V_pinned); outs: list of
        [B,Hq,d] fp32 device tensors.  predict: None, or per layer (x, Wq, q_pred) with
        x [B,Dm] the embedding the prediction starts from, Wq [Hq*d, Dm] the layer's
        query projection and q_pred [B,Hq,d] fp16 receiving the approximate query that
        then selects the layer's rows.  Enqueues one decode step over all layers on the
        current stream (plus the two helper streams) and returns without synchronising."""
        main = torch.cuda.current_stream(self.dev)
        start = torch.cuda.Event()
        start.record(main)
        self.s_sel.wait_event(start)
        self.s_copy.wait_event(start)
        n = len(layers)

        def fetch(l):
            q, label, ch, Kp, Vp = layers[l]
            s = l % 2
            if l >= 2:
                self.s_sel.wait_event(self.ev_free[s])     # attention of layer l-2 released the buffers
            with torch.cuda.stream(self.s_sel):
                if predict is not None:
                    x, Wq, q_pred = predict[l]
                    ds.ds_predict_query(x, Wq, q_pred)
                    q = q_pred
                ds.ds_select(q, label, ch, self.idx[s], self.ws_sel[s], self.shp)
                self.ev_sel[s].record(self.s_sel)
            with torch.cuda.stream(self.s_copy):
                self.s_copy.wait_event(self.ev_sel[s])
                ds.ds_gather_rows_host(Kp, Vp, self.idx[s], self.rows[s], self.shp)
                self.ev_rows[s].record(self.s_copy)

        fetch(0)
        for l in range(n):
            if l + 1 < n:
                fetch(l + 1)
            s = l % 2
            main.wait_event(self.ev_rows[s])
            ds.ds_attend_rows(layers[l][0], self.rows[s], outs[l], self.ws_att, self.shp)
            self.ev_free[s].record(main)
