"""A stack of decoder layers' worth of ClusterKV state, driven the way the paper runs it:
clustering enqueued on a side stream so that it overlaps the rest of the layer's work
(Section IV-B), attention sinks kept out of the clustering and always attended
(Section III-B), generated tokens clustered among themselves every m steps and attended
in full until then (Section III-B), and the first layers left on the full KV cache
(Section V-A).  Only stream/event plumbing and bookkeeping: every computation is a call
into the library.
"""
from __future__ import annotations

import torch

from .binding import (ClusterState, Shape, ck_full_decode_attn, ck_workspace_bytes, decode_step,
                      CK_WS_SPARSE_ATTN, _workspace)


class LayerStack:
    def __init__(self, n_layers: int, S: int, Hq: int, Hkv: int, n_prefill: int, max_new: int,
                 C0: int, budget: int, device, n_sink: int = 16, full_kv_layers: int = 2,
                 m: int = 320, c_plus: int = 4, n_iter: int = 10, dtype: int = 0):
        self.L, self.n_sink, self.m, self.c_plus, self.n_iter = n_layers, n_sink, m, c_plus, n_iter
        self.full_kv_layers = min(full_kv_layers, n_layers)
        self.C0, self.n_prefill = C0, n_prefill
        N_cap = n_prefill + max_new
        C_cap = C0 + c_plus * (max_new // m)
        self.sh = Shape(S, Hq, Hkv, N_cap, C_cap, dtype=dtype)
        self.device = device
        self.side = torch.cuda.Stream(device)             # default priority
        self.ready = [torch.cuda.Event() for _ in range(n_layers)]
        self.pending = [False] * n_layers
        self.states = [None if l < self.full_kv_layers else
                       ClusterState(self.sh, device, budget, max_recent=m, n_sink=n_sink)
                       for l in range(n_layers)]
        self.clustered_to = [n_sink] * n_layers           # tokens below are sinks or in the table
        self.full_out = torch.zeros(S, Hq, self.sh.d, dtype=self.sh.torch_dtype, device=device)
        self.full_ws = _workspace(ck_workspace_bytes(self.sh, CK_WS_SPARSE_ATTN, N_cap),
                                  self.full_out)

    def compressed(self, layer: int) -> bool:
        return layer >= self.full_kv_layers

    def _on_side(self, layer: int, fn):
        """Run fn on the side stream after everything enqueued so far on the current one."""
        cur = torch.cuda.current_stream(self.device)
        self.side.wait_stream(cur)
        with torch.cuda.stream(self.side):
            fn()
            self.ready[layer].record(self.side)
        self.pending[layer] = True

    def cluster_prefill(self, layer: int, K, init_idx):
        """Cluster tokens [n_sink, n_prefill) of a layer into C0 clusters, asynchronously."""
        if not self.compressed(layer):
            return
        st = self.states[layer]
        st.n_clusters = 0
        n = self.n_prefill - self.n_sink
        self._on_side(layer, lambda: st.cluster(K, init_idx, self.n_sink, n, self.C0, self.n_iter))
        self.clustered_to[layer] = self.n_prefill

    def cluster_generated(self, layer: int, K, n_ctx: int, init_idx) -> bool:
        """If m generated tokens of the layer are still unclustered, cluster them into c_plus
        new clusters on the side stream.  init_idx: [S, Hkv, c_plus] rows among those tokens."""
        if not self.compressed(layer) or n_ctx - self.clustered_to[layer] < self.m:
            return False
        st = self.states[layer]
        t0 = self.clustered_to[layer]
        self._on_side(layer, lambda: st.cluster(K, init_idx, t0, self.m, self.c_plus, self.n_iter))
        self.clustered_to[layer] = t0 + self.m
        return True

    def decode(self, layer: int, q, K, V, n_ctx: int):
        """Attention output of one layer for one decode step over a context of n_ctx tokens."""
        if self.pending[layer]:
            torch.cuda.current_stream(self.device).wait_event(self.ready[layer])
            self.pending[layer] = False
        if not self.compressed(layer):
            ck_full_decode_attn(self.sh, q, K, V, n_ctx, self.full_out, workspace=self.full_ws)
            return self.full_out
        return decode_step(self.states[layer], q, K, V, n_sink=self.n_sink,
                           recent_begin=self.clustered_to[layer], recent_end=n_ctx)
