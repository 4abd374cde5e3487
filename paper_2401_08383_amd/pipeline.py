"""Pre-allocated buffers around the C ABI so that a timed loop calls the library and nothing else.

``MoELayerRun`` holds every output and workspace of one MoE layer pass
(gate -> dispatch -> expert FFN -> combine, all enqueued on the current stream with no host
synchronisation in between; with ``fused=True`` the dispatch is index-only and
moe_expert_ffn_fused reads and writes the unsorted token rows, so no combine call follows);
``AffinityRun`` does the same for the affinity statistic over a device-resident trace
(affinity_statistics, or affinity_histogram + placement_locality).  Argument marshalling only.
"""
from __future__ import annotations

import torch

from . import binding as B


class MoELayerRun:
    def __init__(self, x, w_gate, w1, w2, k, renormalize=False, expert_map=None, E_local=None, topk_idx=None,
                 act=B.EXF_ACT_GELU_ERF, fused=False):
        self.lib = B.lib()
        self.fused = bool(fused)
        self.x, self.w_gate, self.w1, self.w2 = x, w_gate, w1, w2
        self.T, self.d = x.shape
        self.E = w_gate.shape[0]
        self.E_local, self.f = w1.shape[0], w1.shape[1]
        if E_local is not None:
            assert E_local == self.E_local
        self.k, self.renorm, self.act = k, int(bool(renormalize)), act
        self.expert_map = expert_map
        self.forced_idx = topk_idx  # routing supplied by the caller (trace-driven configurations)
        self.dt = B.dtype_code(x)
        dev = x.device
        A = self.A = self.T * k
        self.topk_idx = torch.empty((self.T, k), dtype=torch.int32, device=dev)
        self.topk_w = torch.empty((self.T, k), dtype=torch.float32, device=dev)
        self.x_sorted = None if self.fused else torch.empty((A, self.d), dtype=x.dtype, device=dev)
        self.src_of_sorted = torch.empty(A, dtype=torch.int32, device=dev)
        self.sorted_of_src = torch.empty(A, dtype=torch.int32, device=dev)
        self.expert_counts = torch.empty(self.E_local, dtype=torch.int32, device=dev)
        self.expert_offsets = torch.empty(self.E_local + 1, dtype=torch.int32, device=dev)
        self.y_sorted = None if self.fused else torch.empty((A, self.d), dtype=x.dtype, device=dev)
        self.out = torch.empty((self.T, self.d), dtype=x.dtype, device=dev)
        self.ws_dispatch = torch.empty(max(self.lib.moe_dispatch_workspace_bytes(self.T, k, self.E_local), 256),
                                       dtype=torch.uint8, device=dev)
        if self.fused:
            ffn_bytes = self.lib.moe_expert_ffn_fused_workspace_bytes(self.T, k, self.d, self.f, self.E_local, self.dt)
            if ffn_bytes == 0:
                raise ValueError("moe_expert_ffn_fused does not take this shape / dtype")
        else:
            ffn_bytes = self.lib.moe_expert_ffn_workspace_bytes(A, self.d, self.f, self.E_local, self.dt)
        self.ws_ffn = torch.empty(max(ffn_bytes, 256), dtype=torch.uint8, device=dev)

    # each method enqueues one entry point on the current stream
    def gate(self):
        B._check(self.lib.moe_gate_topk(self.x.data_ptr(), self.w_gate.data_ptr(), self.T, self.d, self.E, self.k, self.renorm,
                                        self.dt, None, self.topk_idx.data_ptr(), self.topk_w.data_ptr(), B._stream()))

    def dispatch(self):
        idx = self.forced_idx if self.forced_idx is not None else self.topk_idx
        B._check(self.lib.moe_dispatch(self.x.data_ptr(), idx.data_ptr(), B._ptr(self.expert_map), self.T, self.d, self.k,
                                       self.E, self.E_local, self.dt, B._ptr(self.x_sorted), self.src_of_sorted.data_ptr(),
                                       self.sorted_of_src.data_ptr(), self.expert_counts.data_ptr(),
                                       self.expert_offsets.data_ptr(), self.ws_dispatch.data_ptr(), self.ws_dispatch.numel(),
                                       B._stream()))

    def ffn(self):
        if self.fused:
            B._check(self.lib.moe_expert_ffn_fused(self.x.data_ptr(), self.src_of_sorted.data_ptr(),
                                                   self.sorted_of_src.data_ptr(), self.topk_w.data_ptr(),
                                                   self.expert_offsets.data_ptr(), self.w1.data_ptr(), None, self.w2.data_ptr(),
                                                   None, self.T, self.k, self.d, self.f, self.E_local, self.act, self.dt,
                                                   self.out.data_ptr(), self.ws_ffn.data_ptr(), self.ws_ffn.numel(), B._stream()))
            return
        B._check(self.lib.moe_expert_ffn(self.x_sorted.data_ptr(), self.expert_offsets.data_ptr(), self.w1.data_ptr(), None,
                                         self.w2.data_ptr(), None, self.A, self.d, self.f, self.E_local, self.act, self.dt,
                                         self.y_sorted.data_ptr(), self.ws_ffn.data_ptr(), self.ws_ffn.numel(), B._stream()))

    def combine(self):
        if self.fused:
            return
        B._check(self.lib.moe_combine(self.y_sorted.data_ptr(), self.sorted_of_src.data_ptr(), self.topk_w.data_ptr(), self.T,
                                      self.d, self.k, self.dt, self.out.data_ptr(), B._stream()))

    def step(self):
        self.gate()
        self.dispatch()
        self.ffn()
        self.combine()


class AffinityRun:
    def __init__(self, trace, placement, E, G, one_pass=True):
        self.lib = B.lib()
        self.one_pass = bool(one_pass)  # step() = affinity_statistics, else affinity_histogram + placement_locality
        self.trace, self.placement = trace, placement
        self.L, self.N = trace.shape
        self.E, self.G = E, G
        dev = trace.device
        pairs = max(self.L - 1, 0)
        self.counts = torch.empty((pairs, E, E), dtype=torch.int64, device=dev)
        self.loads = torch.empty((self.L, E), dtype=torch.int64, device=dev)
        self.cond_prob = torch.empty((pairs, E, E), dtype=torch.float32, device=dev)
        self.n_invalid = torch.empty(1, dtype=torch.int64, device=dev)
        self.local_per_pair = torch.empty(pairs, dtype=torch.int64, device=dev)
        self.ws_hist = torch.empty(max(self.lib.affinity_histogram_workspace_bytes(self.L, self.N, E), 256), dtype=torch.uint8,
                                   device=dev)
        self.ws_loc = torch.empty(max(self.lib.placement_locality_workspace_bytes(self.L, self.N), 256), dtype=torch.uint8,
                                  device=dev)

    def histogram(self, trace=None):
        t = self.trace if trace is None else trace
        B._check(self.lib.affinity_histogram(t.data_ptr(), self.L, self.N, self.E, self.counts.data_ptr(),
                                             self.loads.data_ptr(), self.cond_prob.data_ptr(), self.n_invalid.data_ptr(),
                                             self.ws_hist.data_ptr(), self.ws_hist.numel(), B._stream()))

    def locality(self, trace=None):
        t = self.trace if trace is None else trace
        B._check(self.lib.placement_locality(t.data_ptr(), self.placement.data_ptr(), self.L, self.N, self.E, self.G,
                                             self.local_per_pair.data_ptr(), self.ws_loc.data_ptr(), self.ws_loc.numel(),
                                             B._stream()))

    def statistics(self, trace=None):
        """Both results from one pass over the trace (affinity_statistics)."""
        t = self.trace if trace is None else trace
        B._check(self.lib.affinity_statistics(t.data_ptr(), self.placement.data_ptr(), self.L, self.N, self.E, self.G,
                                              self.counts.data_ptr(), self.loads.data_ptr(), self.cond_prob.data_ptr(),
                                              self.n_invalid.data_ptr(), self.local_per_pair.data_ptr(), self.ws_hist.data_ptr(),
                                              self.ws_hist.numel(), B._stream()))

    def step(self):
        if self.one_pass:
            self.statistics()
        else:
            self.histogram()
            self.locality()
