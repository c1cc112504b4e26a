"""Buffer management for a per-layer StructKV scoring sweep (Alg. 1 lines 4, 6, 16, 17).

Owns the torch buffers and calls the C ABI in order; no arithmetic happens here.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


class LayerSweep:
    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, window: int, dtype: torch.dtype,
                 seq_lens: Sequence[int], k_per_seq: Sequence[int], lam: float = 0.9, causal: bool = False,
                 scale: float = 0.0, n_layers_out: int = 1, device="cuda"):
        self.Hq, self.G, self.d, self.w = n_q_heads, n_kv_heads, head_dim, window
        self.seq_lens = [int(n) for n in seq_lens]
        self.k_per_seq = [int(k) for k in k_per_seq]
        self.batch = len(self.seq_lens)
        self.cu = [0]
        for n in self.seq_lens:
            self.cu.append(self.cu[-1] + n)
        self.total = self.cu[-1]
        self.lam = float(lam)
        self.keep_tail = window
        self.rows_per_seq = [k + self.keep_tail for k in self.k_per_seq]
        self.rows = sum(self.rows_per_seq)
        code = {torch.float32: B.STRUCTKV_DTYPE_F32, torch.bfloat16: B.STRUCTKV_DTYPE_BF16}[dtype]
        self.shape = B.make_shape(n_q_heads, n_kv_heads, head_dim, window, code, causal, scale)
        # sized for the fused layer step (scoring and selection scratch live together); the separate calls need less
        ws_bytes = B.structkv_layer_step_workspace_bytes(self.shape, self.batch, self.total)
        dev = torch.device(device)
        self.workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        # second score vector + a workspace of its own for the selection, used when selection and gather of one
        # layer run on a side stream while the next layer is being scored (sweep_overlapped)
        topk_bytes = B.structkv_workspace_bytes(None, self.batch, self.total)
        self.topk_workspace = torch.empty(max(topk_bytes, 256), dtype=torch.uint8, device=dev)
        self._indeg2 = [torch.empty(self.total, dtype=torch.float32, device=dev) for _ in range(2)]
        self.indeg = self._indeg2[0]
        self.centrality = torch.zeros(self.total, dtype=torch.float32, device=dev)
        self.entropy = torch.empty(max(self.batch, 1), dtype=torch.float32, device=dev)
        self.entropy_per_head = torch.empty(max(self.batch, 1), n_q_heads, dtype=torch.float32, device=dev)
        self.idx_kv = torch.empty(max(self.rows, 1), dtype=torch.int32, device=dev)
        self.idx_struct = torch.empty(max(self.rows, 1), dtype=torch.int32, device=dev)
        self.k_cache = torch.empty(n_layers_out, n_kv_heads, max(self.rows, 1), head_dim, dtype=dtype, device=dev)
        self.v_cache = torch.empty_like(self.k_cache)

    def reset(self) -> None:
        self.centrality.zero_()

    def score(self, q_win: torch.Tensor, k: torch.Tensor, stream=None) -> None:
        B.structkv_score_layer(self.shape, q_win, k, self.cu, self.indeg, self.entropy,
                               self.entropy_per_head, self.workspace, stream)

    def accumulate(self, stream=None) -> None:
        B.structkv_accumulate_centrality(self.centrality, self.indeg, self.lam, 1.0 / self.w, stream)

    def score_accumulate(self, q_win: torch.Tensor, k: torch.Tensor, stream=None) -> None:
        """score() then accumulate() as one call of the library (same results, one launch fewer)."""
        B.structkv_score_layer_accumulate(self.shape, q_win, k, self.cu, self.indeg, self.centrality, self.lam,
                                          1.0 / self.w, self.entropy, self.entropy_per_head, self.workspace, stream)

    def pivot_metrics(self, q_win: torch.Tensor, k: torch.Tensor, top_frac: float = 0.1, stream=None):
        """Eq. 5-6 for this layer: (sparsity [B], variance [B]) device tensors; the entropy of Eq. 4 is self.entropy
        after score().  Allocates its scratch on first use."""
        if getattr(self, "_pivot_ws", None) is None:
            nbytes = B.structkv_pivot_workspace_bytes(self.shape, max(self.seq_lens) if self.seq_lens else 0)
            self._pivot_ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.centrality.device)
            self.sparsity = torch.zeros(max(self.batch, 1), dtype=torch.float32, device=self.centrality.device)
            self.variance = torch.zeros_like(self.sparsity)
        B.structkv_pivot_metrics(self.shape, q_win, k, self.cu, top_frac, self.sparsity, self.variance,
                                 self._pivot_ws, stream)
        return self.sparsity, self.variance

    def score_pivot(self, q_win: torch.Tensor, k: torch.Tensor, top_frac: float = 0.1, stream=None):
        """score() and pivot_metrics() from one scoring of the layer: fills indeg, entropy, entropy_per_head and
        returns (sparsity [B], variance [B])."""
        if getattr(self, "_pivot_ws", None) is None:
            self.pivot_metrics(q_win, k, top_frac, stream)          # allocates the scratch and the outputs
        B.structkv_score_layer_pivot(self.shape, q_win, k, self.cu, top_frac, self.indeg, self.entropy,
                                     self.entropy_per_head, self.sparsity, self.variance, self._pivot_ws, stream)
        return self.sparsity, self.variance

    def select_kv(self, stream=None) -> None:
        """Eq. 13: per-layer storage indices from this layer's scores."""
        B.structkv_select_topk(self.indeg, self.cu, self.k_per_seq, self.keep_tail, self.idx_kv,
                               self.workspace, stream)

    def select_struct(self, k_per_seq: Optional[Sequence[int]] = None, stream=None) -> None:
        """Eq. 10: propagation indices from the accumulated centrality."""
        B.structkv_select_topk(self.centrality, self.cu, k_per_seq or self.k_per_seq, self.keep_tail,
                               self.idx_struct, self.workspace, stream)

    def gather(self, k: torch.Tensor, v: torch.Tensor, slot: int = 0, stream=None) -> None:
        B.structkv_gather_kv(k, v, self.k_cache[slot], self.v_cache[slot], self.cu, self.rows_per_seq,
                             self.idx_kv, stream)

    def layer(self, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, slot: int = 0, stream=None) -> None:
        """One pass of the hot path over one layer -- score -> accumulate -> select -> gather -- as ONE call of
        the library (structkv_layer_step: same results as layer_separate_calls, fewer launches)."""
        B.structkv_layer_step(self.shape, q_win, k, v, self.cu, self.k_per_seq, self.keep_tail, self.indeg,
                              self.centrality, self.lam, 1.0 / self.w, self.entropy, self.entropy_per_head,
                              self.idx_kv, self.k_cache[slot], self.v_cache[slot], self.workspace, stream)

    def layer_separate_calls(self, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, slot: int = 0,
                             stream=None) -> None:
        """The same layer through the four entry points one by one."""
        self.score(q_win, k, stream)
        self.accumulate(stream)
        self.select_kv(stream)
        self.gather(k, v, slot, stream)

    def _chains(self, n: int):
        """Per-chain buffers of sweep_chains (chain 0 uses the sweep's own; the others are allocated on first use)."""
        chains = getattr(self, "_chain_bufs", None)
        if chains is None:
            chains = self._chain_bufs = [dict(ws=self.workspace, tws=self.topk_workspace, indeg=self._indeg2[0],
                                              idx=self.idx_kv, ent=self.entropy, enth=self.entropy_per_head)]
        mk = torch.empty_like
        while len(chains) < n:
            indeg = self._indeg2[1] if len(chains) == 1 else mk(self._indeg2[0])
            chains.append(dict(ws=mk(self.workspace), tws=mk(self.topk_workspace), indeg=indeg, idx=mk(chains[0]["idx"]),
                               ent=mk(chains[0]["ent"]), enth=mk(chains[0]["enth"])))
        return chains

    def sweep_chains(self, layers, other_streams, slots=None, fused: bool = True) -> None:
        """All layers of a prefill as 1 + len(other_streams) chains: layer l runs on chain l mod n -- chain 0 is the
        current stream -- as the two halves of a fused layer step (score; select + gather) with the chain's own
        buffers and the centrality update between them (`fused=False`: the four entry points one by one).  Layers
        are independent except for that recurrence, C <- lambda C + D/w, which events keep in layer order, so the
        results are those of layer() in a loop, bit for bit.  The update sits in the MIDDLE of a layer's kernels on
        purpose: with the cross-stream wait at the end of a layer a captured graph ran the chains one after the
        other (3.2 ms against 1.4 ms for the 32K configuration).  One chain's short
        kernels run under another chain's scoring kernels.  Afterwards indeg / idx_kv / entropy / entropy_per_head
        are the LAST layer's.  Ends with all streams joined on the current one."""
        a = torch.cuda.current_stream()
        streams = [a] + list(other_streams)
        n = len(streams)
        chain = self._chains(n)
        start = torch.cuda.Event()
        start.record(a)
        for st in streams[1:]:
            st.wait_event(start)
        acc_done = None
        last = 0
        for l, (q_win, k, v) in enumerate(layers):
            c, st = chain[l % n], streams[l % n]
            slot = l if slots is None else slots[l]
            if fused:
                B.structkv_layer_begin(self.shape, q_win, k, v, self.cu, self.k_per_seq, self.keep_tail, c["indeg"],
                                       None, self.lam, 1.0 / self.w, c["ent"], c["enth"], c["idx"], self.k_cache[slot],
                                       self.v_cache[slot], c["ws"], st)
            else:
                B.structkv_score_layer(self.shape, q_win, k, self.cu, c["indeg"], c["ent"], c["enth"], c["ws"], st)
            if acc_done is not None and n > 1:
                st.wait_event(acc_done)
            B.structkv_accumulate_centrality(self.centrality, c["indeg"], self.lam, 1.0 / self.w, st)
            acc_done = torch.cuda.Event()
            acc_done.record(st)
            if fused:
                B.structkv_layer_finish(self.shape, k, v, self.cu, self.k_per_seq, self.keep_tail, c["indeg"], c["idx"],
                                        self.k_cache[slot], self.v_cache[slot], c["ws"], st)
            else:
                B.structkv_select_topk(c["indeg"], self.cu, self.k_per_seq, self.keep_tail, c["idx"], c["tws"], st)
                B.structkv_gather_kv(k, v, self.k_cache[slot], self.v_cache[slot], self.cu, self.rows_per_seq,
                                     c["idx"], st)
            last = l % n
        for st in streams[1:]:
            done = torch.cuda.Event()
            done.record(st)
            a.wait_event(done)
        c = chain[last]
        self.indeg, self.idx_kv, self.entropy, self.entropy_per_head = c["indeg"], c["idx"], c["ent"], c["enth"]

    def sweep_two_chains(self, layers, stream_b, slots=None) -> None:
        """sweep_chains with two chains: even layers on the current stream, odd layers on `stream_b`."""
        self.sweep_chains(layers, [stream_b], slots)

    def sweep_overlapped(self, layers, side_stream, slots=None) -> None:
        """All layers of a prefill: the scoring chain (score -> accumulate) of layer l+1 runs on the current
        stream while selection and gather of layer l run on `side_stream`.  Same calls and same results as
        calling layer() in a loop; only the streams differ.  `layers` yields (q_win, k, v); per-layer
        outputs go to cache slot slots[l] (default l).  Ends with both streams joined on the current one.
        """
        main = torch.cuda.current_stream()
        scored = []      # events: layer l's scores are complete
        selected = []    # events: layer l's selection has finished reading the score vector
        for l, (q_win, k, v) in enumerate(layers):
            self.indeg = self._indeg2[l & 1]
            if l >= 2:
                main.wait_event(selected[l - 2])          # the score vector about to be overwritten is free
            self.score_accumulate(q_win, k, main)
            ev = torch.cuda.Event()
            ev.record(main)
            scored.append(ev)
            side_stream.wait_event(ev)
            B.structkv_select_topk(self.indeg, self.cu, self.k_per_seq, self.keep_tail, self.idx_kv,
                                   self.topk_workspace, side_stream)
            ev2 = torch.cuda.Event()
            ev2.record(side_stream)
            selected.append(ev2)
            self.gather(k, v, l if slots is None else slots[l], side_stream)
        done = torch.cuda.Event()
        done.record(side_stream)
        main.wait_event(done)
