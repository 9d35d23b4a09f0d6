"""Convenience holder for one decode-step configuration: context, params and workspaces.

Pure plumbing around the C ABI (torch provides device memory and the current stream); every
computation happens inside liborthrus.so.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


def to_device_bits(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """Uploads a numpy array; uint16 bf16 bit patterns travel as int16 (same bits)."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def bits_to_numpy(t: torch.Tensor) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


class DecodeStep:
    """Owns an orthrus context plus the attention / consensus workspaces for fixed shapes."""

    def __init__(self, *, batch, num_q_heads, num_kv_heads, head_dim, block_k, page_size, max_pages_per_seq,
                 max_seq_len, num_pages, vocab=0, num_layers=1, num_splits=0, sm_scale=None, device=0,
                 pool_strides=None, min_seq_len_bound=None, block_strides=None):
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2605_12825_amd needs a HIP device; there is no CPU path")
        self.device = torch.device("cuda", device)
        kw = {}
        if pool_strides is not None:
            kw = dict(pool_stride_layer=pool_strides[0], pool_stride_page=pool_strides[1],
                      pool_stride_head=pool_strides[2], pool_stride_tok=pool_strides[3])
        if block_strides is not None:   # (q_stride_row, q_stride_head, blk_stride_row, blk_stride_head, blk_stride_layer)
            kw.update(q_stride_row=block_strides[0], q_stride_head=block_strides[1], blk_stride_row=block_strides[2],
                      blk_stride_head=block_strides[3], blk_stride_layer=block_strides[4])
        self.params = B.make_params(batch=batch, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                                    head_dim=head_dim, block_k=block_k, page_size=page_size,
                                    max_pages_per_seq=max_pages_per_seq, max_seq_len=max_seq_len,
                                    num_pages=num_pages, num_splits=num_splits, num_layers=num_layers,
                                    vocab=vocab, sm_scale=sm_scale, **kw)
        self.ctx = B.orthrus_create(device)
        # plans and sizes for the device the context lives on
        self.num_splits = B.orthrus_attn_num_splits_on(self.ctx, self.params)
        # workspace for every host bound on the lengths the caller may set later (see set_max_seq_len)
        n = B.orthrus_attn_workspace_bytes_on(self.ctx, self.params)
        lo = max_seq_len if min_seq_len_bound is None else min_seq_len_bound
        for bound in range(lo, max_seq_len, max(block_k, 1)):
            self.params.max_seq_len = bound
            n = max(n, B.orthrus_attn_workspace_bytes_on(self.ctx, self.params))
        self.params.max_seq_len = max_seq_len
        self.attn_ws = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        self.cons_ws = None
        if vocab > 0:
            n = max(B.orthrus_consensus_workspace_bytes(self.params), B.orthrus_sampling_workspace_bytes(self.params))
            self.cons_ws = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)

    def set_max_seq_len(self, bound: int) -> None:
        """Tightens the host upper bound on the sequence lengths (it sizes the attention grid).

        `bound` must lie between the `min_seq_len_bound` and the `max_seq_len` given at construction,
        and must not be below any current sequence length.
        """
        self.params.max_seq_len = int(bound)
        self.num_splits = B.orthrus_attn_num_splits_on(self.ctx, self.params)
        # the constructor sized the workspace for the bounds min_seq_len_bound + i * block_k; any other bound
        # whose plan needs more gets a larger one here (rare, and never inside a captured sequence)
        n = B.orthrus_attn_workspace_bytes_on(self.ctx, self.params)
        if n > self.attn_ws.numel():
            self.attn_ws = torch.empty(n, dtype=torch.uint8, device=self.device)

    def close(self):
        if self.ctx:
            torch.cuda.synchronize(self.device)
            B.orthrus_destroy(self.ctx)
            self.ctx = None

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    def attn(self, view, q, k_blk, v_blk, k_pool, v_pool, page_table, seq_lens, out, lse=None, stream=None):
        return B.orthrus_dual_view_attn(self.ctx, self.params, view, q, k_blk, v_blk, k_pool, v_pool, page_table,
                                        seq_lens, out, lse, self.attn_ws, stream)

    def consensus_commit(self, ar_logits, draft_tokens, k_blk_ar, v_blk_ar, k_pool, v_pool, page_table, seq_lens,
                         accept_len, num_committed, out_tokens, next_anchor, stream=None):
        return B.orthrus_consensus_commit(self.ctx, self.params, ar_logits, draft_tokens, k_blk_ar, v_blk_ar,
                                          k_pool, v_pool, page_table, seq_lens, accept_len, num_committed,
                                          out_tokens, next_anchor, self.cons_ws, stream)

    def sampling_consensus_commit(self, temperature, ar_logits, diff_logits, draft_tokens, accept_u, gumbel,
                                  k_blk_ar, v_blk_ar, k_pool, v_pool, page_table, seq_lens, accept_len,
                                  num_committed, out_tokens, next_anchor, stream=None):
        return B.orthrus_sampling_consensus_commit(self.ctx, self.params, temperature, ar_logits, diff_logits,
                                                   draft_tokens, accept_u, gumbel, k_blk_ar, v_blk_ar, k_pool, v_pool,
                                                   page_table, seq_lens, accept_len, num_committed, out_tokens,
                                                   next_anchor, self.cons_ws, stream)

    def prefill(self, max_new_tokens, q, k_new, v_new, new_lens, k_pool, v_pool, page_table, seq_lens, out,
                stream=None):
        """AR-view prefill attention of one layer (appends the new K/V rows, causal attention over the cache)."""
        need = B.orthrus_prefill_workspace_bytes(self.params, max_new_tokens)
        if getattr(self, "prefill_ws", None) is None or self.prefill_ws.numel() < need:
            self.prefill_ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        return B.orthrus_prefill_attn(self.ctx, self.params, max_new_tokens, q, k_new, v_new, new_lens, k_pool,
                                      v_pool, page_table, seq_lens, out, self.prefill_ws, stream)

    def attn_timing(self, enable: bool) -> None:
        """Attach HIP events to the attention kernels of the following attn() calls (or stop doing so)."""
        B.orthrus_attn_timing(self.ctx, enable)

    def attn_timing_read(self):
        """(split us, launches, combine us, launches) summed over the timed launches since the last read."""
        return B.orthrus_attn_timing_read(self.ctx)

    def attn_timing_samples(self, capacity: int = 4096):
        """[(split kernel us, combine kernel us)] per timed call since the last read, in launch order."""
        return B.orthrus_attn_timing_samples(self.ctx, capacity)

    def kv_stream_probe(self, k_pool, v_pool, page_table, seq_lens, stream=None) -> None:
        """The attention call's K/V stream over this cache with idle compute waves (measurement)."""
        B.orthrus_kv_stream_probe(self.ctx, self.params, k_pool, v_pool, page_table, seq_lens, stream)

    def device_error(self, stream=None) -> int:
        return B.orthrus_last_device_error(self.ctx, stream)


class DecodeStack:
    """One decode cycle over a stack of layers, eagerly or as a replayed HIP graph.

    The cycle is the paper's: the diffusion view's pass through every layer, the AR view's
    verification pass through every layer, then the consensus and the commit of the accepted
    tokens' K/V into every layer's cache (Section 3.2-3.3, Fig. 2(b)).  Only the attention of each
    layer is computed here; whatever produces a layer's queries and block K/V writes them into
    this object's static buffers (`q_diff[l]`, `k_blk_diff[l]`, ... `ar_logits`, `draft_tokens`).
    Argument marshalling only: the loop below calls the C ABI once per layer and view.
    """

    def __init__(self, *, num_layers, batch, num_q_heads, num_kv_heads, head_dim, block_k, page_size,
                 k_pool, v_pool, page_table, seq_lens, max_seq_len, vocab, num_splits=0, temperature=0.0,
                 diffusion_passes=1, device=0):
        if k_pool.dim() != 5 or k_pool.shape[0] != num_layers or not k_pool.is_contiguous():
            raise ValueError("pools must be contiguous [layers, pages, H_kv, P, d]")
        L, pages, H, P, d = k_pool.shape
        self.num_layers, self.temperature = num_layers, float(temperature)
        # forward passes of the diffusion view per cycle: 1 is the paper's single-step projection, 2 the
        # multi-step denoising variant of its ablation (Section 5, Table 3); the passes run back to back
        # over the same buffers (whatever refines the block between them writes q_diff / k_blk_diff / v_blk_diff)
        self.diffusion_passes = int(diffusion_passes)
        if self.diffusion_passes < 1:
            raise ValueError("diffusion_passes must be >= 1")
        self.k_pool, self.v_pool, self.page_table, self.seq_lens = k_pool, v_pool, page_table, seq_lens
        self.step = DecodeStep(batch=batch, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads, head_dim=head_dim,
                               block_k=block_k, page_size=page_size, max_pages_per_seq=page_table.shape[1],
                               max_seq_len=max_seq_len, num_pages=pages, vocab=vocab, num_layers=num_layers,
                               num_splits=num_splits, device=device,
                               pool_strides=(pages * H * P * d, H * P * d, P * d, d))
        dev = self.step.device
        blk = (num_layers, batch, block_k, num_kv_heads, head_dim)
        qs = (num_layers, batch, block_k, num_q_heads, head_dim)
        i16 = dict(dtype=torch.int16, device=dev)
        self.q_diff, self.q_ar = torch.zeros(qs, **i16), torch.zeros(qs, **i16)
        self.k_blk_diff, self.v_blk_diff = torch.zeros(blk, **i16), torch.zeros(blk, **i16)
        self.k_blk_ar, self.v_blk_ar = torch.zeros(blk, **i16), torch.zeros(blk, **i16)
        self.out_diff, self.out_ar = torch.zeros(qs, **i16), torch.zeros(qs, **i16)
        self.ar_logits = torch.zeros((batch, block_k, vocab), dtype=torch.float32, device=dev)
        self.draft_tokens = torch.zeros((batch, block_k), dtype=torch.int32, device=dev)
        if self.temperature > 0:
            self.diff_logits = torch.zeros_like(self.ar_logits)
            self.accept_u = torch.zeros((batch, block_k), dtype=torch.float32, device=dev)
            self.gumbel = torch.zeros((batch, vocab), dtype=torch.float32, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        self.accept_len, self.num_committed, self.next_anchor = (torch.zeros((batch,), **i32) for _ in range(3))
        self.out_tokens = torch.zeros((batch, block_k), **i32)
        self.graph = None
        self.graph_stream = None

    def cycle(self, stream=None) -> None:
        """Issues the whole cycle on `stream` (default: the current stream)."""
        s = self.step
        diff = (0, self.q_diff, self.k_blk_diff, self.v_blk_diff, self.out_diff)
        ar = (1, self.q_ar, self.k_blk_ar, self.v_blk_ar, self.out_ar)
        for view, q, kb, vb, out in (diff,) * self.diffusion_passes + (ar,):
            for l in range(self.num_layers):
                s.attn(view, q[l], kb[l], vb[l], self.k_pool[l], self.v_pool[l], self.page_table, self.seq_lens,
                       out[l], None, stream)
        if self.temperature > 0:
            s.sampling_consensus_commit(self.temperature, self.ar_logits, self.diff_logits, self.draft_tokens,
                                        self.accept_u, self.gumbel, self.k_blk_ar, self.v_blk_ar, self.k_pool,
                                        self.v_pool, self.page_table, self.seq_lens, self.accept_len,
                                        self.num_committed, self.out_tokens, self.next_anchor, stream)
        else:
            s.consensus_commit(self.ar_logits, self.draft_tokens, self.k_blk_ar, self.v_blk_ar, self.k_pool,
                               self.v_pool, self.page_table, self.seq_lens, self.accept_len, self.num_committed,
                               self.out_tokens, self.next_anchor, stream)

    def capture(self) -> None:
        """Records one cycle into a HIP graph (on a stream of its own, default priority)."""
        if self.graph is not None:
            raise RuntimeError("already captured")
        torch.cuda.synchronize(self.step.device)
        self.graph_stream = torch.cuda.Stream(device=self.step.device)
        B.orthrus_graph_begin(self.step.ctx, self.graph_stream)
        try:
            self.cycle(self.graph_stream)
        finally:
            self.graph = B.orthrus_graph_end(self.step.ctx, self.graph_stream)

    def replay(self, stream=None) -> None:
        if self.graph is None:
            raise RuntimeError("capture() first")
        B.orthrus_graph_launch(self.graph, self.graph_stream if stream is None else stream)

    def close(self) -> None:
        if self.graph is not None:
            torch.cuda.synchronize(self.step.device)
            B.orthrus_graph_destroy(self.graph)
            self.graph = None
        self.step.close()
