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
                 pool_strides=None, min_seq_len_bound=None):
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2605_12825_amd needs a HIP device; there is no CPU path")
        self.device = torch.device("cuda", device)
        kw = {}
        if pool_strides is not None:
            kw = dict(pool_stride_layer=pool_strides[0], pool_stride_page=pool_strides[1],
                      pool_stride_head=pool_strides[2], pool_stride_tok=pool_strides[3])
        self.params = B.make_params(batch=batch, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                                    head_dim=head_dim, block_k=block_k, page_size=page_size,
                                    max_pages_per_seq=max_pages_per_seq, max_seq_len=max_seq_len,
                                    num_pages=num_pages, num_splits=num_splits, num_layers=num_layers,
                                    vocab=vocab, sm_scale=sm_scale, **kw)
        self.ctx = B.orthrus_create(device)
        self.num_splits = B.orthrus_attn_num_splits(self.params)
        # workspace for every host bound on the lengths the caller may set later (see set_max_seq_len)
        n = B.orthrus_attn_workspace_bytes(self.params)
        lo = max_seq_len if min_seq_len_bound is None else min_seq_len_bound
        for bound in range(lo, max_seq_len, max(block_k, 1)):
            self.params.max_seq_len = bound
            n = max(n, B.orthrus_attn_workspace_bytes(self.params))
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
        self.num_splits = B.orthrus_attn_num_splits(self.params)

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

    def attn_timing(self, enable: bool) -> None:
        """Attach HIP events to the attention kernels of the following attn() calls (or stop doing so)."""
        B.orthrus_attn_timing(self.ctx, enable)

    def attn_timing_read(self):
        """(split us, launches, combine us, launches) summed over the timed launches since the last read."""
        return B.orthrus_attn_timing_read(self.ctx)

    def device_error(self, stream=None) -> int:
        return B.orthrus_last_device_error(self.ctx, stream)
