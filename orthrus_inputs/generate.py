"""Seeded generators for the dual-view decode step's inputs (numpy, host memory).

Everything here is data preparation: random draws, rounding fp32 values to bf16 bit
patterns, page-table construction and *planting* consensus cases.  Nothing here evaluates
attention, a softmax, an argmax or the accept rule: a planted case is built so that the
answer is known by construction (a chosen token gets a logit above every other entry of
its row), never by computing it.

Layouts (all C-contiguous):
  q                      [B, K, H_q, d]        bf16 bits (uint16)
  k_blk, v_blk           [B, K, H_kv, d]       bf16 bits
  k_pool, v_pool         [pages, H_kv, P, d]   bf16 bits  (one layer)
  page_table             [B, max_pages]        int32, -1 = not mapped
  seq_lens               [B]                   int32, cached tokens before the anchor
  ar_logits              [B, K, V]             float32
  draft_tokens           [B, K]                int32
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .configs import Workload


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, scale: float = 1.0) -> np.ndarray:
    """N(0, scale^2) rounded to bf16 bits; drawn in slabs to bound peak host memory."""
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(-1)
    step = 1 << 24
    for s in range(0, flat.size, step):
        e = min(flat.size, s + step)
        x = rng.standard_normal(e - s, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        flat[s:e] = f32_to_bf16_bits(x)
    return out


def draw_seq_lens(w: Workload, rng: np.random.Generator) -> np.ndarray:
    if w.context_range is not None:
        lo, hi = w.context_range
        return rng.integers(lo, hi + 1, size=w.batch).astype(np.int32)
    return np.full(w.batch, w.context, dtype=np.int32)


def make_cache(w: Workload, seed: Optional[int] = None, value_scale: float = 1.0,
               seq_lens: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Paged K/V pools, page table and lengths for one layer.

    Every pool entry, mapped or not, holds random data, so a kernel that reads past
    seq_lens[b] or through an unmapped page produces visibly wrong output.
    """
    rng = np.random.default_rng(w.seed if seed is None else seed)
    P = w.page_size
    if seq_lens is None:
        seq_lens = draw_seq_lens(w, rng)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    cap = seq_lens.astype(np.int64) + w.steps * w.block_k
    pages_per_seq = (cap + P - 1) // P
    max_pages = int(pages_per_seq.max()) if w.batch else 0
    mapped = int(pages_per_seq.sum())
    if w.paging == "scattered":
        num_pages = mapped + max(1, mapped // 10)
    else:
        num_pages = mapped
    num_pages = max(num_pages, 1)
    if w.paging == "contiguous":
        order = np.arange(num_pages, dtype=np.int64)
    else:
        order = rng.permutation(num_pages)
    page_table = np.full((w.batch, max(max_pages, 1)), -1, dtype=np.int32)
    at = 0
    for b in range(w.batch):
        n = int(pages_per_seq[b])
        page_table[b, :n] = order[at:at + n]
        at += n
    shape = (num_pages, w.num_kv_heads, P, w.head_dim)
    k_pool = _normal_bf16(rng, shape, value_scale)
    v_pool = _normal_bf16(rng, shape, value_scale)
    return dict(k_pool=k_pool, v_pool=v_pool, page_table=page_table, seq_lens=seq_lens.copy(),
                num_pages=num_pages, max_pages_per_seq=page_table.shape[1])


def make_block(w: Workload, seed: int, value_scale: float = 1.0) -> Dict[str, np.ndarray]:
    """Queries and in-block K/V of one K-position block for one view."""
    rng = np.random.default_rng(seed)
    q = _normal_bf16(rng, (w.batch, w.block_k, w.num_q_heads, w.head_dim), value_scale)
    k_blk = _normal_bf16(rng, (w.batch, w.block_k, w.num_kv_heads, w.head_dim), value_scale)
    v_blk = _normal_bf16(rng, (w.batch, w.block_k, w.num_kv_heads, w.head_dim), value_scale)
    return dict(q=q, k_blk=k_blk, v_blk=v_blk)


def draw_accept_lengths(w: Workload, rng: np.random.Generator) -> np.ndarray:
    """Planted accepted-draft counts n_acc in [0, K]."""
    K = w.block_k
    if w.accept == "uniform":
        return rng.integers(0, K + 1, size=w.batch).astype(np.int32)
    g = rng.geometric(w.accept_p, size=w.batch)          # support {1, 2, ...}
    return np.minimum(K, g - 1).astype(np.int32)


def make_consensus_case(w: Workload, seed: int, vocab: Optional[int] = None,
                        n_acc: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """AR logits with a planted per-row maximum and drafts with a planted accepted prefix.

    Row (b, k) of ar_logits is N(0,1) noise except entry top[b, k], which is set to
    8 + U[0,1): above any N(0,1) draw that fits in the row (the chance of a draw above
    8 is ~6e-16 per entry), so top[b, k] is the row's unique largest entry by construction.
    Drafts copy top for k < n_acc[b], differ from it at k = n_acc[b] (when n_acc[b] < K) and
    are uniform random after that (so later positions may match by chance, which the accept
    rule must ignore).
    """
    rng = np.random.default_rng(seed)
    V = int(vocab if vocab is not None else w.vocab)
    B, K = w.batch, w.block_k
    logits = np.empty((B, K, V), dtype=np.float32)
    flat = logits.reshape(B * K, V)
    for r in range(B * K):
        flat[r] = rng.standard_normal(V, dtype=np.float32)
    top = rng.integers(0, V, size=(B, K)).astype(np.int32)
    bump = (8.0 + rng.random((B, K))).astype(np.float32)
    bi, ki = np.meshgrid(np.arange(B), np.arange(K), indexing="ij")
    logits[bi, ki, top] = bump
    if n_acc is None:
        n_acc = draw_accept_lengths(w, rng)
    n_acc = np.asarray(n_acc, dtype=np.int32)
    draft = rng.integers(0, V, size=(B, K)).astype(np.int32)
    for b in range(B):
        n = int(n_acc[b])
        draft[b, :n] = top[b, :n]
        if n < K:
            # any token other than the planted maximum
            draft[b, n] = (top[b, n] + 1 + rng.integers(0, max(V - 1, 1))) % V if V > 1 else top[b, n]
    return dict(ar_logits=logits, draft_tokens=draft, planted_top=top, planted_n_acc=n_acc)


def make_sampling_case(w: Workload, seed: int, vocab: Optional[int] = None, temperature: float = 1.0,
                       divergence: float = 0.5, logit_scale: float = 2.0) -> Dict[str, np.ndarray]:
    """Inputs of the temperature > 0 consensus: target and draft logits, drafts, and the random numbers.

    ar_logits ~ logit_scale * N(0,1); diff_logits = ar_logits + divergence * N(0,1) (a draft
    distribution close to, but not equal to, the target); each draft token is drawn from
    softmax(diff_logits / temperature) by perturbing the scaled logits with Gumbel noise and taking the
    largest (the way a sampler outside the path would produce it); accept_u ~ U[0,1) and one row of
    standard Gumbel noise per sequence are the random numbers the consensus step consumes.
    """
    rng = np.random.default_rng(seed)
    V = int(vocab if vocab is not None else w.vocab)
    B, K = w.batch, w.block_k
    ar = np.empty((B, K, V), dtype=np.float32)
    df = np.empty((B, K, V), dtype=np.float32)
    draft = np.empty((B, K), dtype=np.int32)
    for b in range(B):
        for k in range(K):
            a = rng.standard_normal(V, dtype=np.float32) * np.float32(logit_scale)
            ar[b, k] = a
            df[b, k] = a + rng.standard_normal(V, dtype=np.float32) * np.float32(divergence)
            noise = rng.gumbel(size=V)
            draft[b, k] = int(np.argmax(df[b, k].astype(np.float64) / temperature + noise))
    accept_u = rng.random((B, K), dtype=np.float32)
    gumbel = rng.gumbel(size=(B, V)).astype(np.float32)
    return dict(ar_logits=ar, diff_logits=df, draft_tokens=draft, accept_u=accept_u, gumbel=gumbel,
                temperature=float(temperature))


def make_step_inputs(w: Workload, step: int = 0, value_scale: float = 1.0,
                     with_cache: bool = True) -> Dict[str, np.ndarray]:
    """All inputs of one decode step: cache (step 0 only), both views' blocks, consensus case."""
    out: Dict[str, np.ndarray] = {}
    if with_cache:
        out.update(make_cache(w, value_scale=value_scale))
    base = w.seed * 1000 + step * 10
    d = make_block(w, base + 1, value_scale)
    a = make_block(w, base + 2, value_scale)
    out.update(q_diff=d["q"], k_blk_diff=d["k_blk"], v_blk_diff=d["v_blk"],
               q_ar=a["q"], k_blk_ar=a["k_blk"], v_blk_ar=a["v_blk"])
    if w.vocab:
        out.update(make_consensus_case(w, base + 3))
    return out
