"""Workload shapes for the dual-view decode step (one attention layer).

The shapes follow the decoding setting of the paper (Section 4.1: Qwen3-class GQA
models, block size K up to 32; Section 4.4, long-context stability: contexts up to ~40K tokens) and stand in for
its benchmark workloads; every tensor is synthetic and seeded.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_k: int
    # cached context: either one fixed length or a (lo, hi) uniform range per sequence
    context: int = 0
    context_range: Optional[Tuple[int, int]] = None
    page_size: int = 16
    # "contiguous": identity page table; "shuffled": each sequence's pages permuted inside a
    # pool that holds exactly the mapped pages; "scattered": pages drawn at random from a
    # shared pool with ~10 % unmapped pages left over
    paging: str = "shuffled"
    vocab: int = 0                      # 0: the workload names no consensus step
    accept: str = "geometric"           # "uniform" (0..K) or "geometric" (p below, capped at K)
    accept_p: float = 0.3
    steps: int = 1                      # looped decode steps (cache grows by the committed counts)
    num_splits: int = 0                 # 0 = library picks; -1 = balanced partition (ragged batches)
    seed: int = 0
    description: str = ""

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def sm_scale(self) -> float:
        return 1.0 / float(self.head_dim) ** 0.5

    def max_context(self) -> int:
        return self.context_range[1] if self.context_range else self.context

    def capacity_tokens(self) -> int:
        """Token capacity mapped per sequence: context plus room for every looped step."""
        return self.max_context() + self.steps * self.block_k

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "tiny": Workload(
        name="tiny", batch=1, num_q_heads=4, num_kv_heads=2, head_dim=64, block_k=4,
        context=128, paging="contiguous", vocab=512, accept="uniform", seed=1000,
        description="batch 1, 4/2 heads, d=64, context 128, K=4, contiguous cache, vocab 512"),
    "layer8b": Workload(
        name="layer8b", batch=1, num_q_heads=32, num_kv_heads=8, head_dim=128, block_k=16,
        context=4096, paging="shuffled", vocab=128256, accept="geometric", seed=1001,
        description="batch 1, 32/8 heads, d=128, context 4096, K=16, shuffled 16-token pages, vocab 128256"),
    "mixed": Workload(
        name="mixed", batch=16, num_q_heads=28, num_kv_heads=4, head_dim=128, block_k=32,
        context_range=(512, 8192), paging="scattered", vocab=0, seed=1002, num_splits=-1,
        description="batch 16, 28/4 heads, d=128, context U[512,8192], K=32, pages scattered in a shared pool"),
    "long": Workload(
        name="long", batch=4, num_q_heads=32, num_kv_heads=8, head_dim=128, block_k=16,
        context=32768, paging="shuffled", vocab=128256, accept="geometric", seed=1003,
        description="batch 4, 32/8 heads, d=128, context 32768, K=16, 16-token pages, vocab 128256"),
    "stress": Workload(
        name="stress", batch=64, num_q_heads=32, num_kv_heads=8, head_dim=128, block_k=16,
        context=2048, paging="shuffled", vocab=151936, accept="geometric", steps=32, seed=1004,
        description="batch 64, 32/8 heads, d=128, context 2048, K=16, vocab 151936, 32 looped steps"),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]
