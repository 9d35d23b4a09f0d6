"""Seeded random shapes against the fp64 oracle: head dimension, head counts, group size, block size K,
batch, page size, paging layout, ragged lengths (empty sequences included), split setting and view are
all drawn per case, so that combinations nobody wrote down by hand get run too (compute-wave counts
1..8, ragged last tiles, in-block tiles shorter than 32, the three merge forms, the balanced partition).
Then whole decode steps on random shapes: both attention views, the greedy consensus and the commit,
with tokens, lengths and pool bytes bit-exact.  Same bars as every other parity test.
"""
import numpy as np
import pytest

import oracle
from orthrus_inputs import Workload, make_block, make_cache, make_consensus_case

from test_gpu_parity import (AR, DIFF, GpuCase, _check_attn, _gathered_equal, _oracle_attn, _run_consensus,
                             _same_consensus)

pytestmark = pytest.mark.gpu


def _draw_shape(rng, max_len_choices):
    d = int(rng.choice([64, 128]))
    hkv = int(rng.integers(1, 5))
    kblk = int(rng.integers(1, 33))
    g = int(rng.integers(1, max(1, min(8, 256 // kblk)) + 1))  # at most 256 query rows per KV head
    batch = int(rng.integers(1, 9))
    page = int(rng.choice([16, 32, 64]))
    hi = int(rng.choice(max_len_choices))
    lens = rng.integers(0, hi + 1, size=batch).astype(np.int32)
    if rng.random() < 0.3:
        lens[int(rng.integers(0, batch))] = 0
    paging = str(rng.choice(["contiguous", "shuffled", "scattered"]))
    return d, hkv, g, kblk, batch, page, hi, lens, paging


@pytest.mark.parametrize("case_id", range(32))
def test_attention_on_a_random_shape(case_id):
    rng = np.random.default_rng(7100 + case_id)
    d, hkv, g, kblk, batch, page, hi, lens, paging = _draw_shape(rng, [60, 300, 1500, 3000])
    splits = int(rng.choice([0, 1, 2, 5, 12, 20, -1, -1]))
    view = int(rng.integers(0, 2))
    what = "case %d: d=%d hkv=%d g=%d K=%d B=%d P=%d lens=%s splits=%d %s view=%d" % (
        case_id, d, hkv, g, kblk, batch, page, lens.tolist(), splits, paging, view)
    w = Workload(name="rnd", seed=7100 + case_id, batch=batch, num_q_heads=g * hkv, num_kv_heads=hkv, head_dim=d,
                 block_k=kblk, context=hi, page_size=page, paging=paging)
    cache = make_cache(w, seq_lens=lens)
    blk = make_block(w, 9100 + case_id)
    # a host bound somewhere between the longest sequence and what the page table maps
    mapped = cache["page_table"].shape[1] * page
    bound = int(rng.integers(max(int(lens.max()), 1), max(min(hi, mapped), int(lens.max()), 1) + 1))
    case = GpuCase(w, cache, num_splits=splits, max_seq_len=bound)
    got, lse = case.attn(view, blk)
    want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
    _check_attn(got, want, what)
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3, err_msg=what)
    assert case.step.device_error() == 0, what
    again, _ = case.attn(view, blk)
    np.testing.assert_array_equal(again, got, err_msg=what)  # deterministic
    case.step.close()


@pytest.mark.parametrize("case_id", range(10))
def test_decode_steps_on_a_random_shape(case_id):
    rng = np.random.default_rng(7300 + case_id)
    d, hkv, g, kblk, batch, page, hi, lens, paging = _draw_shape(rng, [40, 200, 900])
    vocab = int(rng.choice([97, 1000, 8193, 30011]))
    steps = 3
    what = "case %d: d=%d hkv=%d g=%d K=%d B=%d P=%d lens=%s vocab=%d %s" % (
        case_id, d, hkv, g, kblk, batch, page, lens.tolist(), vocab, paging)
    w = Workload(name="rnd_step", seed=7300 + case_id, batch=batch, num_q_heads=g * hkv, num_kv_heads=hkv, head_dim=d,
                 block_k=kblk, context=hi, page_size=page, paging=paging, vocab=vocab, accept="uniform", steps=steps)
    cache = make_cache(w, seq_lens=lens)
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in cache.items()}
    case = GpuCase(w, cache, vocab=vocab, max_seq_len=min(w.capacity_tokens(), cache["page_table"].shape[1] * page))
    for step in range(steps):
        blk_d, blk_a = make_block(w, 9300 + 20 * case_id + 2 * step), make_block(w, 9301 + 20 * case_id + 2 * step)
        for view, blk in ((DIFF, blk_d), (AR, blk_a)):
            got = case.attn(view, blk, want_lse=False)
            _check_attn(got, _oracle_attn(view, w, blk, ref), "%s step %d view %d" % (what, step, view))
        cc = make_consensus_case(w, seed=9500 + 10 * case_id + step)
        got = _run_consensus(case, cc["ar_logits"], cc["draft_tokens"], blk_a)
        want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"], blk_a["k_blk"], blk_a["v_blk"],
                                       ref["k_pool"], ref["v_pool"], ref["page_table"], ref["seq_lens"])
        _same_consensus(got, want)
        _gathered_equal(case, ref)  # the oracle appended into `ref` in place: lengths and every pool byte agree
    assert case.step.device_error() == 0, what
    case.step.close()
