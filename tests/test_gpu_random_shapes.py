"""Seeded random shapes against the fp64 oracle: head dimension, head counts, group size, block size K,
batch, page size, paging layout, ragged lengths (empty sequences included), split setting and view are
all drawn per case, so that combinations nobody wrote down by hand get run too (compute-wave counts
1..8, ragged last tiles, in-block tiles shorter than 32, the three merge forms, the balanced partition).
Then whole decode steps on random shapes: both attention views, the greedy consensus and the commit,
with tokens, lengths and pool bytes bit-exact; the AR prefill and the temperature > 0 consensus on random
shapes.  Same bars as every other parity test.
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


@pytest.mark.parametrize("case_id", range(12))
def test_prefill_on_a_random_shape(case_id):
    """AR prefill (Section 3.1): random head shapes, ragged cache lengths and ragged new-token counts."""
    from test_gpu_prefill import Case, _check, _new_tokens
    rng = np.random.default_rng(7500 + case_id)
    d = int(rng.choice([64, 128]))
    hkv = int(rng.integers(1, 4))
    g = int(rng.integers(1, 9))           # 32 new tokens x g query heads per work item: every wave count 1..8
    batch = int(rng.integers(1, 5))
    page = int(rng.choice([16, 32, 64]))
    hi = int(rng.choice([0, 50, 300]))
    T = int(rng.choice([1, 31, 33, 70, 150]))
    lens = rng.integers(0, hi + 1, size=batch).astype(np.int32)
    new_lens = rng.integers(0, T + 1, size=batch).astype(np.int32)
    new_lens[int(rng.integers(0, batch))] = T
    paging = str(rng.choice(["contiguous", "shuffled", "scattered"]))
    w = Workload(name="rnd_pf", seed=7500 + case_id, batch=batch, num_q_heads=g * hkv, num_kv_heads=hkv, head_dim=d,
                 block_k=8, context=hi, page_size=page, paging=paging, steps=(T + 7) // 8 + 1)
    cache = make_cache(w, seq_lens=lens)
    q, kn, vn = _new_tokens(w, T, 9700 + case_id)
    ref_k, ref_v, ref_l = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    want, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn, new_lens, ref_k, ref_v, cache["page_table"], ref_l)
    case = Case(w, cache, max_seq_len=min(int(lens.max()) + T, cache["page_table"].shape[1] * page))
    got = case.prefill(q, kn, vn, new_lens)
    _check(got, want, new_lens)
    k, v, l = case.state()
    np.testing.assert_array_equal(l, ref_l)
    np.testing.assert_array_equal(k, ref_k)
    np.testing.assert_array_equal(v, ref_v)
    assert case.step.device_error() == 0
    case.step.close()


@pytest.mark.parametrize("case_id", range(8))
def test_sampling_consensus_on_a_random_shape(case_id):
    """Temperature > 0 consensus + commit on random shapes; cases whose decisions sit within fp32 rounding of
    flipping are replaced by the next seed (the oracle reports the margins)."""
    from test_gpu_sampling import _clear_case, _run, _same
    rng = np.random.default_rng(7700 + case_id)
    d = int(rng.choice([64, 128]))
    hkv = int(rng.integers(1, 4))
    kblk = int(rng.integers(1, 17))
    batch = int(rng.integers(1, 7))
    page = int(rng.choice([16, 32]))
    vocab = int(rng.choice([97, 1000, 8193, 20011]))
    temperature = float(rng.choice([0.6, 1.0, 1.4]))
    divergence = float(rng.choice([0.2, 0.5, 1.0]))
    lens = rng.integers(0, 120, size=batch).astype(np.int32)
    w = Workload(name="rnd_smp", seed=7700 + case_id, batch=batch, num_q_heads=2 * hkv, num_kv_heads=hkv, head_dim=d,
                 block_k=kblk, context=120, page_size=page, paging="shuffled", vocab=vocab, steps=1)
    c, _ = _clear_case(w, 9900 + 50 * case_id, temperature=temperature, divergence=divergence)
    cache = make_cache(w, seq_lens=lens)
    blk = make_block(w, 9800 + case_id)
    rk, rv, rl = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    want = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                            c["gumbel"], temperature, blk["k_blk"], blk["v_blk"], rk, rv,
                                            cache["page_table"], rl)
    got = _run(w, cache, c, blk)
    _same(got, want)
    assert got["err"] == 0
    np.testing.assert_array_equal(got["seq_lens"], rl)
    np.testing.assert_array_equal(got["k_pool"], rk)
    np.testing.assert_array_equal(got["v_pool"], rv)
