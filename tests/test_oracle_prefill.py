"""Pins for the AR prefill oracle (causal self-attention that builds the cache; Section 3.1 / 2.1).

Each test ties the oracle to something other than itself: the textbook definition written out with numpy on
tiny inputs, closed forms, and the already pinned decode oracle (prefilling n tokens must equal n single-token
AR decode steps, and any chunking of the prompt must give the same result).
"""
import numpy as np
import pytest

import oracle
from orthrus_inputs import Workload, bf16_bits_to_f32, make_cache, f32_to_bf16_bits


def _w(**kw):
    base = dict(name="pf", batch=2, num_q_heads=4, num_kv_heads=2, head_dim=16, block_k=1, context_range=(0, 40),
                page_size=16, paging="shuffled", seed=5, steps=64)
    base.update(kw)
    return Workload(**base)


def _new_tokens(w, T, seed):
    rng = np.random.default_rng(seed)
    mk = lambda h: f32_to_bf16_bits(rng.standard_normal((w.batch, T, h, w.head_dim), dtype=np.float32))
    return mk(w.num_q_heads), mk(w.num_kv_heads), mk(w.num_kv_heads)


def _gather(pool, pt, b, L):
    P = pool.shape[2]
    return np.stack([bf16_bits_to_f32(pool[pt[b, j // P], :, j % P, :]).astype(np.float64) for j in range(L)]) \
        if L else np.zeros((0, pool.shape[1], pool.shape[3]))


def test_prefill_equals_textbook_causal_attention_written_out():
    w = _w()
    cache = make_cache(w)
    T = 9
    q, kn, vn = _new_tokens(w, T, 11)
    new_lens = np.array([9, 4], np.int32)
    L0 = cache["seq_lens"].copy()
    kp, vp, lens = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    out, rc = oracle.prefill_attn(w.sm_scale, q, kn, vn, new_lens, kp, vp, cache["page_table"], lens)
    assert rc == 0
    np.testing.assert_array_equal(lens, L0 + new_lens)
    G = w.num_q_heads // w.num_kv_heads
    for b in range(w.batch):
        n = int(new_lens[b])
        # keys / values: the old cache followed by the new rows (independent of the oracle's paging code)
        K_all = np.concatenate([_gather(cache["k_pool"], cache["page_table"], b, int(L0[b])),
                                bf16_bits_to_f32(kn[b, :n]).astype(np.float64)])
        V_all = np.concatenate([_gather(cache["v_pool"], cache["page_table"], b, int(L0[b])),
                                bf16_bits_to_f32(vn[b, :n]).astype(np.float64)])
        for i in range(n):
            vis = int(L0[b]) + i + 1
            for h in range(w.num_q_heads):
                qv = bf16_bits_to_f32(q[b, i, h]).astype(np.float64)
                s = K_all[:vis, h // G] @ qv * w.sm_scale
                pr = np.exp(s - s.max()); pr /= pr.sum()
                np.testing.assert_allclose(out[b, i, h], pr @ V_all[:vis, h // G], rtol=1e-12, atol=1e-13)
        assert np.isnan(out[b, n:]).all()
        # the cache now holds the new rows bit for bit
        np.testing.assert_array_equal(_gather(kp, cache["page_table"], b, int(lens[b]))[int(L0[b]):],
                                      bf16_bits_to_f32(kn[b, :n]).astype(np.float64))
        np.testing.assert_array_equal(_gather(vp, cache["page_table"], b, int(lens[b]))[int(L0[b]):],
                                      bf16_bits_to_f32(vn[b, :n]).astype(np.float64))


def test_first_token_of_an_empty_cache_returns_its_own_value_row():
    w = _w(batch=1, context=0, context_range=None)
    cache = make_cache(w)
    q, kn, vn = _new_tokens(w, 3, 12)
    out, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn, np.array([3], np.int32), cache["k_pool"], cache["v_pool"],
                                 cache["page_table"], cache["seq_lens"])
    G = w.num_q_heads // w.num_kv_heads
    for h in range(w.num_q_heads):   # softmax over a single key is 1
        np.testing.assert_array_equal(out[0, 0, h], bf16_bits_to_f32(vn[0, 0, h // G]).astype(np.float64))


def test_constant_values_give_that_constant_and_equal_keys_give_the_mean():
    w = _w(batch=1, context=21, context_range=None)
    cache = make_cache(w)
    T = 5
    q, kn, vn = _new_tokens(w, T, 13)
    one = f32_to_bf16_bits(np.array([1.5], np.float32))[0]
    kp, vp = cache["k_pool"].copy(), cache["v_pool"].copy()
    vp[:] = one
    vn_c = np.full_like(vn, one)
    out, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn_c, np.array([T], np.int32), kp, vp, cache["page_table"],
                                 cache["seq_lens"].copy())
    np.testing.assert_allclose(out, 1.5, rtol=0, atol=1e-12)
    # all keys equal -> uniform weights -> row i returns the mean of the first L+i+1 value rows
    kp2, vp2 = cache["k_pool"].copy(), cache["v_pool"].copy()
    kp2[:] = one
    lens = cache["seq_lens"].copy()
    out2, _ = oracle.prefill_attn(w.sm_scale, q, np.full_like(kn, one), vn, np.array([T], np.int32), kp2, vp2,
                                  cache["page_table"], lens)
    V_all = _gather(vp2, cache["page_table"], 0, int(lens[0]))
    G = w.num_q_heads // w.num_kv_heads
    for i in range(T):
        for h in range(w.num_q_heads):
            np.testing.assert_allclose(out2[0, i, h], V_all[:21 + i + 1, h // G].mean(axis=0), rtol=1e-12, atol=1e-13)


def test_prefill_equals_single_token_ar_decode_steps():
    """Prefilling n tokens == n cycles of the (separately pinned) decode oracle with a block of one row:
    AR-verify attention of the token over the cache and itself, then a commit of that one row."""
    w = _w(batch=2, context_range=(3, 30))
    cache = make_cache(w)
    T = 6
    q, kn, vn = _new_tokens(w, T, 14)
    new_lens = np.array([T, T], np.int32)
    kp, vp, lens = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    out, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn, new_lens, kp, vp, cache["page_table"], lens)
    kp2, vp2, lens2 = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    V = 7
    logits = np.zeros((w.batch, 1, V), np.float32); logits[:, :, 3] = 1.0
    drafts = np.full((w.batch, 1), 3, np.int32)
    for i in range(T):
        c = np.ascontiguousarray
        step = oracle.dual_view_attn(oracle.VIEW_AR_VERIFY, w.sm_scale, c(q[:, i:i + 1]), c(kn[:, i:i + 1]),
                                     c(vn[:, i:i + 1]), kp2, vp2, cache["page_table"], lens2)
        np.testing.assert_allclose(step[:, 0], out[:, i], rtol=1e-12, atol=1e-13)
        oracle.consensus_commit(logits, drafts, np.ascontiguousarray(kn[:, i:i + 1]),
                                np.ascontiguousarray(vn[:, i:i + 1]), kp2, vp2, cache["page_table"], lens2)
    np.testing.assert_array_equal(lens, lens2)
    np.testing.assert_array_equal(kp, kp2)
    np.testing.assert_array_equal(vp, vp2)


def test_any_chunking_of_the_prompt_gives_the_same_result():
    w = _w(batch=2, context_range=(0, 25))
    cache = make_cache(w)
    T = 11
    q, kn, vn = _new_tokens(w, T, 15)
    whole_k, whole_v, whole_l = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    whole, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn, np.array([T, 7], np.int32), whole_k, whole_v,
                                   cache["page_table"], whole_l)
    ck, cv, cl = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    parts = []
    for lo, hi, n in ((0, 4, [4, 4]), (4, 5, [1, 1]), (5, 11, [6, 2])):
        o, _ = oracle.prefill_attn(w.sm_scale, np.ascontiguousarray(q[:, lo:hi]), np.ascontiguousarray(kn[:, lo:hi]),
                                   np.ascontiguousarray(vn[:, lo:hi]), np.array(n, np.int32), ck, cv,
                                   cache["page_table"], cl)
        parts.append(o)
    chunked = np.concatenate(parts, axis=1)
    np.testing.assert_array_equal(cl, whole_l)
    np.testing.assert_array_equal(ck, whole_k)
    np.testing.assert_array_equal(cv, whole_v)
    m = ~np.isnan(whole)
    np.testing.assert_array_equal(np.isnan(chunked), np.isnan(whole))
    np.testing.assert_allclose(chunked[m], whole[m], rtol=1e-12, atol=1e-13)


def test_unmapped_page_leaves_the_sequence_untouched():
    w = _w(batch=2, context=14, context_range=None, steps=1)
    cache = make_cache(w)
    pt = cache["page_table"].copy()
    pt[1, 1:] = -1                    # sequence 1 cannot grow past 16 tokens
    q, kn, vn = _new_tokens(w, 5, 16)
    kp, vp, lens = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    out, rc = oracle.prefill_attn(w.sm_scale, q, kn, vn, np.array([1, 5], np.int32), kp, vp, pt, lens,
                                  allow_capacity_error=True)
    assert rc == -4
    assert lens.tolist() == [15, 14]
    assert np.isnan(out[1]).all() and not np.isnan(out[0, 0]).any()
    np.testing.assert_array_equal(_gather(kp, pt, 1, 14), _gather(cache["k_pool"], pt, 1, 14))
