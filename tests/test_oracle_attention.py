"""Pins for the attention oracle (CPU only).

The oracle is checked against things other than itself:
  * Eq. 4 of the paper evaluated literally with numpy on a materialised key axis and an
    explicit boolean mask (different code route: gather + matmul + masked softmax);
  * torch's scaled_dot_product_attention on CPU in fp64 with the same boolean mask (library);
  * a hand-worked example whose softmax weights are 1/6, 2/6, 3/6;
  * closed forms and invariants: equal keys -> mean of the visible values, constant values,
    a dominant key, convex-hull bound, K=1 == ordinary causal decode attention, AR-view row i
    == decode over cache + first i+1 block rows, diffusion view invariant under in-block
    permutation, last AR row == last diffusion row, page-permutation invariance.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from orthrus_inputs import Workload, bf16_bits_to_f32, f32_to_bf16_bits, make_block, make_cache

DIFF, AR = oracle.VIEW_DIFFUSION, oracle.VIEW_AR_VERIFY


def _w(**kw):
    base = dict(name="t", batch=2, num_q_heads=4, num_kv_heads=2, head_dim=16, block_k=3,
                context=20, page_size=4, paging="shuffled", seed=7)
    base.update(kw)
    return Workload(**base)


def _inputs(w, seed=0, seq_lens=None):
    c = make_cache(w, seed=w.seed + seed, seq_lens=seq_lens)
    b = make_block(w, seed=w.seed + 100 + seed)
    return c, b


def _gather_logical(pool, page_table, b, L):
    """[L, H_kv, d] fp64 logical cache of sequence b, gathered with numpy indexing."""
    P = pool.shape[2]
    pos = np.arange(L)
    pages = page_table[b, pos // P]
    return bf16_bits_to_f32(pool[pages, :, pos % P, :]).astype(np.float64)


def _brute_force(view, scale, q, k_blk, v_blk, k_pool, v_pool, page_table, seq_lens):
    """Eq. 4 literally: concatenate keys along the sequence axis, mask, softmax, multiply by values."""
    B, K, Hq, d = q.shape
    Hkv = k_blk.shape[2]
    G = Hq // Hkv
    qf = bf16_bits_to_f32(q).astype(np.float64)
    kb = bf16_bits_to_f32(k_blk).astype(np.float64)
    vb = bf16_bits_to_f32(v_blk).astype(np.float64)
    out = np.zeros((B, K, Hq, d))
    for b in range(B):
        L = int(seq_lens[b])
        kc = _gather_logical(k_pool, page_table, b, L)
        vc = _gather_logical(v_pool, page_table, b, L)
        for h in range(Hq):
            g = h // G
            keys = np.concatenate([kc[:, g, :], kb[b, :, g, :]], axis=0)        # [L+K, d]
            vals = np.concatenate([vc[:, g, :], vb[b, :, g, :]], axis=0)
            mask = np.ones((K, L + K), dtype=bool)
            if view == AR:
                mask[:, L:] = np.tril(np.ones((K, K), dtype=bool))
            s = (qf[b, :, h, :] @ keys.T) * scale
            s = np.where(mask, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            out[b, :, h, :] = p @ vals
    return out


SHAPES = [
    dict(batch=1, num_q_heads=1, num_kv_heads=1, head_dim=8, block_k=1, context=1, page_size=1),
    dict(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=16, block_k=3, context=20, page_size=4),
    dict(batch=3, num_q_heads=6, num_kv_heads=2, head_dim=32, block_k=5, context_range=(0, 40), page_size=16),
    dict(batch=2, num_q_heads=7, num_kv_heads=1, head_dim=64, block_k=4, context_range=(1, 70), page_size=16,
         paging="scattered"),
    dict(batch=1, num_q_heads=4, num_kv_heads=4, head_dim=128, block_k=8, context=33, page_size=16,
         paging="contiguous"),
]


@pytest.mark.parametrize("view", [DIFF, AR])
@pytest.mark.parametrize("shape", SHAPES)
def test_matches_literal_eq4_brute_force(shape, view):
    w = _w(**shape)
    c, b = _inputs(w)
    got = oracle.dual_view_attn(view, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                c["page_table"], c["seq_lens"])
    want = _brute_force(view, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                        c["page_table"], c["seq_lens"])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("view", [DIFF, AR])
def test_matches_torch_sdpa_fp64(view):
    w = _w(batch=2, num_q_heads=6, num_kv_heads=3, head_dim=32, block_k=4, context_range=(5, 30), page_size=8)
    c, b = _inputs(w, seed=3)
    got = oracle.dual_view_attn(view, 0.37, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                c["page_table"], c["seq_lens"])
    G, K = w.group, w.block_k
    for bi in range(w.batch):
        L = int(c["seq_lens"][bi])
        kc = torch.from_numpy(_gather_logical(c["k_pool"], c["page_table"], bi, L))
        vc = torch.from_numpy(_gather_logical(c["v_pool"], c["page_table"], bi, L))
        kb = torch.from_numpy(bf16_bits_to_f32(b["k_blk"][bi]).astype(np.float64))
        vb = torch.from_numpy(bf16_bits_to_f32(b["v_blk"][bi]).astype(np.float64))
        keys = torch.cat([kc, kb], 0).permute(1, 0, 2).repeat_interleave(G, dim=0)   # [Hq, L+K, d]
        vals = torch.cat([vc, vb], 0).permute(1, 0, 2).repeat_interleave(G, dim=0)
        qq = torch.from_numpy(bf16_bits_to_f32(b["q"][bi]).astype(np.float64)).permute(1, 0, 2)  # [Hq, K, d]
        mask = torch.ones(K, L + K, dtype=torch.bool)
        if view == AR:
            mask[:, L:] = torch.tril(torch.ones(K, K, dtype=torch.bool))
        ref = torch.nn.functional.scaled_dot_product_attention(qq, keys, vals, attn_mask=mask, scale=0.37)
        np.testing.assert_allclose(got[bi], ref.permute(1, 0, 2).numpy(), rtol=1e-11, atol=1e-12)


def _manual_case(q_rows, cache_k, cache_v, blk_k, blk_v, page_size=2):
    """Single head, batch 1, identity paging, from python lists (values exactly representable in bf16)."""
    d = len(q_rows[0])
    K, L = len(q_rows), len(cache_k)
    npages = max(1, (L + page_size - 1) // page_size)
    kp = np.zeros((npages, 1, page_size, d), np.float32)
    vp = np.zeros_like(kp)
    for j in range(L):
        kp[j // page_size, 0, j % page_size] = cache_k[j]
        vp[j // page_size, 0, j % page_size] = cache_v[j]
    conv = lambda x: f32_to_bf16_bits(np.asarray(x, np.float32))
    q = conv(q_rows).reshape(1, K, 1, d)
    kb = conv(blk_k).reshape(1, K, 1, d)
    vb = conv(blk_v).reshape(1, K, 1, d)
    pt = np.arange(npages, dtype=np.int32).reshape(1, npages)
    return q, kb, vb, conv(kp), conv(vp), pt, np.array([L], np.int32)


def test_hand_worked_weights_one_two_three_sixths():
    # scores s = q.k with q = (1, 0): choose k_x = ln 1, ln 2 (cache) and ln 3 (in-block anchor row).
    # bf16 rounds ln 2 and ln 3, so the expected weights use the rounded values exactly.
    ks = [float(bf16_bits_to_f32(f32_to_bf16_bits(np.array([math.log(x)], np.float32)))[0]) for x in (1, 2, 3)]
    e = [math.exp(k) for k in ks]
    vals = [4.0, -2.0, 8.0]
    want = math.fsum(a * v for a, v in zip(e, vals)) / math.fsum(e)
    args = _manual_case([[1.0, 0.0]], [[ks[0], 5.0], [ks[1], -3.0]], [[vals[0], 0.0], [vals[1], 0.0]],
                        [[ks[2], 9.0]], [[vals[2], 0.0]])
    for view in (DIFF, AR):
        out, lse = oracle.dual_view_attn(view, 1.0, *args, want_lse=True)
        assert out.shape == (1, 1, 1, 2)
        assert abs(out[0, 0, 0, 0] - want) < 1e-14
        assert out[0, 0, 0, 1] == 0.0
        assert abs(lse[0, 0, 0] - math.log(math.fsum(e))) < 1e-14
    # the weights are within bf16 rounding of 1/6, 2/6, 3/6 -> value close to (4 - 4 + 24)/6 = 4
    assert abs(want - 4.0) < 0.05


def test_sm_scale_is_applied_to_scores_only():
    # one cache key and the anchor key; q.k = 2 and 0 -> weights sigmoid(2*scale)
    args = _manual_case([[2.0, 0.0]], [[1.0, 0.0]], [[1.0, 10.0]], [[0.0, 0.0]], [[3.0, 20.0]])
    for scale in (1.0, 0.5, 0.125):
        out = oracle.dual_view_attn(DIFF, scale, *args)
        a = 1.0 / (1.0 + math.exp(-2.0 * scale))
        assert abs(out[0, 0, 0, 0] - (a * 1.0 + (1 - a) * 3.0)) < 1e-14
        assert abs(out[0, 0, 0, 1] - (a * 10.0 + (1 - a) * 20.0)) < 1e-13


def test_equal_keys_give_mean_of_visible_values():
    # every key identical -> uniform softmax -> mean over exactly the visible rows.
    # This separates the two views: diffusion rows all see L+K values, AR row i sees L+i+1.
    w = _w(batch=1, num_q_heads=2, num_kv_heads=1, head_dim=8, block_k=4, context=6, page_size=4,
           paging="contiguous")
    c, b = _inputs(w)
    one = f32_to_bf16_bits(np.float32(0.75))
    c["k_pool"][...] = one
    b["k_blk"][...] = one
    L, K = 6, 4
    vc = _gather_logical(c["v_pool"], c["page_table"], 0, L)[:, 0, :]
    vb = bf16_bits_to_f32(b["v_blk"][0, :, 0, :]).astype(np.float64)
    out_d = oracle.dual_view_attn(DIFF, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                  c["page_table"], c["seq_lens"])
    out_a = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                  c["page_table"], c["seq_lens"])
    full_mean = (vc.sum(0) + vb.sum(0)) / (L + K)
    for i in range(K):
        for h in range(2):
            np.testing.assert_allclose(out_d[0, i, h], full_mean, rtol=1e-13, atol=1e-14)
            causal_mean = (vc.sum(0) + vb[: i + 1].sum(0)) / (L + i + 1)
            np.testing.assert_allclose(out_a[0, i, h], causal_mean, rtol=1e-13, atol=1e-14)


def test_constant_values_and_convex_hull():
    w = _w()
    c, b = _inputs(w, seed=5)
    out = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                c["page_table"], c["seq_lens"])
    for bi in range(w.batch):
        L = int(c["seq_lens"][bi])
        vc = _gather_logical(c["v_pool"], c["page_table"], bi, L)
        vb = bf16_bits_to_f32(b["v_blk"][bi]).astype(np.float64)
        allv = np.concatenate([vc, vb], 0)                      # [L+K, Hkv, d]
        for h in range(w.num_q_heads):
            g = h // w.group
            lo, hi = allv[:, g].min(0), allv[:, g].max(0)
            assert np.all(out[bi, :, h] >= lo - 1e-12) and np.all(out[bi, :, h] <= hi + 1e-12)
    const = f32_to_bf16_bits(np.float32(-1.5))
    c["v_pool"][...] = const
    b["v_blk"][...] = const
    out = oracle.dual_view_attn(DIFF, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                c["page_table"], c["seq_lens"])
    np.testing.assert_allclose(out, -1.5, rtol=0, atol=1e-14)


def test_dominant_key_selects_its_value():
    # key j* = 64 * q direction: its score exceeds the rest by hundreds -> output == that value row
    d = 4
    qrow = [1.0, 1.0, 0.0, 0.0]
    cache_k = [[0.5, -0.5, 1.0, 1.0], [64.0, 64.0, 0.0, 0.0], [1.0, 0.0, 0.0, 2.0]]
    cache_v = [[1.0, 2.0, 3.0, 4.0], [-7.0, 0.5, 0.25, 100.0], [9.0, 9.0, 9.0, 9.0]]
    args = _manual_case([qrow], cache_k, cache_v, [[0.0] * d], [[5.0] * d])
    out = oracle.dual_view_attn(AR, 1.0, *args)
    np.testing.assert_allclose(out[0, 0, 0], cache_v[1], rtol=0, atol=1e-40)


def test_block_of_one_is_ordinary_causal_decode():
    """K=1: both views coincide and equal single-query attention over cache + the token itself."""
    w = _w(batch=3, num_q_heads=8, num_kv_heads=2, head_dim=32, block_k=1, context_range=(0, 50), page_size=16)
    c, b = _inputs(w, seed=2)
    args = (b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"], c["page_table"], c["seq_lens"])
    out_d = oracle.dual_view_attn(DIFF, w.sm_scale, *args)
    out_a = oracle.dual_view_attn(AR, w.sm_scale, *args)
    np.testing.assert_array_equal(out_d, out_a)
    for bi in range(w.batch):
        L = int(c["seq_lens"][bi])
        kc = _gather_logical(c["k_pool"], c["page_table"], bi, L)
        vc = _gather_logical(c["v_pool"], c["page_table"], bi, L)
        keys = torch.from_numpy(np.concatenate([kc, bf16_bits_to_f32(b["k_blk"][bi]).astype(np.float64)], 0))
        vals = torch.from_numpy(np.concatenate([vc, bf16_bits_to_f32(b["v_blk"][bi]).astype(np.float64)], 0))
        keys = keys.permute(1, 0, 2).repeat_interleave(w.group, 0)
        vals = vals.permute(1, 0, 2).repeat_interleave(w.group, 0)
        qq = torch.from_numpy(bf16_bits_to_f32(b["q"][bi]).astype(np.float64)).permute(1, 0, 2)
        ref = torch.nn.functional.scaled_dot_product_attention(qq, keys, vals)   # default scale 1/sqrt(d), no mask
        np.testing.assert_allclose(out_a[bi], ref.permute(1, 0, 2).numpy(), rtol=1e-11, atol=1e-12)


def test_ar_row_equals_sequential_decode_with_growing_cache():
    """AR-view row i == the K=1 case run on a cache that already holds block rows 0..i-1."""
    w = _w(batch=1, num_q_heads=4, num_kv_heads=2, head_dim=16, block_k=4, context=9, page_size=4,
           paging="contiguous", steps=1)
    c, b = _inputs(w)
    out = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                c["page_table"], c["seq_lens"])
    kp, vp = c["k_pool"].copy(), c["v_pool"].copy()
    L, P = 9, 4
    for i in range(w.block_k):
        one = dict(q=b["q"][:, i:i + 1].copy(), k=b["k_blk"][:, i:i + 1].copy(), v=b["v_blk"][:, i:i + 1].copy())
        got = oracle.dual_view_attn(AR, w.sm_scale, one["q"], one["k"], one["v"], kp, vp, c["page_table"],
                                    np.array([L + i], np.int32))
        np.testing.assert_allclose(got[0, 0], out[0, i], rtol=1e-12, atol=1e-13)
        pos = L + i                       # append row i, as one AR decode step would
        pg = c["page_table"][0, pos // P]
        kp[pg, :, pos % P, :] = b["k_blk"][0, i]
        vp[pg, :, pos % P, :] = b["v_blk"][0, i]


def test_diffusion_view_is_bidirectional_inside_the_block():
    w = _w(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=16, block_k=5, context=11, page_size=4)
    c, b = _inputs(w, seed=9)
    args = (c["k_pool"], c["v_pool"], c["page_table"], c["seq_lens"])
    base = oracle.dual_view_attn(DIFF, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], *args)
    perm = np.array([3, 0, 4, 2, 1])
    shuf = oracle.dual_view_attn(DIFF, w.sm_scale, b["q"], np.ascontiguousarray(b["k_blk"][:, perm]),
                                 np.ascontiguousarray(b["v_blk"][:, perm]), *args)
    np.testing.assert_allclose(shuf, base, rtol=1e-12, atol=1e-13)
    ar = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], *args)
    np.testing.assert_allclose(ar[:, -1], base[:, -1], rtol=1e-12, atol=1e-13)       # last row sees everything
    assert np.abs(ar[:, 0] - base[:, 0]).max() > 1e-3                                  # earlier rows do not
    # the AR view must ignore later in-block rows entirely
    kb2, vb2 = b["k_blk"].copy(), b["v_blk"].copy()
    kb2[:, 3:] = f32_to_bf16_bits(np.float32(50.0))
    vb2[:, 3:] = f32_to_bf16_bits(np.float32(-50.0))
    ar2 = oracle.dual_view_attn(AR, w.sm_scale, b["q"], kb2, vb2, *args)
    np.testing.assert_array_equal(ar2[:, :3], ar[:, :3])


def test_page_permutation_invariance_and_garbage_beyond_length():
    w = _w(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=16, block_k=3, context_range=(3, 30), page_size=4,
           paging="scattered")
    c, b = _inputs(w, seed=4)
    base = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                 c["page_table"], c["seq_lens"])
    rng = np.random.default_rng(0)
    n = c["k_pool"].shape[0]
    perm = rng.permutation(n)                    # new physical id of old page p is perm[p]
    kp2 = np.empty_like(c["k_pool"]); vp2 = np.empty_like(c["v_pool"])
    kp2[perm] = c["k_pool"]; vp2[perm] = c["v_pool"]
    pt2 = np.where(c["page_table"] >= 0, perm[np.maximum(c["page_table"], 0)], -1).astype(np.int32)
    moved = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], kp2, vp2, pt2, c["seq_lens"])
    np.testing.assert_array_equal(moved, base)
    # entries past seq_lens (same page, later slots) and unmapped pages must not matter
    kp3, vp3 = c["k_pool"].copy(), c["v_pool"].copy()
    P = 4
    used = np.zeros((n, P), bool)
    for bi in range(w.batch):
        for j in range(int(c["seq_lens"][bi])):
            used[c["page_table"][bi, j // P], j % P] = True
    junk = f32_to_bf16_bits(np.float32(77.0))
    for pg in range(n):
        for s in range(P):
            if not used[pg, s]:
                kp3[pg, :, s, :] = junk
                vp3[pg, :, s, :] = junk
    same = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], kp3, vp3, c["page_table"],
                                 c["seq_lens"])
    np.testing.assert_array_equal(same, base)


def test_empty_cache_first_ar_row_returns_its_own_value():
    w = _w(batch=1, num_q_heads=2, num_kv_heads=1, head_dim=8, block_k=3, context=0, page_size=4)
    c, b = _inputs(w)
    out = oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                                c["page_table"], c["seq_lens"])
    v0 = bf16_bits_to_f32(b["v_blk"][0, 0, 0]).astype(np.float64)
    np.testing.assert_array_equal(out[0, 0, 0], v0)
    np.testing.assert_array_equal(out[0, 0, 1], v0)


def test_unmapped_page_is_an_error():
    w = _w(batch=1, context=10, page_size=4)
    c, b = _inputs(w)
    c["page_table"][0, 1] = -1
    with pytest.raises(RuntimeError):
        oracle.dual_view_attn(AR, w.sm_scale, b["q"], b["k_blk"], b["v_blk"], c["k_pool"], c["v_pool"],
                              c["page_table"], c["seq_lens"])
