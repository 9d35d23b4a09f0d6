"""Pins for the training block-mask oracle (Section 3.2, Eq. 6): it must agree with the separately pinned
decode oracle block by block (a block with anchor a is a diffusion-view decode step over a cache of a tokens),
and it must have the two isolation properties the paper states for the mask."""
import numpy as np

import oracle
from orthrus_inputs import f32_to_bf16_bits


def _inputs(seed, L=37, NB=5, K=4, Hq=4, Hkv=2, d=16):
    rng = np.random.default_rng(seed)
    mk = lambda n, h: f32_to_bf16_bits(rng.standard_normal((n, h, d), dtype=np.float32))
    anchors = np.sort(rng.integers(1, L + 1, size=NB)).astype(np.int32)
    return dict(K=K, anchors=anchors, q=mk(NB * K, Hq), k_ar=mk(L, Hkv), v_ar=mk(L, Hkv),
                k_diff=mk(NB * K, Hkv), v_diff=mk(NB * K, Hkv), L=L, NB=NB, Hq=Hq, Hkv=Hkv, d=d)


def _run(x, **over):
    y = dict(x); y.update(over)
    return oracle.block_mask_attn(0.25, y["K"], y["anchors"], y["q"], y["k_ar"], y["v_ar"], y["k_diff"], y["v_diff"])


def test_each_block_is_a_diffusion_view_decode_step_over_the_context_before_its_anchor():
    x = _inputs(1)
    out = _run(x)
    L, NB, K, Hkv, d, P = x["L"], x["NB"], x["K"], x["Hkv"], x["d"], 16
    pages = (L + P - 1) // P
    pool_k = np.zeros((pages, Hkv, P, d), np.uint16); pool_v = np.zeros_like(pool_k)
    for t in range(L):
        pool_k[t // P, :, t % P] = x["k_ar"][t]; pool_v[t // P, :, t % P] = x["v_ar"][t]
    pt = np.tile(np.arange(pages, dtype=np.int32), (NB, 1))
    blk = lambda a: np.ascontiguousarray(a.reshape(NB, K, *a.shape[1:]))
    want = oracle.dual_view_attn(oracle.VIEW_DIFFUSION, 0.25, blk(x["q"]), blk(x["k_diff"]), blk(x["v_diff"]),
                                 pool_k, pool_v, pt, x["anchors"])
    np.testing.assert_allclose(out.reshape(want.shape), want, rtol=1e-12, atol=1e-13)


def test_blocks_do_not_see_each_other_and_nothing_at_or_after_the_anchor_leaks():
    x = _inputs(2)
    base = _run(x)
    K, NB, L = x["K"], x["NB"], x["L"]
    rng = np.random.default_rng(9)
    # another block's diffusion keys / values change nothing outside that block
    kd, vd = x["k_diff"].copy(), x["v_diff"].copy()
    kd[2 * K:3 * K] = f32_to_bf16_bits(rng.standard_normal(kd[2 * K:3 * K].shape, dtype=np.float32))
    vd[2 * K:3 * K] = f32_to_bf16_bits(rng.standard_normal(vd[2 * K:3 * K].shape, dtype=np.float32))
    moved = _run(x, k_diff=kd, v_diff=vd)
    keep = np.ones(NB * K, bool); keep[2 * K:3 * K] = False
    np.testing.assert_array_equal(moved[keep], base[keep])
    assert np.abs(moved[~keep] - base[~keep]).max() > 1e-3
    # clean-context keys at positions >= the largest anchor are invisible to every block
    amax = int(x["anchors"].max())
    if amax < L:
        ka, va = x["k_ar"].copy(), x["v_ar"].copy()
        ka[amax:] = f32_to_bf16_bits(rng.standard_normal(ka[amax:].shape, dtype=np.float32))
        va[amax:] = f32_to_bf16_bits(rng.standard_normal(va[amax:].shape, dtype=np.float32))
        np.testing.assert_array_equal(_run(x, k_ar=ka, v_ar=va), base)
    # a key just before a block's anchor is visible to it
    a0 = int(x["anchors"][0])
    va = x["v_ar"].copy()
    va[a0 - 1] = f32_to_bf16_bits(np.full(va[a0 - 1].shape, 50.0, np.float32))
    assert np.abs(_run(x, v_ar=va)[:K] - base[:K]).max() > 1e-3


def test_equal_keys_give_the_mean_over_exactly_the_allowed_set():
    x = _inputs(3)
    one = f32_to_bf16_bits(np.array([0.5], np.float32))[0]
    out = _run(x, k_ar=np.full_like(x["k_ar"], one), k_diff=np.full_like(x["k_diff"], one))
    from orthrus_inputs import bf16_bits_to_f32
    VA = bf16_bits_to_f32(x["v_ar"]).astype(np.float64); VD = bf16_bits_to_f32(x["v_diff"]).astype(np.float64)
    K, G = x["K"], x["Hq"] // x["Hkv"]
    for nb, a in enumerate(x["anchors"]):
        for h in range(x["Hq"]):
            vis = np.concatenate([VA[:a, h // G], VD[nb * K:(nb + 1) * K, h // G]])
            for i in range(K):
                np.testing.assert_allclose(out[nb * K + i, h], vis.mean(axis=0), rtol=1e-12, atol=1e-13)
