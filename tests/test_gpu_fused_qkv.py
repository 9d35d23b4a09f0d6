"""The block's inputs read in place from a fused Q/K/V projection output (Section 3.1, "Parallel Diffusion
View": the K block positions are projected by the view's W_Q, W_K, W_V; Fig. 2(b): the AR view's K/V of the
accepted positions enter the cache).  The projection itself is outside the path; what the path fixes is that
q, k_blk and v_blk of a view are the three column ranges of one [B*K, (H_q + 2 H_kv) * d] buffer per layer,
which the kernels address through strides instead of a copy.  The oracle sees dense copies cut out with numpy
slicing; attention within the contract tolerance, commit bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from orthrus_inputs import Workload, bf16_bits_to_f32, f32_to_bf16_bits, make_cache, make_consensus_case

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS, REL_L2 = 2e-2, 2e-3, 1e-2


def _fused(w, layers, seed):
    """bf16 bits [layers, B*K, (H_q + 2 H_kv) * d] ~ N(0,1) plus dense views of its three column ranges."""
    rng = np.random.default_rng(seed)
    width = (w.num_q_heads + 2 * w.num_kv_heads) * w.head_dim
    buf = f32_to_bf16_bits(rng.standard_normal((layers, w.batch * w.block_k, width), dtype=np.float32))
    nq, nk = w.num_q_heads * w.head_dim, w.num_kv_heads * w.head_dim
    shape = lambda h: (layers, w.batch, w.block_k, h, w.head_dim)
    q = np.ascontiguousarray(buf[:, :, :nq]).reshape(shape(w.num_q_heads))
    k = np.ascontiguousarray(buf[:, :, nq:nq + nk]).reshape(shape(w.num_kv_heads))
    v = np.ascontiguousarray(buf[:, :, nq + nk:]).reshape(shape(w.num_kv_heads))
    return buf, q, k, v


@pytest.mark.parametrize("shape", [dict(batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=16),
                                   dict(batch=2, num_q_heads=6, num_kv_heads=2, head_dim=64, block_k=7),
                                   dict(batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=32)])
@pytest.mark.parametrize("splits", [0, 3, -1])
def test_attention_and_commit_read_the_fused_projection_output_in_place(shape, splits):
    from paper_2605_12825_amd import runtime as rt
    layers = 2
    w = Workload(name="fused", context_range=(0, 400), page_size=16, vocab=3000, accept="uniform", steps=1,
                 seed=700 + shape["block_k"], **shape)
    caches = [make_cache(w, seed=w.seed + l, seq_lens=None if l == 0 else None) for l in range(layers)]
    lens = caches[0]["seq_lens"]
    caches = [make_cache(w, seed=w.seed + l, seq_lens=lens) for l in range(layers)]
    kp = np.stack([c["k_pool"] for c in caches]); vp = np.stack([c["v_pool"] for c in caches])
    pt = caches[0]["page_table"]
    buf_d, q_d, k_d, v_d = _fused(w, layers, w.seed + 10)      # diffusion view's projections of the block
    buf_a, q_a, k_a, v_a = _fused(w, layers, w.seed + 11)      # AR view's
    width = buf_d.shape[2]
    nq, nk = w.num_q_heads * w.head_dim, w.num_kv_heads * w.head_dim
    D = rt.to_device_bits
    dkp, dvp, dpt, dlen = D(kp), D(vp), D(pt), D(lens)
    dev_d, dev_a = D(buf_d), D(buf_a)
    pages, H, P, d = kp.shape[1:]
    step = rt.DecodeStep(batch=w.batch, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                         block_k=w.block_k, page_size=P, max_pages_per_seq=pt.shape[1],
                         max_seq_len=min(int(lens.max()) + w.block_k, pt.shape[1] * P), num_pages=pages, vocab=w.vocab,
                         num_layers=layers, num_splits=splits, pool_strides=(pages * H * P * d, H * P * d, P * d, d),
                         block_strides=(width, w.head_dim, width, w.head_dim, w.batch * w.block_k * width))
    esz = 2
    for view, dev, q, k, v in ((0, dev_d, q_d, k_d, v_d), (1, dev_a, q_a, k_a, v_a)):
        for l in range(layers):
            base = dev.data_ptr() + l * w.batch * w.block_k * width * esz
            out = torch.full((w.batch, w.block_k, w.num_q_heads, w.head_dim), 0x7FC0, dtype=torch.int16, device="cuda")
            step.attn(view, base, base + nq * esz, base + (nq + nk) * esz, dkp[l], dvp[l], dpt, dlen, out)
            torch.cuda.synchronize()
            got = bf16_bits_to_f32(rt.bits_to_numpy(out)).astype(np.float64)
            want = oracle.dual_view_attn(view, w.sm_scale, q[l], k[l], v[l], kp[l], vp[l], pt, lens)
            err = np.abs(got - want)
            assert np.isfinite(got).all() and err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (view, l, err.max())
            rel = np.sqrt((err ** 2).sum(axis=(1, 3))) / np.maximum(np.sqrt((want ** 2).sum(axis=(1, 3))), 1e-30)
            assert rel.max() <= REL_L2, (view, l, rel.max())
    # consensus + commit of the AR view's K/V rows straight out of the fused buffers (all layers in one call)
    cc = make_consensus_case(w, seed=w.seed + 20)
    outs = [torch.full((w.batch,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
    toks = torch.full((w.batch, w.block_k), -7, dtype=torch.int32, device="cuda")
    base = dev_a.data_ptr()
    step.consensus_commit(D(cc["ar_logits"]), D(cc["draft_tokens"]), base + nq * esz, base + (nq + nk) * esz, dkp, dvp,
                          dpt, dlen, outs[0], outs[1], toks, outs[2])
    torch.cuda.synchronize()
    ref_k, ref_v, ref_len = kp.copy(), vp.copy(), lens.copy()
    want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"], k_a, v_a, ref_k, ref_v, pt, ref_len)
    np.testing.assert_array_equal(outs[0].cpu().numpy(), want["accept_len"])
    np.testing.assert_array_equal(outs[1].cpu().numpy(), want["num_committed"])
    np.testing.assert_array_equal(toks.cpu().numpy(), want["out_tokens"])
    np.testing.assert_array_equal(dlen.cpu().numpy(), ref_len)
    np.testing.assert_array_equal(rt.bits_to_numpy(dkp), ref_k)
    np.testing.assert_array_equal(rt.bits_to_numpy(dvp), ref_v)
    assert step.device_error() == 0
    step.close()
