"""The diffusion view's training block mask (Section 3.2, Eq. 6) on the GPU: a block with anchor a is one
batch entry of orthrus_dual_view_attn(DIFFUSION) whose cache is the first a tokens of the clean context.  The
clean context's K/V stay in their plain [L, H_kv, d] layout: the pool strides describe it as 16-token pages."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from orthrus_inputs import bf16_bits_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def _run_gpu(L, NB, K, Hq, Hkv, d, anchors, q, k_ar, v_ar, k_diff, v_diff, sm_scale):
    from paper_2605_12825_amd import runtime as rt
    P = 16
    pages = (L + P - 1) // P
    step = rt.DecodeStep(batch=NB, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, block_k=K, page_size=P,
                         max_pages_per_seq=pages, max_seq_len=L, num_pages=pages, sm_scale=sm_scale,
                         pool_strides=(0, P * Hkv * d, d, Hkv * d))
    D = rt.to_device_bits
    page_table = D(np.tile(np.arange(pages, dtype=np.int32), (NB, 1)))
    out = torch.zeros((NB, K, Hq, d), dtype=torch.int16, device="cuda")
    step.attn(0, D(q.reshape(NB, K, Hq, d)), D(k_diff.reshape(NB, K, Hkv, d)), D(v_diff.reshape(NB, K, Hkv, d)),
              D(k_ar), D(v_ar), page_table, D(anchors), out)
    torch.cuda.synchronize()
    assert step.device_error() == 0
    res = bf16_bits_to_f32(rt.bits_to_numpy(out)).astype(np.float64).reshape(NB * K, Hq, d)
    step.close()
    return res


@pytest.mark.parametrize("shape", [
    dict(L=2048, NB=256, K=32, Hq=32, Hkv=8, d=128),      # the paper's training geometry (Appendix A) at the 8B head shape
    dict(L=333, NB=9, K=8, Hq=4, Hkv=2, d=64),
    dict(L=100, NB=3, K=32, Hq=14, Hkv=2, d=128),
])
def test_training_block_mask_forward(shape):
    L, NB, K, Hq, Hkv, d = (shape[k] for k in ("L", "NB", "K", "Hq", "Hkv", "d"))
    rng = np.random.default_rng(900 + L)
    mk = lambda n, h: f32_to_bf16_bits(rng.standard_normal((n, h, d), dtype=np.float32))
    anchors = np.sort(rng.integers(1, L + 1, size=NB)).astype(np.int32)
    q, k_ar, v_ar = mk(NB * K, Hq), mk(L, Hkv), mk(L, Hkv)
    k_diff, v_diff = mk(NB * K, Hkv), mk(NB * K, Hkv)
    sm = 1.0 / np.sqrt(d)
    got = _run_gpu(L, NB, K, Hq, Hkv, d, anchors, q, k_ar, v_ar, k_diff, v_diff, sm)
    assert np.all(np.isfinite(got))
    # the oracle evaluates Eq. 6 on a sample of blocks (blocks cannot see each other, so a subset of blocks is
    # a problem of its own: a property the oracle's own pins establish)
    pick = np.arange(NB) if NB <= 12 else np.sort(rng.choice(NB, size=12, replace=False))
    rows = (pick[:, None] * K + np.arange(K)[None, :]).reshape(-1)
    want = oracle.block_mask_attn(sm, K, anchors[pick], q[rows], k_ar, v_ar, k_diff[rows], v_diff[rows])
    err = np.abs(got[rows] - want)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (err.max(), err.mean())
