"""AR-view prefill attention on the GPU (orthrus_prefill_attn) against the CPU oracle: the causal
self-attention that builds the shared cache (Section 3.1)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from orthrus_inputs import Workload, bf16_bits_to_f32, f32_to_bf16_bits, make_block, make_cache

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3   # bf16 in, fp32 accumulate, bf16 out
SENTINEL = 0x7FC1                # a NaN pattern: rows the call must not write keep it


def _rt():
    from paper_2605_12825_amd import runtime
    return runtime


def _new_tokens(w, T, seed):
    rng = np.random.default_rng(seed)
    mk = lambda h: f32_to_bf16_bits(rng.standard_normal((w.batch, T, h, w.head_dim), dtype=np.float32))
    return mk(w.num_q_heads), mk(w.num_kv_heads), mk(w.num_kv_heads)


class Case:
    def __init__(self, w, cache, max_seq_len):
        rt = _rt()
        self.w, self.cache = w, cache
        self.k_pool, self.v_pool = rt.to_device_bits(cache["k_pool"]), rt.to_device_bits(cache["v_pool"])
        self.page_table, self.seq_lens = rt.to_device_bits(cache["page_table"]), rt.to_device_bits(cache["seq_lens"])
        self.step = rt.DecodeStep(batch=w.batch, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                                  head_dim=w.head_dim, block_k=w.block_k, page_size=w.page_size,
                                  max_pages_per_seq=cache["page_table"].shape[1], max_seq_len=max_seq_len,
                                  num_pages=cache["k_pool"].shape[0])

    def prefill(self, q, kn, vn, new_lens):
        rt = _rt()
        T = q.shape[1]
        out = torch.full(q.shape, SENTINEL, dtype=torch.int16, device="cuda")
        self.step.prefill(T, rt.to_device_bits(q), rt.to_device_bits(kn), rt.to_device_bits(vn),
                          rt.to_device_bits(new_lens), self.k_pool, self.v_pool, self.page_table, self.seq_lens, out)
        torch.cuda.synchronize()
        return rt.bits_to_numpy(out)

    def state(self):
        rt = _rt()
        return rt.bits_to_numpy(self.k_pool), rt.bits_to_numpy(self.v_pool), self.seq_lens.cpu().numpy()


def _check(bits, want, new_lens):
    got = bf16_bits_to_f32(bits).astype(np.float64)
    for b, n in enumerate(new_lens):
        n = int(n)
        if n:
            err = np.abs(got[b, :n] - want[b, :n])
            assert np.all(np.isfinite(got[b, :n]))
            assert err.max() <= MAX_ABS, "sequence %d max-abs %.4g" % (b, err.max())
            assert err.mean() <= MEAN_ABS, "sequence %d mean-abs %.4g" % (b, err.mean())
        assert (bits[b, n:] == SENTINEL).all(), "rows past new_lens[%d] were written" % b


SHAPES = [
    # (workload kwargs, T, new_lens)
    (dict(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=64, context_range=(0, 100), page_size=16), 40, [40, 13]),
    (dict(batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, context_range=(1, 200), page_size=16), 70, [70, 0, 33]),
    (dict(batch=2, num_q_heads=4, num_kv_heads=4, head_dim=128, context_range=(0, 64), page_size=32), 65, [64, 65]),
    (dict(batch=2, num_q_heads=14, num_kv_heads=2, head_dim=128, context_range=(5, 90), page_size=16,
          paging="scattered"), 50, [50, 31]),
    (dict(batch=1, num_q_heads=8, num_kv_heads=1, head_dim=64, context=0, page_size=64), 100, [100]),
    (dict(batch=4, num_q_heads=6, num_kv_heads=2, head_dim=128, context_range=(0, 40), page_size=16), 32, [1, 32, 31, 2]),
    (dict(batch=1, num_q_heads=2, num_kv_heads=2, head_dim=128, context=0, page_size=16), 1, [1]),
    (dict(batch=2, num_q_heads=5, num_kv_heads=1, head_dim=128, context_range=(3, 70), page_size=16), 45, [45, 20]),
    (dict(batch=2, num_q_heads=12, num_kv_heads=2, head_dim=64, context_range=(0, 50), page_size=16), 33, [33, 32]),
]


@pytest.mark.parametrize("shape", range(len(SHAPES)))
def test_prefill_small_shapes(shape):
    kw, T, nl = SHAPES[shape]
    kw = dict(kw)
    kw.setdefault("paging", "shuffled")
    w = Workload(name="p%d" % shape, seed=700 + shape, block_k=8, steps=(T + 7) // 8 + 1, **kw)
    cache = make_cache(w)
    new_lens = np.array(nl, np.int32)
    q, kn, vn = _new_tokens(w, T, 800 + shape)
    ref_k, ref_v, ref_l = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    want, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn, new_lens, ref_k, ref_v, cache["page_table"], ref_l)
    case = Case(w, cache, max_seq_len=int(cache["seq_lens"].max()) + T)
    got = case.prefill(q, kn, vn, new_lens)
    _check(got, want, new_lens)
    k, v, l = case.state()
    np.testing.assert_array_equal(l, ref_l)
    np.testing.assert_array_equal(k, ref_k)
    np.testing.assert_array_equal(v, ref_v)
    assert case.step.device_error() == 0


def test_chunked_prefill_then_a_decode_step():
    """Two prefill calls in a row (the second continues the first), then the decode path reads that cache."""
    w = Workload(name="pc", seed=720, batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=8,
                 context=0, page_size=16, paging="shuffled", steps=20)
    cache = make_cache(w)
    ref_k, ref_v, ref_l = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    case = Case(w, cache, max_seq_len=w.capacity_tokens())
    for call, (T, nl) in enumerate(((48, [48, 20]), (37, [37, 37]))):
        q, kn, vn = _new_tokens(w, T, 730 + call)
        new_lens = np.array(nl, np.int32)
        want, _ = oracle.prefill_attn(w.sm_scale, q, kn, vn, new_lens, ref_k, ref_v, cache["page_table"], ref_l)
        _check(case.prefill(q, kn, vn, new_lens), want, new_lens)
    k, v, l = case.state()
    np.testing.assert_array_equal(l, ref_l)
    np.testing.assert_array_equal(k, ref_k)
    np.testing.assert_array_equal(v, ref_v)
    assert ref_l.tolist() == [85, 57]
    # the diffusion view now attends the cache the prefill built
    rt = _rt()
    blk = make_block(w, 740)
    out = torch.zeros((w.batch, w.block_k, w.num_q_heads, w.head_dim), dtype=torch.int16, device="cuda")
    case.step.attn(0, rt.to_device_bits(blk["q"]), rt.to_device_bits(blk["k_blk"]), rt.to_device_bits(blk["v_blk"]),
                   case.k_pool, case.v_pool, case.page_table, case.seq_lens, out)
    torch.cuda.synchronize()
    want = oracle.dual_view_attn(0, w.sm_scale, blk["q"], blk["k_blk"], blk["v_blk"], ref_k, ref_v,
                                 cache["page_table"], ref_l)
    err = np.abs(bf16_bits_to_f32(rt.bits_to_numpy(out)).astype(np.float64) - want)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


def test_prefill_capacity_error_leaves_the_sequence_untouched():
    w = Workload(name="pe", seed=750, batch=2, num_q_heads=4, num_kv_heads=2, head_dim=64, block_k=8, context=14,
                 page_size=16, paging="shuffled", steps=4)
    cache = make_cache(w)
    cache["page_table"][1, 1:] = -1        # sequence 1 cannot grow past 16 tokens
    q, kn, vn = _new_tokens(w, 20, 751)
    new_lens = np.array([20, 5], np.int32)
    ref_k, ref_v, ref_l = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    want, rc = oracle.prefill_attn(w.sm_scale, q, kn, vn, new_lens, ref_k, ref_v, cache["page_table"], ref_l,
                                   allow_capacity_error=True)
    assert rc == -4
    case = Case(w, cache, max_seq_len=14 + 20)
    got = case.prefill(q, kn, vn, new_lens)
    _check(got, want, np.array([20, 0]))
    k, v, l = case.state()
    np.testing.assert_array_equal(l, ref_l)
    np.testing.assert_array_equal(k, ref_k)
    np.testing.assert_array_equal(v, ref_v)
    assert case.step.device_error() == -4


def test_prefill_at_the_8b_layer_shape_sampled_rows():
    """32/8 heads, d=128, 2048 new tokens on an empty cache: the oracle checks a sample of sequences' rows
    through its chunking invariance (a prefix of the prompt is a prefill of its own)."""
    w = Workload(name="p8b", seed=760, batch=1, num_q_heads=32, num_kv_heads=8, head_dim=128, block_k=16,
                 context=0, page_size=16, paging="shuffled", steps=129)
    cache = make_cache(w)
    T = 2048
    q, kn, vn = _new_tokens(w, T, 761)
    new_lens = np.array([T], np.int32)
    case = Case(w, cache, max_seq_len=T)
    got = bf16_bits_to_f32(case.prefill(q, kn, vn, new_lens)).astype(np.float64)
    k, v, l = case.state()
    assert l.tolist() == [T]
    # cache rows: bit-exact against the inputs (gathered through the page table)
    pt, P = cache["page_table"], w.page_size
    for pos in (0, 1, 15, 16, 1023, 2047):
        np.testing.assert_array_equal(k[pt[0, pos // P], :, pos % P, :], kn[0, pos])
        np.testing.assert_array_equal(v[pt[0, pos // P], :, pos % P, :], vn[0, pos])
    # attention rows: the oracle prefills the first n tokens only; its last rows are rows n-3..n-1 of the whole
    for n in (3, 33, 700, 2048):
        rk, rv, rl = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
        lo = max(0, n - 40)
        if lo:   # cache the first `lo` tokens without attending, then prefill the last 40 of the prefix
            zq = np.zeros_like(q[:, :1])
            for pos in range(lo):
                rk[pt[0, pos // P], :, pos % P, :] = kn[0, pos]
                rv[pt[0, pos // P], :, pos % P, :] = vn[0, pos]
            rl[:] = lo
        c = np.ascontiguousarray
        want, _ = oracle.prefill_attn(w.sm_scale, c(q[:, lo:n]), c(kn[:, lo:n]), c(vn[:, lo:n]),
                                      np.array([n - lo], np.int32), rk, rv, pt, rl)
        err = np.abs(got[0, lo:n] - want[0])
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, "prefix %d" % n
