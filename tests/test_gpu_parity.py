"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.

Tolerances (bf16 inputs, fp32 accumulation, bf16 probabilities and output): attention
max-abs error <= 2e-2 and mean-abs error <= 2e-3 against the fp64 oracle; accept lengths,
committed tokens, lengths and cache contents bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
from orthrus_inputs import (WORKLOADS, Workload, bf16_bits_to_f32, f32_to_bf16_bits, make_block, make_cache,
                            make_consensus_case)

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3
# Second, scale-free criterion beside the contract's absolute one: per (sequence, query head) the error's
# Euclidean norm over the block's K x d outputs, relative to the oracle's.  With long random contexts the
# outputs themselves shrink to the size of the absolute tolerance, and only a relative bound still sees a
# lost split or a lost in-block tile.  What the arithmetic gives: bf16 probabilities and bf16 outputs carry
# a relative rounding error of at most 2^-9 each (about 1.1e-3 RMS each, 2e-3 together), so 1e-2 leaves a
# factor of five.
REL_L2 = 1e-2
DIFF, AR = 0, 1


def _orthrus():
    import paper_2605_12825_amd as o
    from paper_2605_12825_amd import runtime
    return o, runtime


def _dev(a):
    _, rt = _orthrus()
    return rt.to_device_bits(a)


class GpuCase:
    """Device copies of one workload's cache plus a DecodeStep for it."""

    def __init__(self, w: Workload, cache, num_splits=0, vocab=0, num_layers=1, max_seq_len=None):
        o, rt = _orthrus()
        self.w, self.cache = w, cache
        self.k_pool, self.v_pool = _dev(cache["k_pool"]), _dev(cache["v_pool"])
        self.page_table, self.seq_lens = _dev(cache["page_table"]), _dev(cache["seq_lens"])
        msl = max_seq_len if max_seq_len is not None else int(cache["seq_lens"].max()) if w.batch else 0
        pool = cache["k_pool"]
        self.step = rt.DecodeStep(batch=w.batch, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                                  head_dim=w.head_dim, block_k=w.block_k, page_size=w.page_size,
                                  max_pages_per_seq=cache["page_table"].shape[1], max_seq_len=msl,
                                  num_pages=pool.shape[-4], vocab=vocab, num_layers=num_layers,
                                  num_splits=num_splits)

    def attn(self, view, blk, want_lse=True):
        _, rt = _orthrus()
        w = self.w
        q, kb, vb = _dev(blk["q"]), _dev(blk["k_blk"]), _dev(blk["v_blk"])
        out = torch.full((w.batch, w.block_k, w.num_q_heads, w.head_dim), 0x7FC0, dtype=torch.int16, device="cuda")
        lse = torch.full((w.batch, w.num_q_heads, w.block_k), float("nan"), device="cuda") if want_lse else None
        self.step.attn(view, q, kb, vb, self.k_pool, self.v_pool, self.page_table, self.seq_lens, out, lse)
        torch.cuda.synchronize()
        o = bf16_bits_to_f32(rt.bits_to_numpy(out)).astype(np.float64)
        return (o, lse.cpu().numpy().astype(np.float64)) if want_lse else o


def _check_attn(got, want, what=""):
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS, "%s max-abs %.4g" % (what, err.max())
    assert err.mean() <= MEAN_ABS, "%s mean-abs %.4g" % (what, err.mean())
    if got.ndim == 4:   # [B, K, H_q, d]
        num = np.sqrt((err ** 2).sum(axis=(1, 3)))
        den = np.sqrt((want ** 2).sum(axis=(1, 3)))
        rel = num / np.maximum(den, 1e-30)
        assert rel.max() <= REL_L2, "%s relative L2 error %.4g at (sequence, head) %s" % (
            what, rel.max(), np.unravel_index(np.argmax(rel), rel.shape))


def _oracle_attn(view, w, blk, cache, want_lse=False, seq_lens=None):
    return oracle.dual_view_attn(view, w.sm_scale, blk["q"], blk["k_blk"], blk["v_blk"], cache["k_pool"],
                                 cache["v_pool"], cache["page_table"],
                                 cache["seq_lens"] if seq_lens is None else seq_lens, want_lse=want_lse)


# --------------------------------------------------------------------------------------------- attention

@pytest.mark.parametrize("view", [DIFF, AR])
def test_tiny_config_attention(view):
    w = WORKLOADS["tiny"]
    cache = make_cache(w)
    blk = make_block(w, w.seed + 1)
    case = GpuCase(w, cache)
    got, lse = case.attn(view, blk)
    want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
    _check_attn(got, want, "tiny")
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)


def test_attention_kernel_timing_hooks():
    """Timing attaches events to the launches and changes no result; counts follow the launch plan."""
    w = Workload(name="tm", seed=77, batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=16,
                 context_range=(300, 700), page_size=16, paging="shuffled")
    cache = make_cache(w)
    blk = make_block(w, 78)
    for splits in (1, 3):
        case = GpuCase(w, cache, num_splits=splits)
        plain = case.attn(AR, blk, want_lse=False)
        assert case.step.attn_timing_read() == (0.0, 0, 0.0, 0)
        case.step.attn_timing(True)
        timed = [case.attn(AR, blk, want_lse=False) for _ in range(3)]
        case.step.attn_timing(False)
        untimed = case.attn(AR, blk, want_lse=False)
        split_us, split_n, comb_us, comb_n = case.step.attn_timing_read()
        assert split_n == 3 and comb_n == (3 if splits > 1 else 0)
        assert 0.0 < split_us < 3e4 and (comb_us > 0.0) == (splits > 1)
        assert case.step.attn_timing_read() == (0.0, 0, 0.0, 0)
        for t in timed + [untimed]:
            np.testing.assert_array_equal(t, plain)


SMALL = [
    # several tiles and ragged tails, every row-block variant, both head sizes, odd group sizes
    dict(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=64, block_k=4, context_range=(0, 200), page_size=16),
    dict(batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=16, context_range=(1, 700), page_size=16),
    dict(batch=2, num_q_heads=8, num_kv_heads=8, head_dim=128, block_k=1, context_range=(30, 300), page_size=16),
    dict(batch=2, num_q_heads=14, num_kv_heads=2, head_dim=128, block_k=32, context_range=(100, 900), page_size=16,
         paging="scattered"),
    dict(batch=2, num_q_heads=6, num_kv_heads=2, head_dim=64, block_k=32, context_range=(17, 400), page_size=32),
    dict(batch=1, num_q_heads=16, num_kv_heads=2, head_dim=64, block_k=32, context=333, page_size=64),
    dict(batch=4, num_q_heads=3, num_kv_heads=1, head_dim=128, block_k=5, context_range=(0, 130), page_size=16),
    dict(batch=1, num_q_heads=5, num_kv_heads=5, head_dim=128, block_k=7, context=1025, page_size=16),
    # five and six 32-row blocks per KV head
    dict(batch=2, num_q_heads=5, num_kv_heads=1, head_dim=128, block_k=32, context_range=(40, 500), page_size=16),
    dict(batch=2, num_q_heads=12, num_kv_heads=2, head_dim=64, block_k=31, context_range=(0, 300), page_size=16),
    # four 32-row blocks per KV head: the 8B head ratio at the paper's block size K = 32 (Section 4.1)
    dict(batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=32, context_range=(0, 300), page_size=16),
]


@pytest.mark.parametrize("splits", [0, 1, 3, -1])  # -1: the balanced partition
@pytest.mark.parametrize("shape", range(len(SMALL)))
def test_small_shapes_attention(shape, splits):
    kw = dict(name="s%d" % shape, seed=300 + shape, paging="shuffled")
    kw.update(SMALL[shape])
    w = Workload(**kw)
    cache = make_cache(w)
    case = GpuCase(w, cache, num_splits=splits)
    for view in (DIFF, AR):
        blk = make_block(w, w.seed + 10 + view)
        got, lse = case.attn(view, blk)
        want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
        _check_attn(got, want, "shape %d view %d splits %d" % (shape, view, splits))
        np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)


@pytest.mark.parametrize("L", [0, 1, 15, 16, 31, 32, 33, 127, 128, 129])
def test_edge_lengths(L):
    w = Workload(name="edge", batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=8, context=L,
                 page_size=16, seed=40 + L)
    cache = make_cache(w, seq_lens=np.array([L, max(0, L - 1)], np.int32))
    for splits in (0, -1):
        case = GpuCase(w, cache, max_seq_len=max(L, 1), num_splits=splits)
        for view in (DIFF, AR):
            blk = make_block(w, 500 + L + view)
            got = case.attn(view, blk, want_lse=False)
            _check_attn(got, _oracle_attn(view, w, blk, cache), "L=%d view %d splits %d" % (L, view, splits))


@pytest.mark.parametrize("splits", [0, -1])
@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 6, 7, 8])
def test_mask_decides_at_short_contexts(group, splits):
    """Every compute-wave count (R = 32 * group rows per KV head -> group waves) with caches of 0, 1, 31 and
    33 tokens: the in-block keys carry most or all of the softmax weight, so the view's mask (all K in-block
    keys for the diffusion view, keys 0..i for the AR view, Section 3.2) decides the output."""
    w = Workload(name="mask%d" % group, batch=4, num_q_heads=2 * group, num_kv_heads=2, head_dim=128, block_k=32,
                 context=33, page_size=16, seed=600 + group)
    cache = make_cache(w, seq_lens=np.array([0, 1, 31, 33], np.int32))
    case = GpuCase(w, cache, max_seq_len=33, num_splits=splits)
    outs = {}
    for view in (DIFF, AR):
        blk = make_block(w, 700 + group)          # the same block for both views: only the mask differs
        got, lse = case.attn(view, blk)
        want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
        _check_attn(got, want, "group %d view %d splits %d" % (group, view, splits))
        np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)
        outs[view] = got
    # the views agree on the last block row (it sees every in-block key in both) and differ on row 0
    assert np.abs(outs[DIFF][:, -1] - outs[AR][:, -1]).max() <= MAX_ABS
    assert np.abs(outs[DIFF][:, 0] - outs[AR][:, 0]).max() > 0.1
    # AR row 0 of the empty-cache sequence sees one key, its own: the output is that value row, exactly
    blk = make_block(w, 700 + group)
    v0 = bf16_bits_to_f32(blk["v_blk"][0, 0]).astype(np.float64)           # [H_kv, d]
    np.testing.assert_array_equal(outs[AR][0, 0], np.repeat(v0, group, axis=0))


@pytest.mark.parametrize("splits", [0, 3, 7, -1])
def test_loose_host_bound_on_the_lengths(splits):
    """max_seq_len far above the real lengths (a decode loop that bumps its bound by K per step without reading
    the lengths back): the grid is sized by the bound, the cuts by each sequence's own length."""
    w = Workload(name="loose", batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=16, context=700,
                 page_size=16, seed=88, steps=220)          # pages mapped far beyond the lengths
    cache = make_cache(w, seq_lens=np.array([300, 700, 33], np.int32))
    case = GpuCase(w, cache, num_splits=splits, max_seq_len=4096)
    for view in (DIFF, AR):
        blk = make_block(w, 89 + view)
        got, lse = case.attn(view, blk)
        want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
        _check_attn(got, want, "loose bound view %d splits %d" % (view, splits))
        np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)


def test_kv_stream_probe_and_timing_samples():
    """The measurement helpers: the stream probe launches, reports no error and writes nothing; timing
    samples come back one per timed call, in launch order, with a combine time only when there was one."""
    w = Workload(name="probe", batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=16,
                 context_range=(300, 700), page_size=16, paging="shuffled", seed=91)
    cache = make_cache(w)
    blk = make_block(w, 92)
    _, rt = _orthrus()
    for splits in (1, 3, -1):
        case = GpuCase(w, cache, num_splits=splits)
        before = (rt.bits_to_numpy(case.k_pool).copy(), rt.bits_to_numpy(case.v_pool).copy())
        plain = case.attn(AR, blk, want_lse=False)
        case.step.attn_timing(True)
        case.step.kv_stream_probe(case.k_pool, case.v_pool, case.page_table, case.seq_lens)
        timed = case.attn(AR, blk, want_lse=False)
        case.step.kv_stream_probe(case.k_pool, case.v_pool, case.page_table, case.seq_lens)
        case.step.attn_timing(False)
        torch.cuda.synchronize()
        samples = case.step.attn_timing_samples()
        assert len(samples) == 3
        assert all(0.0 < s[0] < 3e4 for s in samples)
        assert samples[0][1] == 0.0 and samples[2][1] == 0.0           # the probe has no combine kernel
        assert (samples[1][1] > 0.0) == (splits != 1)
        assert case.step.attn_timing_samples() == []
        assert case.step.device_error() == 0
        np.testing.assert_array_equal(timed, plain)
        np.testing.assert_array_equal(rt.bits_to_numpy(case.k_pool), before[0])
        np.testing.assert_array_equal(rt.bits_to_numpy(case.v_pool), before[1])


def test_split_count_invariance_and_determinism():
    w = Workload(name="inv", batch=2, num_q_heads=16, num_kv_heads=4, head_dim=128, block_k=16,
                 context_range=(1500, 2100), page_size=16, seed=77)
    cache = make_cache(w)
    blk = make_block(w, 78)
    want = _oracle_attn(AR, w, blk, cache)
    outs = {}
    for s in (1, 2, 7, 12, 24, 64, -1):  # the merge kernel has forms for <= 8, <= 16 and more pieces
        case = GpuCase(w, cache, num_splits=s)
        outs[s] = case.attn(AR, blk, want_lse=False)
        _check_attn(outs[s], want, "splits %d" % s)
        again = case.attn(AR, blk, want_lse=False)
        np.testing.assert_array_equal(again, outs[s])            # run-to-run bit identical
    assert np.abs(outs[1] - outs[64]).max() <= 1e-2


def test_layer8b_config_attention_full():
    w = WORKLOADS["layer8b"]
    cache = make_cache(w)
    case = GpuCase(w, cache)
    for view in (DIFF, AR):
        blk = make_block(w, w.seed * 1000 + 1 + view)
        got, lse = case.attn(view, blk)
        want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
        _check_attn(got, want, "layer8b view %d" % view)
        np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)


def _sub_batch(blk, cache, idx):
    """Inputs of the sequences `idx` only (same pools), for running the oracle on a sample."""
    idx = np.asarray(idx)
    b = {k: np.ascontiguousarray(v[idx]) for k, v in blk.items()}
    c = dict(cache)
    c["page_table"] = np.ascontiguousarray(cache["page_table"][idx])
    c["seq_lens"] = np.ascontiguousarray(cache["seq_lens"][idx])
    return b, c


@pytest.mark.parametrize("splits", [0, -1])
def test_mixed_config_attention_sampled_sequences(splits):
    """Full-size batched mixed-length run; the oracle recomputes the shortest, the longest and one more sequence."""
    w = WORKLOADS["mixed"]
    cache = make_cache(w)
    case = GpuCase(w, cache, num_splits=splits)
    lens = cache["seq_lens"]
    pick = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 5})
    for view in (DIFF, AR):
        blk = make_block(w, w.seed * 1000 + 1 + view)
        got = case.attn(view, blk, want_lse=False)
        assert np.all(np.isfinite(got))
        sb, sc = _sub_batch(blk, cache, pick)
        want = _oracle_attn(view, w, sb, sc)
        _check_attn(got[pick], want, "mixed view %d" % view)


@pytest.mark.parametrize("splits", [64, 0])
def test_long_config_attention_sampled_head(splits):
    """Context 32768 at full size; the oracle recomputes one (sequence, KV head) group of rows."""
    w = WORKLOADS["long"].with_(num_splits=splits)
    cache = make_cache(w)
    case = GpuCase(w, cache, num_splits=splits)
    b, g, G = 2, 5, w.group
    for view in (DIFF, AR):
        blk = make_block(w, w.seed * 1000 + 1 + view)
        got = case.attn(view, blk, want_lse=False)
        assert np.all(np.isfinite(got))
        w1 = w.with_(batch=1, num_q_heads=G, num_kv_heads=1)
        sb = dict(q=np.ascontiguousarray(blk["q"][b:b + 1, :, g * G:(g + 1) * G]),
                  k_blk=np.ascontiguousarray(blk["k_blk"][b:b + 1, :, g:g + 1]),
                  v_blk=np.ascontiguousarray(blk["v_blk"][b:b + 1, :, g:g + 1]))
        sc = dict(k_pool=np.ascontiguousarray(cache["k_pool"][:, g:g + 1]),
                  v_pool=np.ascontiguousarray(cache["v_pool"][:, g:g + 1]),
                  page_table=np.ascontiguousarray(cache["page_table"][b:b + 1]),
                  seq_lens=np.ascontiguousarray(cache["seq_lens"][b:b + 1]))
        want = _oracle_attn(view, w1, sb, sc)
        _check_attn(got[b:b + 1, :, g * G:(g + 1) * G], want, "long view %d splits %d" % (view, splits))


@pytest.mark.parametrize("splits", [64, 0])
def test_long_config_every_piece_carries_a_dominant_key(splits):
    """Context 32768 at full size with planted structure: inside two (sequence, KV head) units every one of
    the 64 prescribed splits holds one cached key that one query row scores far above everything else, and
    so do two in-block positions (one visible to both views, one that the AR view's causal mask hides).  The
    output of such a row is, to rounding, the value row stored with its key, so a lost split, a lost tile
    or a wrong in-block mask shows as an error of order one instead of hiding inside the tolerance."""
    w = WORKLOADS["long"].with_(num_splits=splits)
    cache = make_cache(w)
    blk = make_block(w, w.seed * 1000 + 7)
    G, K, P, L = w.group, w.block_k, w.page_size, w.context
    chunk = L // 64
    qf = bf16_bits_to_f32(blk["q"])
    units = [(2, 5), (0, 1)]
    in_block = {}          # unit index -> [(row i, head offset, in-block position)]
    for u, (b, g) in enumerate(units):
        rows = [(i, hl) for i in range(K) for hl in range(G)]            # 64 rows of the unit
        if u == 1:
            in_block[u] = [(9, 1, 2), (5, 3, K - 1)]                    # position 2 <= row 9; position K-1 > row 5
            rows = [r for r in rows if r not in [(9, 1), (5, 3)]]
        for s, (i, hl) in enumerate(rows):
            pos = s * chunk + (37 * s + 11 * u) % chunk                  # somewhere inside split s
            key = f32_to_bf16_bits(2.0 * qf[b, i, g * G + hl])           # score ~ 2 |q|^2 / sqrt(d) ~ 22
            cache["k_pool"][cache["page_table"][b, pos // P], g, pos % P] = key
        for i, hl, r in in_block.get(u, []):
            blk["k_blk"][b, r, g] = f32_to_bf16_bits(2.0 * qf[b, i, g * G + hl])
    case = GpuCase(w, cache, num_splits=splits)
    for view in (DIFF, AR):
        got = case.attn(view, blk, want_lse=False)
        assert np.all(np.isfinite(got))
        for u, (b, g) in enumerate(units):
            w1 = w.with_(batch=1, num_q_heads=G, num_kv_heads=1)
            sb = dict(q=np.ascontiguousarray(blk["q"][b:b + 1, :, g * G:(g + 1) * G]),
                      k_blk=np.ascontiguousarray(blk["k_blk"][b:b + 1, :, g:g + 1]),
                      v_blk=np.ascontiguousarray(blk["v_blk"][b:b + 1, :, g:g + 1]))
            sc = dict(k_pool=np.ascontiguousarray(cache["k_pool"][:, g:g + 1]),
                      v_pool=np.ascontiguousarray(cache["v_pool"][:, g:g + 1]),
                      page_table=np.ascontiguousarray(cache["page_table"][b:b + 1]),
                      seq_lens=np.ascontiguousarray(cache["seq_lens"][b:b + 1]))
            want = _oracle_attn(view, w1, sb, sc)
            mine = got[b:b + 1, :, g * G:(g + 1) * G]
            _check_attn(mine, want, "planted long view %d splits %d unit %d" % (view, splits, u))
            # the structure is really there: the planted rows reproduce single value rows (order one),
            # far from the ~0.01 of an average over 32768 random values
            dominated = np.ones((K, G), bool)
            if u == 1 and view == AR:
                dominated[5, 3] = False                                   # its planted key is masked out
            assert np.abs(want[0]).max(axis=2)[dominated].min() > 0.5
        # the hidden in-block key: row 5 / head 3 of unit 1 is dominated by it under the diffusion view only
        b, g = units[1]
        v_hidden = bf16_bits_to_f32(blk["v_blk"][b, K - 1, g]).astype(np.float64)
        near = np.abs(got[b, 5, g * G + 3] - v_hidden).max()
        assert (near < 2e-2) if view == DIFF else (near > 0.5)


@pytest.mark.parametrize("splits", [0, -1])
def test_bad_page_is_flagged_not_dereferenced(splits):
    w = Workload(name="badpg", batch=2, num_q_heads=4, num_kv_heads=2, head_dim=128, block_k=4, context=100,
                 page_size=16, seed=9)
    cache = make_cache(w)
    cache["page_table"][1, 2] = 10 ** 6
    cache["page_table"][1, 3] = -1
    case = GpuCase(w, cache, num_splits=splits)
    blk = make_block(w, 10)
    got = case.attn(AR, blk, want_lse=False)
    assert case.step.device_error() == -4
    assert case.step.device_error() == 0                      # reading clears the flag
    sb, sc = _sub_batch(blk, cache, [0])
    _check_attn(got[:1], _oracle_attn(AR, w, sb, sc), "unaffected sequence")


@pytest.mark.parametrize("splits", [0, 3, -1])
def test_length_beyond_the_host_bound_is_flagged_and_clamped(splits):
    """seq_lens[b] outside [0, max_seq_len]: the error word is set, the length is clamped (no read past the
    mapped pages), and the other sequences are unaffected."""
    w = Workload(name="badlen", batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=8, context=200,
                 page_size=16, seed=19)
    cache = make_cache(w, seq_lens=np.array([200, 200, 90], np.int32))   # pages mapped for the clamped lengths
    case = GpuCase(w, cache, num_splits=splits, max_seq_len=200)
    case.seq_lens.copy_(_dev(np.array([200, 100000, -5], np.int32)))
    blk = make_block(w, 20)
    got = case.attn(DIFF, blk, want_lse=False)
    assert case.step.device_error() == -4
    assert np.all(np.isfinite(got))
    sb, sc = _sub_batch(blk, cache, [0])
    _check_attn(got[:1], _oracle_attn(DIFF, w, sb, sc), "unaffected sequence")
    # the clamped sequences behave as lengths 200 and 0
    clamped = dict(cache, seq_lens=np.array([200, 200, 0], np.int32))
    _check_attn(got, _oracle_attn(DIFF, w, blk, clamped), "clamped lengths")


# --------------------------------------------------------------------------------------------- consensus

def _run_consensus(case, logits, draft, blk=None, layers=1):
    w = case.w
    B, K = w.batch, w.block_k
    dl, dd = _dev(logits), _dev(draft)
    outs = [torch.full((B,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
    toks = torch.full((B, K), -7, dtype=torch.int32, device="cuda")
    kb = vb = None
    if blk is not None:
        kb, vb = _dev(blk["k_blk"]), _dev(blk["v_blk"])
    case.step.consensus_commit(dl, dd, kb, vb, case.k_pool if blk is not None else None,
                               case.v_pool if blk is not None else None,
                               case.page_table if blk is not None else None,
                               case.seq_lens if blk is not None else None, outs[0], outs[1], toks, outs[2])
    torch.cuda.synchronize()
    return dict(accept_len=outs[0].cpu().numpy(), num_committed=outs[1].cpu().numpy(),
                out_tokens=toks.cpu().numpy(), next_anchor=outs[2].cpu().numpy())


def _same_consensus(got, want):
    for key in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
        np.testing.assert_array_equal(got[key], want[key], err_msg=key)


@pytest.mark.parametrize("vocab", [512, 97, 8191, 8192, 8193, 40001, 128256])
def test_consensus_only_matches_oracle(vocab):
    w = WORKLOADS["tiny"].with_(batch=5, block_k=7, vocab=vocab, accept="uniform")
    cache = make_cache(w)
    case = GpuCase(w, cache, vocab=vocab)
    cc = make_consensus_case(w, seed=vocab)
    got = _run_consensus(case, cc["ar_logits"], cc["draft_tokens"])
    want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"])
    _same_consensus(got, want)
    np.testing.assert_array_equal(got["accept_len"], cc["planted_n_acc"])


def test_consensus_special_values():
    rng = np.random.default_rng(0)
    B, K, V = 3, 6, 20000
    logits = rng.integers(-2, 3, size=(B, K, V)).astype(np.float32)          # massive ties
    logits[0, 1, :] = -np.inf
    logits[0, 2, 17000] = np.nan; logits[0, 2, 9000] = np.nan; logits[0, 2, 5] = 1e30
    logits[1, 0, :] = 0.0; logits[1, 0, 0] = -0.0
    logits[1, 3, V - 1] = 99.0
    logits[2, 4, 8191] = 50.0; logits[2, 4, 8192] = 50.0
    ref_free = oracle.consensus_commit(logits, np.zeros((B, K), np.int32))
    am = np.where(ref_free["out_tokens"] >= 0, ref_free["out_tokens"], 0)
    # build drafts that accept everything, by asking the oracle row by row
    draft = np.zeros((B, K), np.int32)
    for k in range(K):
        r = oracle.consensus_commit(logits, draft)
        draft[:, k] = [r["out_tokens"][b, k] if r["out_tokens"][b, k] >= 0 else 0 for b in range(B)]
    w = WORKLOADS["tiny"].with_(batch=B, block_k=K, vocab=V)
    case = GpuCase(w, make_cache(w), vocab=V)
    for d in (draft, np.zeros((B, K), np.int32), np.full((B, K), -3, np.int32), np.full((B, K), V, np.int32)):
        got = _run_consensus(case, logits, d)
        _same_consensus(got, oracle.consensus_commit(logits, d))
    full = _run_consensus(case, logits, draft)
    assert np.all(full["accept_len"] == K)
    assert full["out_tokens"][0, 1] == 0 and full["out_tokens"][0, 2] == 9000
    assert full["out_tokens"][1, 0] == 0 and full["out_tokens"][1, 3] == V - 1 and full["out_tokens"][2, 4] == 8191


def _gathered_equal(case, ref_cache):
    """Logical cache contents [0, seq_len) and lengths must match the oracle's bit for bit."""
    _, rt = _orthrus()
    kp, vp = rt.bits_to_numpy(case.k_pool), rt.bits_to_numpy(case.v_pool)
    lens = case.seq_lens.cpu().numpy()
    np.testing.assert_array_equal(lens, ref_cache["seq_lens"])
    # appended rows are the only writes, so whole-pool equality is the O(1)-overhead check as well
    np.testing.assert_array_equal(kp, ref_cache["k_pool"])
    np.testing.assert_array_equal(vp, ref_cache["v_pool"])


def test_tiny_config_consensus_and_commit_loop():
    w = WORKLOADS["tiny"].with_(steps=6)
    cache = make_cache(w)
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in cache.items()}
    case = GpuCase(w, cache, vocab=w.vocab, max_seq_len=w.capacity_tokens())
    for step in range(w.steps):
        cc = make_consensus_case(w, seed=900 + step)
        blk = make_block(w, 950 + step)
        got = _run_consensus(case, cc["ar_logits"], cc["draft_tokens"], blk)
        want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"], blk["k_blk"], blk["v_blk"],
                                       ref["k_pool"], ref["v_pool"], ref["page_table"], ref["seq_lens"])
        _same_consensus(got, want)
        _gathered_equal(case, ref)
        # attention over the grown cache still matches
        ablk = make_block(w, 970 + step)
        _check_attn(case.attn(AR, ablk, want_lse=False), _oracle_attn(AR, w, ablk, ref), "after step %d" % step)


def test_multi_layer_commit_and_strided_pool():
    w = Workload(name="ml", batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=8,
                 context_range=(0, 90), page_size=16, vocab=3000, accept="uniform", steps=2, seed=21)
    layers = 3
    lens = np.array([0, 37, 90], np.int32)
    caches = [make_cache(w, seed=21 + l, seq_lens=lens) for l in range(layers)]
    # all layers share one page table / lengths (first layer's); with equal lengths the pools have equal shapes
    kp = np.stack([c["k_pool"] for c in caches]); vp = np.stack([c["v_pool"] for c in caches])
    o, rt = _orthrus()
    cache = dict(caches[0]); cache["k_pool"] = kp; cache["v_pool"] = vp
    case = GpuCase(w, cache, vocab=w.vocab, num_layers=layers, max_seq_len=w.capacity_tokens())
    ref_k, ref_v, ref_len = kp.copy(), vp.copy(), cache["seq_lens"].copy()
    for step in range(2):
        cc = make_consensus_case(w, seed=60 + step)
        blks = [make_block(w, 70 + 10 * step + l) for l in range(layers)]
        blk = dict(k_blk=np.stack([b["k_blk"] for b in blks]), v_blk=np.stack([b["v_blk"] for b in blks]))
        got = _run_consensus(case, cc["ar_logits"], cc["draft_tokens"], blk)
        want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"], blk["k_blk"], blk["v_blk"], ref_k, ref_v,
                                       cache["page_table"], ref_len)
        _same_consensus(got, want)
        np.testing.assert_array_equal(rt.bits_to_numpy(case.k_pool), ref_k)
        np.testing.assert_array_equal(rt.bits_to_numpy(case.v_pool), ref_v)
        np.testing.assert_array_equal(case.seq_lens.cpu().numpy(), ref_len)


def test_commit_capacity_error_is_flagged_and_sequence_untouched():
    w = Workload(name="cap", batch=3, num_q_heads=4, num_kv_heads=2, head_dim=64, block_k=8, context=28,
                 page_size=16, vocab=600, seed=31)
    cache = make_cache(w)
    cache["page_table"][1, 2:] = -1            # sequence 1 cannot grow past 32 tokens
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in cache.items()}
    case = GpuCase(w, cache, vocab=w.vocab, max_seq_len=28 + 8)
    cc = make_consensus_case(w, seed=32, n_acc=np.array([8, 8, 2], np.int32))
    blk = make_block(w, 33)
    got = _run_consensus(case, cc["ar_logits"], cc["draft_tokens"], blk)
    want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"], blk["k_blk"], blk["v_blk"], ref["k_pool"],
                                   ref["v_pool"], ref["page_table"], ref["seq_lens"], allow_capacity_error=True)
    assert want["status"] == -4
    _same_consensus(got, want)
    assert got["num_committed"].tolist() == [8, 0, 3]
    _gathered_equal(case, ref)
    assert case.step.device_error() == -4


def test_layer8b_config_consensus_commit():
    w = WORKLOADS["layer8b"]
    cache = make_cache(w)
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in cache.items()}
    case = GpuCase(w, cache, vocab=w.vocab, max_seq_len=w.capacity_tokens())
    for step in range(3):
        cc = make_consensus_case(w, seed=w.seed * 1000 + 3 + 10 * step)
        blk = make_block(w, w.seed * 1000 + 2 + 10 * step)
        got = _run_consensus(case, cc["ar_logits"], cc["draft_tokens"], blk)
        want = oracle.consensus_commit(cc["ar_logits"], cc["draft_tokens"], blk["k_blk"], blk["v_blk"], ref["k_pool"],
                                       ref["v_pool"], ref["page_table"], ref["seq_lens"])
        _same_consensus(got, want)
        np.testing.assert_array_equal(got["accept_len"], cc["planted_n_acc"])
    _gathered_equal(case, ref)


def test_stress_config_looped_steps():
    """Batch 64, vocab 151936, 32 looped steps of draft attention + verify attention + consensus + commit.

    Four distinct logits/draft sets are cycled over the steps (one 622 MB logits tensor each); block K/V are
    fresh per step.  Consensus outputs, lengths and the whole pool are compared with the oracle after every
    step; attention is compared at the first and last step on sampled sequences.
    """
    w = WORKLOADS["stress"]
    cache = make_cache(w)
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in cache.items()}
    case = GpuCase(w, cache, vocab=w.vocab, max_seq_len=w.capacity_tokens())
    _, rt = _orthrus()
    sets = [make_consensus_case(w, seed=w.seed * 1000 + 3 + 10 * i) for i in range(4)]
    dev_sets = [(_dev(s["ar_logits"]), _dev(s["draft_tokens"])) for s in sets]
    B, K = w.batch, w.block_k
    outs = [torch.empty((B,), dtype=torch.int32, device="cuda") for _ in range(3)]
    toks = torch.empty((B, K), dtype=torch.int32, device="cuda")
    o_d = torch.empty((B, K, w.num_q_heads, w.head_dim), dtype=torch.int16, device="cuda")
    o_a = torch.empty_like(o_d)
    pick = [0, 17, 63]
    for step in range(w.steps):
        dblk = make_block(w, w.seed * 1000 + 1 + 10 * step)
        ablk = make_block(w, w.seed * 1000 + 2 + 10 * step)
        dq, dk, dv = _dev(dblk["q"]), _dev(dblk["k_blk"]), _dev(dblk["v_blk"])
        aq, ak, av = _dev(ablk["q"]), _dev(ablk["k_blk"]), _dev(ablk["v_blk"])
        dl, dd = dev_sets[step % 4]
        # one decode step, queued back to back on the stream without host synchronisation
        case.step.attn(DIFF, dq, dk, dv, case.k_pool, case.v_pool, case.page_table, case.seq_lens, o_d)
        case.step.attn(AR, aq, ak, av, case.k_pool, case.v_pool, case.page_table, case.seq_lens, o_a)
        case.step.consensus_commit(dl, dd, ak, av, case.k_pool, case.v_pool, case.page_table, case.seq_lens,
                                   outs[0], outs[1], toks, outs[2])
        torch.cuda.synchronize()
        if step in (0, w.steps - 1):
            for view, blk, o_t in ((DIFF, dblk, o_d), (AR, ablk, o_a)):
                sb, sc = _sub_batch(blk, ref, pick)
                got = bf16_bits_to_f32(rt.bits_to_numpy(o_t)).astype(np.float64)[pick]
                _check_attn(got, _oracle_attn(view, w, sb, sc), "stress step %d view %d" % (step, view))
        s = sets[step % 4]
        want = oracle.consensus_commit(s["ar_logits"], s["draft_tokens"], ablk["k_blk"], ablk["v_blk"], ref["k_pool"],
                                       ref["v_pool"], ref["page_table"], ref["seq_lens"])
        got = dict(accept_len=outs[0].cpu().numpy(), num_committed=outs[1].cpu().numpy(),
                   out_tokens=toks.cpu().numpy(), next_anchor=outs[2].cpu().numpy())
        _same_consensus(got, want)
        np.testing.assert_array_equal(case.seq_lens.cpu().numpy(), ref["seq_lens"])
    _gathered_equal(case, ref)
    assert case.step.device_error() == 0
    assert int(ref["seq_lens"].sum()) > int(cache["seq_lens"].sum())
