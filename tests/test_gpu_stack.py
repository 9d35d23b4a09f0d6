"""Multi-layer decode cycle (diffusion pass, AR pass, consensus + commit; Section 3.2-3.3, Fig. 2(b)),
eagerly and as a replayed HIP graph, against the CPU oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from orthrus_inputs import Workload, bf16_bits_to_f32, make_block, make_cache, make_consensus_case, make_sampling_case

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3   # attention tolerance of the path (bf16 in, fp32 accumulate)
LAYERS, CYCLES = 3, 4


def _rt():
    from paper_2605_12825_amd import runtime
    return runtime


def _workload():
    return Workload(name="stack", batch=3, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=8,
                    context_range=(0, 90), page_size=16, vocab=2000, accept="uniform", steps=CYCLES, seed=91)


def _initial_state(w):
    lens = np.array([5, 37, 90], np.int32)
    caches = [make_cache(w, seed=91 + l, seq_lens=lens) for l in range(LAYERS)]
    kp = np.stack([c["k_pool"] for c in caches])
    vp = np.stack([c["v_pool"] for c in caches])
    return kp, vp, caches[0]["page_table"].copy(), lens.copy()


def _cycle_inputs(w, c):
    d = [make_block(w, 1000 + 100 * c + l) for l in range(LAYERS)]
    a = [make_block(w, 2000 + 100 * c + l) for l in range(LAYERS)]
    st = lambda blks, k: np.stack([b[k] for b in blks])
    cons = make_consensus_case(w, seed=3000 + c)
    return dict(q_diff=st(d, "q"), k_blk_diff=st(d, "k_blk"), v_blk_diff=st(d, "v_blk"),
                q_ar=st(a, "q"), k_blk_ar=st(a, "k_blk"), v_blk_ar=st(a, "v_blk"),
                ar_logits=cons["ar_logits"], draft_tokens=cons["draft_tokens"])


def _make_stack(w, kp, vp, pt, lens, **kw):
    rt = _rt()
    return rt.DecodeStack(num_layers=LAYERS, batch=w.batch, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                          head_dim=w.head_dim, block_k=w.block_k, page_size=w.page_size,
                          k_pool=rt.to_device_bits(kp), v_pool=rt.to_device_bits(vp),
                          page_table=rt.to_device_bits(pt), seq_lens=rt.to_device_bits(lens),
                          max_seq_len=w.capacity_tokens(), vocab=w.vocab, **kw)


def _upload(stack, inp):
    rt = _rt()
    for k, v in inp.items():
        getattr(stack, k).copy_(rt.to_device_bits(v))


def _snapshot(stack):
    rt = _rt()
    torch.cuda.synchronize()
    names = ("out_diff", "out_ar", "accept_len", "num_committed", "out_tokens", "next_anchor", "k_pool", "v_pool",
             "seq_lens")
    return {n: rt.bits_to_numpy(getattr(stack, n)).copy() for n in names}


def _check_attn(got_bits, want):
    got = bf16_bits_to_f32(got_bits).astype(np.float64)
    err = np.abs(got - want)
    assert np.all(np.isfinite(got)) and err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


@pytest.mark.parametrize("splits", [0, -1])   # the library's fixed splits; the balanced partition
def test_stack_cycle_eager_and_graph_replay_match_oracle(splits):
    w = _workload()
    kp, vp, pt, lens = _initial_state(w)
    ref_k, ref_v, ref_len = kp.copy(), vp.copy(), lens.copy()
    eager = _make_stack(w, kp, vp, pt, lens, num_splits=splits)
    graph = _make_stack(w, kp, vp, pt, lens, num_splits=splits)
    graph.capture()                       # records only: nothing has run, the state is still the initial one
    np.testing.assert_array_equal(graph.seq_lens.cpu().numpy(), lens)
    for c in range(CYCLES):
        inp = _cycle_inputs(w, c)
        # oracle: both passes see the cache as it is before the commit of this cycle
        want_d = np.stack([oracle.dual_view_attn(0, w.sm_scale, inp["q_diff"][l], inp["k_blk_diff"][l],
                                                 inp["v_blk_diff"][l], ref_k[l], ref_v[l], pt, ref_len)
                           for l in range(LAYERS)])
        want_a = np.stack([oracle.dual_view_attn(1, w.sm_scale, inp["q_ar"][l], inp["k_blk_ar"][l],
                                                 inp["v_blk_ar"][l], ref_k[l], ref_v[l], pt, ref_len)
                           for l in range(LAYERS)])
        want_c = oracle.consensus_commit(inp["ar_logits"], inp["draft_tokens"], inp["k_blk_ar"], inp["v_blk_ar"],
                                         ref_k, ref_v, pt, ref_len)
        _upload(eager, inp)
        eager.cycle()
        e = _snapshot(eager)
        # the program's own eager work and a synchronisation sit between the replays
        _upload(graph, inp)
        torch.cuda.synchronize()
        graph.replay()
        graph.graph_stream.synchronize()
        g = _snapshot(graph)
        for snap in (e, g):
            _check_attn(snap["out_diff"], want_d)
            _check_attn(snap["out_ar"], want_a)
            for n in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
                np.testing.assert_array_equal(snap[n], want_c[n], err_msg="%s cycle %d" % (n, c))
            np.testing.assert_array_equal(snap["k_pool"], ref_k)
            np.testing.assert_array_equal(snap["v_pool"], ref_v)
            np.testing.assert_array_equal(snap["seq_lens"], ref_len)
        for n in e:                      # same kernels, same inputs: the replay is bit-identical to eager
            np.testing.assert_array_equal(e[n], g[n], err_msg="%s cycle %d" % (n, c))
    assert ref_len.sum() > lens.sum()
    assert eager.step.device_error() == 0 and graph.step.device_error() == 0
    eager.close()
    graph.close()


SAMPLING_MARGIN = 2e-3   # decisions closer than this (log domain) to flipping are not compared: fp32 vs fp64


def _clear_sampling_case(w, seed0, temperature):
    """A seeded sampling case whose every accept / draw decision is clear of fp32 rounding (the oracle says)."""
    for seed in range(seed0, seed0 + 50):
        sc = make_sampling_case(w, seed=seed, temperature=temperature)
        r = oracle.sampling_consensus_commit(sc["ar_logits"], sc["diff_logits"], sc["draft_tokens"], sc["accept_u"],
                                             sc["gumbel"], temperature)
        ma, md = r["margin_accept"], r["margin_draw"]
        if np.all(ma[ma >= 0] > SAMPLING_MARGIN) and np.all(md[md >= 0] > SAMPLING_MARGIN):
            return sc
    raise AssertionError("no seed with clear margins")


def test_stack_sampling_cycle_eager_and_graph_replay_match_oracle():
    w = _workload()
    kp, vp, pt, lens = _initial_state(w)
    ref_k, ref_v, ref_len = kp.copy(), vp.copy(), lens.copy()
    eager = _make_stack(w, kp, vp, pt, lens, temperature=0.8)
    graph = _make_stack(w, kp, vp, pt, lens, temperature=0.8)
    graph.capture()
    for c in range(3):
        inp = _cycle_inputs(w, c)
        sc = _clear_sampling_case(w, 4000 + 100 * c, 0.8)
        for k in ("ar_logits", "diff_logits", "draft_tokens", "accept_u", "gumbel"):
            inp[k] = sc[k]
        want_d = np.stack([oracle.dual_view_attn(0, w.sm_scale, inp["q_diff"][l], inp["k_blk_diff"][l],
                                                 inp["v_blk_diff"][l], ref_k[l], ref_v[l], pt, ref_len)
                           for l in range(LAYERS)])
        want_a = np.stack([oracle.dual_view_attn(1, w.sm_scale, inp["q_ar"][l], inp["k_blk_ar"][l],
                                                 inp["v_blk_ar"][l], ref_k[l], ref_v[l], pt, ref_len)
                           for l in range(LAYERS)])
        want_c = oracle.sampling_consensus_commit(sc["ar_logits"], sc["diff_logits"], sc["draft_tokens"],
                                                  sc["accept_u"], sc["gumbel"], 0.8, inp["k_blk_ar"], inp["v_blk_ar"],
                                                  ref_k, ref_v, pt, ref_len)
        _upload(eager, inp)
        eager.cycle()
        e = _snapshot(eager)
        _upload(graph, inp)
        torch.cuda.synchronize()
        graph.replay()
        graph.graph_stream.synchronize()
        g = _snapshot(graph)
        for snap in (e, g):
            _check_attn(snap["out_diff"], want_d)
            _check_attn(snap["out_ar"], want_a)
            for n in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
                np.testing.assert_array_equal(snap[n], want_c[n], err_msg="%s cycle %d" % (n, c))
            np.testing.assert_array_equal(snap["k_pool"], ref_k)
            np.testing.assert_array_equal(snap["v_pool"], ref_v)
            np.testing.assert_array_equal(snap["seq_lens"], ref_len)
        for n in e:
            np.testing.assert_array_equal(e[n], g[n], err_msg="%s cycle %d" % (n, c))
        assert (e["num_committed"] >= 1).all()
    eager.close()
    graph.close()


def test_two_diffusion_passes_per_cycle_match_oracle():
    """The multi-step variant of the paper's ablation (Section 5, Table 3) runs the diffusion view twice per cycle;
    over unchanged inputs the second pass reproduces the first, so the cycle's results are the oracle's for one
    pass: eagerly and in a replayed graph, and identical to the one-pass stack."""
    w = _workload()
    kp, vp, pt, lens = _initial_state(w)
    ref_k, ref_v, ref_len = kp.copy(), vp.copy(), lens.copy()
    one = _make_stack(w, kp, vp, pt, lens)
    two = _make_stack(w, kp, vp, pt, lens, diffusion_passes=2)
    two_g = _make_stack(w, kp, vp, pt, lens, diffusion_passes=2)
    two_g.capture()
    for c in range(2):
        inp = _cycle_inputs(w, c)
        want_d = np.stack([oracle.dual_view_attn(0, w.sm_scale, inp["q_diff"][l], inp["k_blk_diff"][l],
                                                 inp["v_blk_diff"][l], ref_k[l], ref_v[l], pt, ref_len)
                           for l in range(LAYERS)])
        want_a = np.stack([oracle.dual_view_attn(1, w.sm_scale, inp["q_ar"][l], inp["k_blk_ar"][l],
                                                 inp["v_blk_ar"][l], ref_k[l], ref_v[l], pt, ref_len)
                           for l in range(LAYERS)])
        want_c = oracle.consensus_commit(inp["ar_logits"], inp["draft_tokens"], inp["k_blk_ar"], inp["v_blk_ar"],
                                         ref_k, ref_v, pt, ref_len)
        snaps = []
        for st in (one, two):
            _upload(st, inp)
            st.cycle()
            snaps.append(_snapshot(st))
        _upload(two_g, inp)
        torch.cuda.synchronize()
        two_g.replay()
        two_g.graph_stream.synchronize()
        snaps.append(_snapshot(two_g))
        for snap in snaps:
            _check_attn(snap["out_diff"], want_d)
            _check_attn(snap["out_ar"], want_a)
            for n in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
                np.testing.assert_array_equal(snap[n], want_c[n], err_msg="%s cycle %d" % (n, c))
            np.testing.assert_array_equal(snap["k_pool"], ref_k)
            np.testing.assert_array_equal(snap["seq_lens"], ref_len)
        for other in snaps[1:]:
            for n in snaps[0]:
                np.testing.assert_array_equal(snaps[0][n], other[n], err_msg="%s cycle %d" % (n, c))
    for st in (one, two, two_g):
        st.close()


def test_graph_begin_rejects_null_stream_and_timing():
    from paper_2605_12825_amd import binding as B
    w = _workload()
    kp, vp, pt, lens = _initial_state(w)
    stack = _make_stack(w, kp, vp, pt, lens)
    with pytest.raises(B.OrthrusError):
        B.orthrus_graph_begin(stack.step.ctx, 0)
    stack.step.attn_timing(True)
    with pytest.raises(B.OrthrusError):
        B.orthrus_graph_begin(stack.step.ctx, torch.cuda.Stream())
    stack.step.attn_timing(False)
    stack.close()
