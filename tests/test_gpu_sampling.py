"""GPU parity for the temperature > 0 consensus: HIP path through the C ABI vs the fp64 oracle.

Accept lengths, tokens, lengths and pool bytes must be identical.  The oracle decides in fp64, the
kernels in fp32, so every compared case is first checked to have decision margins far above fp32
rounding of a log-sum-exp over the vocabulary (the oracle reports the margins); a seeded case that
does not is replaced by the next seed, which keeps the test deterministic.
"""
import numpy as np
import pytest
import torch

import oracle
from orthrus_inputs import WORKLOADS, Workload, make_block, make_cache, make_sampling_case

pytestmark = pytest.mark.gpu

MARGIN = 2e-3   # log-domain distance of every decision from flipping


def _rt():
    from paper_2605_12825_amd import runtime
    return runtime


def _clear_case(w, seed0, **kw):
    for seed in range(seed0, seed0 + 50):
        c = make_sampling_case(w, seed=seed, **kw)
        r = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                             c["gumbel"], c["temperature"])
        ma = r["margin_accept"]
        examined = ma >= 0
        in_range = (c["draft_tokens"] >= 0) & (c["draft_tokens"] < c["ar_logits"].shape[2])
        ok_acc = np.all(ma[examined & in_range] > MARGIN)
        md = r["margin_draw"]
        ok_draw = np.all(md[md >= 0] > MARGIN)
        if ok_acc and ok_draw:
            return c, seed
    raise AssertionError("no seed with clear margins")


def _run(w, cache, c, blk=None, layers=1):
    rt = _rt()
    D = rt.to_device_bits
    B, K = w.batch, w.block_k
    V = c["ar_logits"].shape[2]
    pool = cache["k_pool"]
    step = rt.DecodeStep(batch=B, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                         block_k=K, page_size=w.page_size, max_pages_per_seq=cache["page_table"].shape[1],
                         max_seq_len=cache["page_table"].shape[1] * w.page_size, num_pages=pool.shape[-4], vocab=V,
                         num_layers=layers)
    dev = {k: D(v) for k, v in c.items() if isinstance(v, np.ndarray)}
    kp, vp, pt, sl = D(cache["k_pool"]), D(cache["v_pool"]), D(cache["page_table"]), D(cache["seq_lens"])
    outs = [torch.full((B,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
    toks = torch.full((B, K), -7, dtype=torch.int32, device="cuda")
    kb = vb = None
    if blk is not None:
        kb, vb = D(blk["k_blk"]), D(blk["v_blk"])
    step.sampling_consensus_commit(c["temperature"], dev["ar_logits"], dev["diff_logits"], dev["draft_tokens"],
                                   dev["accept_u"], dev["gumbel"], kb, vb, kp if blk is not None else None,
                                   vp if blk is not None else None, pt if blk is not None else None,
                                   sl if blk is not None else None, outs[0], outs[1], toks, outs[2])
    torch.cuda.synchronize()
    err = step.device_error()
    got = dict(accept_len=outs[0].cpu().numpy(), num_committed=outs[1].cpu().numpy(), out_tokens=toks.cpu().numpy(),
               next_anchor=outs[2].cpu().numpy(), k_pool=rt.bits_to_numpy(kp), v_pool=rt.bits_to_numpy(vp),
               seq_lens=sl.cpu().numpy(), err=err)
    step.close()
    return got


def _same(got, want):
    for key in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
        np.testing.assert_array_equal(got[key], want[key], err_msg=key)


@pytest.mark.parametrize("vocab,temperature,divergence", [
    (512, 1.0, 0.5), (97, 0.7, 1.0), (8191, 1.0, 0.3), (8193, 1.3, 0.5), (40001, 1.0, 0.5), (128256, 1.0, 0.5),
    (128256, 0.6, 1.0), (151936, 1.0, 0.2),
])
def test_sampling_consensus_matches_oracle(vocab, temperature, divergence):
    w = WORKLOADS["tiny"].with_(batch=6, block_k=8, vocab=vocab)
    c, seed = _clear_case(w, 100 + vocab % 97, temperature=temperature, divergence=divergence)
    cache = make_cache(w)
    got = _run(w, cache, c)
    want = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                            c["gumbel"], temperature)
    _same(got, want)
    assert got["err"] == 0


def test_sampling_special_cases():
    w = WORKLOADS["tiny"].with_(batch=4, block_k=5, vocab=3000)
    c, _ = _clear_case(w, 7, divergence=0.0)                      # p == q: everything kept
    cache = make_cache(w)
    got = _run(w, cache, c)
    assert np.all(got["accept_len"] == 5)
    np.testing.assert_array_equal(got["out_tokens"], c["draft_tokens"])
    d = dict(c); d["draft_tokens"] = c["draft_tokens"].copy(); d["draft_tokens"][:, 1] = [-1, 3000, 2 ** 30, -5]
    got = _run(w, cache, d)
    want = oracle.sampling_consensus_commit(d["ar_logits"], d["diff_logits"], d["draft_tokens"], d["accept_u"],
                                            d["gumbel"], 1.0)
    _same(got, want)                                               # invalid drafts: replacement drawn from p
    assert np.all(got["accept_len"] == 1)


def test_sampling_commit_loop_layer8b_shape():
    """Vocab 128256, K=16, paged cache: three looped steps with commit, everything compared bit for bit."""
    w = WORKLOADS["layer8b"].with_(steps=3)
    cache = make_cache(w)
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in cache.items()}
    rt = _rt()
    D = rt.to_device_bits
    B, K = w.batch, w.block_k
    step = rt.DecodeStep(batch=B, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                         block_k=K, page_size=w.page_size, max_pages_per_seq=cache["page_table"].shape[1],
                         max_seq_len=w.capacity_tokens(), num_pages=cache["num_pages"], vocab=w.vocab)
    kp, vp, pt, sl = D(cache["k_pool"]), D(cache["v_pool"]), D(cache["page_table"]), D(cache["seq_lens"])
    outs = [torch.empty((B,), dtype=torch.int32, device="cuda") for _ in range(3)]
    toks = torch.empty((B, K), dtype=torch.int32, device="cuda")
    seed = 500
    for s in range(w.steps):
        c, seed = _clear_case(w, seed + 1, temperature=1.0, divergence=0.4)
        blk = make_block(w, 600 + s)
        dev = {k: D(v) for k, v in c.items() if isinstance(v, np.ndarray)}
        step.sampling_consensus_commit(1.0, dev["ar_logits"], dev["diff_logits"], dev["draft_tokens"], dev["accept_u"],
                                       dev["gumbel"], D(blk["k_blk"]), D(blk["v_blk"]), kp, vp, pt, sl, outs[0], outs[1],
                                       toks, outs[2])
        torch.cuda.synchronize()
        want = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                                c["gumbel"], 1.0, blk["k_blk"], blk["v_blk"], ref["k_pool"], ref["v_pool"],
                                                ref["page_table"], ref["seq_lens"])
        got = dict(accept_len=outs[0].cpu().numpy(), num_committed=outs[1].cpu().numpy(),
                   out_tokens=toks.cpu().numpy(), next_anchor=outs[2].cpu().numpy())
        _same(got, want)
        np.testing.assert_array_equal(sl.cpu().numpy(), ref["seq_lens"])
    np.testing.assert_array_equal(rt.bits_to_numpy(kp), ref["k_pool"])
    np.testing.assert_array_equal(rt.bits_to_numpy(vp), ref["v_pool"])
    assert step.device_error() == 0
    step.close()


def test_sampling_capacity_error_and_multi_layer():
    w = Workload(name="cap", batch=3, num_q_heads=4, num_kv_heads=2, head_dim=64, block_k=8, context=28,
                 page_size=16, vocab=600, seed=31)
    layers = 3
    lens = np.array([28, 28, 28], np.int32)
    caches = [make_cache(w, seed=40 + l, seq_lens=lens) for l in range(layers)]
    cache = dict(caches[0])
    cache["k_pool"] = np.stack([c["k_pool"] for c in caches]); cache["v_pool"] = np.stack([c["v_pool"] for c in caches])
    cache["page_table"] = cache["page_table"].copy(); cache["page_table"][1, 2:] = -1
    c, _ = _clear_case(w, 3, divergence=0.0)                     # all kept: 8 rows to append everywhere
    blks = [make_block(w, 50 + l) for l in range(layers)]
    blk = dict(k_blk=np.stack([b["k_blk"] for b in blks]), v_blk=np.stack([b["v_blk"] for b in blks]))
    rk, rv, rl = cache["k_pool"].copy(), cache["v_pool"].copy(), lens.copy()
    want = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                            c["gumbel"], 1.0, blk["k_blk"], blk["v_blk"], rk, rv, cache["page_table"], rl,
                                            allow_capacity_error=True)
    assert want["status"] == -4 and want["num_committed"].tolist() == [8, 0, 8]
    got = _run(w, cache, c, blk, layers=layers)
    _same(got, want)
    assert got["err"] == -4
    np.testing.assert_array_equal(got["seq_lens"], rl)
    np.testing.assert_array_equal(got["k_pool"], rk)
    np.testing.assert_array_equal(got["v_pool"], rv)
