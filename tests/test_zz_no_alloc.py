"""GPU test of the allocation-free consensus entry point: orthrus_consensus_commit_noalloc (static device
scratch instead of a caller workspace) against orthrus_consensus_commit on the same inputs, bit for bit,
twice in a row with the second call on a smaller problem, plus the size limit."""
import numpy as np
import pytest
import torch

from orthrus_inputs import Workload, make_block, make_cache, make_consensus_case

pytestmark = pytest.mark.gpu


def _dev(a):
    from paper_2605_12825_amd import runtime as rt
    return rt.to_device_bits(a)


def _run(entry, w, cache, cc, blk):
    """One consensus + commit call through `entry` ("workspace" or "noalloc") on fresh device copies."""
    from paper_2605_12825_amd import binding as B
    from paper_2605_12825_amd import runtime as rt
    Bn, K = w.batch, w.block_k
    k_pool, v_pool = _dev(cache["k_pool"]), _dev(cache["v_pool"])
    page_table, seq_lens = _dev(cache["page_table"]), _dev(cache["seq_lens"])
    logits, draft = _dev(cc["ar_logits"]), _dev(cc["draft_tokens"])
    kb, vb = _dev(blk["k_blk"]), _dev(blk["v_blk"])
    outs = [torch.full((Bn,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
    toks = torch.full((Bn, K), -7, dtype=torch.int32, device="cuda")
    step = rt.DecodeStep(batch=Bn, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                         block_k=K, page_size=w.page_size, max_pages_per_seq=cache["page_table"].shape[1],
                         max_seq_len=min(w.capacity_tokens(), cache["page_table"].shape[1] * w.page_size),
                         num_pages=cache["k_pool"].shape[0], vocab=w.vocab)
    if entry == "noalloc":
        B.orthrus_consensus_commit_noalloc(step.ctx, step.params, logits, draft, kb, vb, k_pool, v_pool, page_table,
                                           seq_lens, outs[0], outs[1], toks, outs[2])
    else:
        step.consensus_commit(logits, draft, kb, vb, k_pool, v_pool, page_table, seq_lens, outs[0], outs[1], toks,
                              outs[2])
    torch.cuda.synchronize()
    assert step.device_error() == 0
    res = dict(accept_len=outs[0].cpu().numpy(), num_committed=outs[1].cpu().numpy(), out_tokens=toks.cpu().numpy(),
               next_anchor=outs[2].cpu().numpy(), seq_lens=seq_lens.cpu().numpy(),
               k_pool=rt.bits_to_numpy(k_pool), v_pool=rt.bits_to_numpy(v_pool))
    step.close()
    return res


def _case(batch, block_k, vocab, seed):
    w = Workload(name="na%d" % seed, batch=batch, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=block_k,
                 context_range=(5, 200), page_size=16, vocab=vocab, accept="uniform", steps=1, seed=seed)
    return w, make_cache(w), make_consensus_case(w, seed + 1), make_block(w, seed + 2)


def test_noalloc_entry_matches_the_workspace_entry_twice_second_call_smaller():
    from paper_2605_12825_amd import binding as B
    assert B.orthrus_noalloc_scratch_bytes() == 1 << 20
    # first a larger problem (64 rows x 5 chunks of the scratch), then a smaller one that reuses its start
    for batch, block_k, vocab, seed in ((4, 16, 40001, 510), (2, 5, 8193, 520)):
        w, cache, cc, blk = _case(batch, block_k, vocab, seed)
        want = _run("workspace", w, cache, cc, blk)
        got = _run("noalloc", w, cache, cc, blk)
        for key in want:
            np.testing.assert_array_equal(got[key], want[key], err_msg="%s (batch %d)" % (key, batch))
        np.testing.assert_array_equal(got["accept_len"], cc["planted_n_acc"])
        assert (got["seq_lens"] > cache["seq_lens"]).all()


def test_noalloc_entry_rejects_a_problem_beyond_its_scratch():
    from paper_2605_12825_amd import binding as B
    from paper_2605_12825_amd import runtime as rt
    # 64 x 32 rows x 75 chunks x 8 bytes > 1 MiB: refused on the host, nothing launched, nothing written
    step = rt.DecodeStep(batch=64, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=32, page_size=16,
                         max_pages_per_seq=4, max_seq_len=32, num_pages=256, vocab=75 * 8192)
    assert B.orthrus_consensus_workspace_bytes(step.params) > B.orthrus_noalloc_scratch_bytes()
    sentinel = torch.full((64,), -7, dtype=torch.int32, device="cuda")
    toks = torch.full((64, 32), -7, dtype=torch.int32, device="cuda")
    logits = torch.zeros((8,), dtype=torch.float32, device="cuda")      # never read: the call is refused first
    draft = torch.zeros((64, 32), dtype=torch.int32, device="cuda")
    st = B.orthrus_consensus_commit_noalloc(step.ctx, step.params, logits, draft, None, None, None, None, None, None,
                                            sentinel, sentinel, toks, sentinel, check=False)
    torch.cuda.synchronize()
    assert st == B.ORTHRUS_EWORKSPACE
    assert (sentinel.cpu().numpy() == -7).all() and (toks.cpu().numpy() == -7).all()
    step.close()
