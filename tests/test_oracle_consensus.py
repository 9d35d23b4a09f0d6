"""Pins for the consensus + commit oracle (CPU only).

Checked against things other than the oracle itself:
  * cases planted by the input generator (the accepted prefix is known by construction);
  * numpy's argmax (library routine, first index on ties) on random and tied rows;
  * hand-built rows: ties, -inf, NaN, out-of-range drafts, chance matches after a divergence;
  * the paper's own accounting: acceptance length 11.7 <-> TPF 6.35 at two passes per cycle,
    TPF floor 0.5, and the 4.5 MiB constant KV overhead at K=32;
  * losslessness: a speculative loop driven by the oracle emits exactly the token sequence of
    a one-token-at-a-time greedy loop over the same toy model;
  * commit == sequential AR appends (a python list per sequence, one row appended per token).
"""
import json
import os

import numpy as np
import pytest

import oracle
from orthrus_inputs import Workload, make_block, make_cache, make_consensus_case

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.json")))


def _w(**kw):
    base = dict(name="t", batch=4, num_q_heads=4, num_kv_heads=2, head_dim=8, block_k=6, context=10,
                page_size=4, vocab=97, accept="uniform", seed=11)
    base.update(kw)
    return Workload(**base)


@pytest.mark.parametrize("accept", ["uniform", "geometric"])
def test_planted_prefix_is_recovered(accept):
    w = _w(batch=64, accept=accept, block_k=8, vocab=301)
    case = make_consensus_case(w, seed=5)
    r = oracle.consensus_commit(case["ar_logits"], case["draft_tokens"])
    K = w.block_k
    np.testing.assert_array_equal(r["accept_len"], case["planted_n_acc"])
    m = np.minimum(case["planted_n_acc"] + 1, K)
    np.testing.assert_array_equal(r["num_committed"], m)
    for b in range(w.batch):
        np.testing.assert_array_equal(r["out_tokens"][b, :m[b]], case["planted_top"][b, :m[b]])
        assert np.all(r["out_tokens"][b, m[b]:] == -1)
        assert r["next_anchor"][b] == case["planted_top"][b, m[b] - 1]
    # every planted length 0..K occurs in the uniform case, so both ends of the rule are exercised
    if accept == "uniform":
        assert set(case["planted_n_acc"].tolist()) == set(range(K + 1))


def test_argmax_matches_numpy_including_ties():
    rng = np.random.default_rng(3)
    B, K, V = 5, 7, 50
    logits = rng.integers(-3, 4, size=(B, K, V)).astype(np.float32)      # many exact ties
    am = np.argmax(logits, axis=-1).astype(np.int32)                      # first index of the maximum
    draft = am.copy()
    r = oracle.consensus_commit(logits, draft)
    assert np.all(r["accept_len"] == K) and np.all(r["num_committed"] == K)
    np.testing.assert_array_equal(r["out_tokens"], am)
    np.testing.assert_array_equal(r["next_anchor"], am[:, -1])
    # a draft equal to a *later* tied maximum is not the greedy token
    b, k = 0, 2
    ties = np.flatnonzero(logits[b, k] == logits[b, k].max())
    assert len(ties) > 1
    draft[b, k] = ties[1]
    r = oracle.consensus_commit(logits, draft)
    assert r["accept_len"][b] == k and r["num_committed"][b] == k + 1
    assert r["out_tokens"][b, k] == ties[0]


def test_special_values_and_rejections():
    V, K = 8, 5
    ninf, nan = -np.inf, np.nan
    logits = np.array([[
        [ninf] * V,                                   # all -inf: index 0
        [0, 1, nan, 5, nan, 9, 0, 0],                 # NaN outranks numbers, first NaN wins: index 2
        [1, 3, 3, 2, 3, 0, 0, 0],                     # tie: index 1
        [-0.0, 0.0, -1, -1, -1, -1, -1, -1],          # -0.0 == +0.0: index 0
        [0, 0, 0, 0, 0, 0, 0, 7],                     # last index
    ]], dtype=np.float32)
    want = np.array([[0, 2, 1, 0, 7]], np.int32)
    r = oracle.consensus_commit(logits, want.copy())
    assert r["accept_len"][0] == K
    np.testing.assert_array_equal(r["out_tokens"], want)
    # divergence at k=1; later positions match by chance and must be ignored
    draft = want.copy(); draft[0, 1] = 4
    r = oracle.consensus_commit(logits, draft)
    assert r["accept_len"][0] == 1 and r["num_committed"][0] == 2
    np.testing.assert_array_equal(r["out_tokens"][0], [0, 2, -1, -1, -1])
    assert r["next_anchor"][0] == 2                                        # the AR correction token
    # out-of-range drafts never match
    for bad in (-1, V, 2 ** 31 - 1):
        draft = want.copy(); draft[0, 0] = bad
        r = oracle.consensus_commit(logits, draft)
        assert r["accept_len"][0] == 0 and r["num_committed"][0] == 1
        np.testing.assert_array_equal(r["out_tokens"][0], [0, -1, -1, -1, -1])


def test_paper_accounting_acceptance_length_vs_tpf():
    """Acceptance length 11.7 with K=32 must give TPF 6.35 at 2 passes per cycle (accept + 1 correction)."""
    K = GOLDEN["block_k_train"]["value"]
    n_acc = np.array([12, 11, 13, 10, 14, 9, 15, 8, 16, 9], np.int32)       # mean 11.7, all < K
    assert abs(n_acc.mean() - GOLDEN["math500_acceptance_length"]["value"]) < 1e-12
    w = _w(batch=len(n_acc), block_k=K, vocab=64)
    case = make_consensus_case(w, seed=1, n_acc=n_acc)
    r = oracle.consensus_commit(case["ar_logits"], case["draft_tokens"])
    np.testing.assert_array_equal(r["accept_len"], n_acc)
    passes = GOLDEN["forward_passes_per_cycle"]["value"] * len(n_acc)
    tpf = r["num_committed"].sum() / passes
    assert abs(tpf - GOLDEN["math500_tpf_k32"]["value"]) < 1e-12
    # floor: nothing accepted anywhere still emits one token per cycle
    case0 = make_consensus_case(w, seed=2, n_acc=np.zeros(len(n_acc), np.int32))
    r0 = oracle.consensus_commit(case0["ar_logits"], case0["draft_tokens"])
    assert r0["num_committed"].sum() / passes == GOLDEN["tpf_lower_bound"]["value"]
    # ceiling: everything accepted emits K tokens, never K+1
    caseK = make_consensus_case(w, seed=3, n_acc=np.full(len(n_acc), K, np.int32))
    rK = oracle.consensus_commit(caseK["ar_logits"], caseK["draft_tokens"])
    assert np.all(rK["num_committed"] == K) and np.all(rK["accept_len"] == K)


def test_constant_kv_overhead_closed_form():
    """The only extra KV state is the block's K/V staging: layers*2*K*H_kv*d*2 bytes = 4.5 MiB at K=32."""
    g = GOLDEN["qwen3_8b_geometry"]
    K = GOLDEN["block_k_train"]["value"]
    w = _w(batch=1, num_q_heads=g["num_kv_heads"] * 4, num_kv_heads=g["num_kv_heads"], head_dim=g["head_dim"],
           block_k=K)
    blk = make_block(w, seed=0)
    per_layer = blk["k_blk"].nbytes + blk["v_blk"].nbytes
    assert per_layer * g["layers"] == GOLDEN["kv_overhead_mib_k32"]["value"] * 2 ** 20


def _toy_logits(prefix, V, salt):
    """Deterministic 'model': logits for the next token depend only on the token prefix."""
    h = np.random.default_rng([salt] + [int(t) for t in prefix]).standard_normal(V).astype(np.float32)
    return h


def test_lossless_speculative_loop_equals_greedy_loop():
    V, K, T, salt = 23, 5, 60, 99
    prompt = [3, 1, 4]
    # greedy one-token-at-a-time reference
    seq = list(prompt)
    while len(seq) < len(prompt) + T:
        seq.append(int(np.argmax(_toy_logits(seq, V, salt))))
    greedy = seq[len(prompt):]
    # speculative loop: anchor = last emitted token; drafts are right with probability 0.7
    rng = np.random.default_rng(5)
    out = list(prompt)
    # the first generated token comes from the AR view (prefill), as in the paper's block construction
    out.append(int(np.argmax(_toy_logits(out, V, salt))))
    cycles = 0
    while len(out) < len(prompt) + T:
        draft = []
        ctx = list(out)
        for k in range(K):
            true_next = int(np.argmax(_toy_logits(ctx, V, salt)))
            tok = true_next if rng.random() < 0.7 else int(rng.integers(0, V))
            draft.append(tok)
            ctx.append(tok)
        # verify pass: row k is conditioned on the anchor and drafts 0..k-1
        rows = [_toy_logits(out + draft[:k], V, salt) for k in range(K)]
        r = oracle.consensus_commit(np.stack(rows)[None], np.array([draft], np.int32))
        m = int(r["num_committed"][0])
        assert 1 <= m <= K and m == min(int(r["accept_len"][0]) + 1, K)
        out.extend(int(t) for t in r["out_tokens"][0, :m])
        assert r["next_anchor"][0] == out[-1]
        cycles += 1
    got = out[len(prompt):len(prompt) + T]
    assert got == greedy
    assert cycles < T                      # some drafts were accepted, otherwise the test is vacuous


def _logical(pool, page_table, b, L):
    P = pool.shape[-2]
    pos = np.arange(L)
    return pool[page_table[b, pos // P], :, pos % P, :]


def test_commit_equals_sequential_appends_over_steps():
    w = _w(batch=3, num_q_heads=4, num_kv_heads=2, head_dim=8, block_k=4, context_range=(0, 13), page_size=4,
           vocab=31, steps=6, paging="scattered")
    c = make_cache(w)
    kp, vp, pt, lens = c["k_pool"], c["v_pool"], c["page_table"], c["seq_lens"]
    ref_k = [list(_logical(kp, pt, b, lens[b])) for b in range(w.batch)]
    ref_v = [list(_logical(vp, pt, b, lens[b])) for b in range(w.batch)]
    kp0, vp0, lens0 = kp.copy(), vp.copy(), lens.copy()
    total = np.zeros(w.batch, np.int64)
    for step in range(w.steps):
        case = make_consensus_case(w, seed=100 + step)
        blk = make_block(w, seed=200 + step)
        r = oracle.consensus_commit(case["ar_logits"], case["draft_tokens"], blk["k_blk"], blk["v_blk"],
                                    kp, vp, pt, lens)
        for b in range(w.batch):
            m = int(r["num_committed"][b])
            assert m == min(int(case["planted_n_acc"][b]) + 1, w.block_k)
            for k in range(m):                       # sequential AR: one appended row per emitted token
                ref_k[b].append(blk["k_blk"][b, k])
                ref_v[b].append(blk["v_blk"][b, k])
            total[b] += m
    np.testing.assert_array_equal(lens, lens0 + total)
    touched = np.zeros(kp.shape[:1] + kp.shape[2:3], bool)
    for b in range(w.batch):
        np.testing.assert_array_equal(_logical(kp, pt, b, lens[b]), np.stack(ref_k[b]) if ref_k[b] else
                                      np.empty((0,) + kp.shape[1:2] + kp.shape[3:], kp.dtype))
        np.testing.assert_array_equal(_logical(vp, pt, b, lens[b]), np.stack(ref_v[b]))
        for pos in range(int(lens0[b]), int(lens[b])):
            touched[pt[b, pos // 4], pos % 4] = True
    # O(1) footprint: nothing outside the appended positions changed
    same_k = (kp == kp0).all(axis=(1, 3)); same_v = (vp == vp0).all(axis=(1, 3))
    assert np.all(same_k | touched) and np.all(same_v | touched)


def test_multi_layer_commit_and_consensus_only_mode():
    w = _w(batch=2, num_kv_heads=2, head_dim=8, block_k=3, context=5, page_size=4, vocab=19)
    layers = 3
    caches = [make_cache(w, seed=50 + l) for l in range(layers)]
    kp = np.stack([c["k_pool"] for c in caches]); vp = np.stack([c["v_pool"] for c in caches])
    pt, lens = caches[0]["page_table"], caches[0]["seq_lens"].copy()
    blks = [make_block(w, seed=60 + l) for l in range(layers)]
    kb = np.stack([b["k_blk"] for b in blks]); vb = np.stack([b["v_blk"] for b in blks])
    case = make_consensus_case(w, seed=9, n_acc=np.array([2, 0], np.int32))
    kp0 = kp.copy()
    r0 = oracle.consensus_commit(case["ar_logits"], case["draft_tokens"])          # consensus only
    r = oracle.consensus_commit(case["ar_logits"], case["draft_tokens"], kb, vb, kp, vp, pt, lens)
    for key in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
        np.testing.assert_array_equal(r[key], r0[key])
    np.testing.assert_array_equal(lens, [5 + 3, 5 + 1])
    for l in range(layers):
        for b, m in ((0, 3), (1, 1)):
            for k in range(m):
                pos = 5 + k
                np.testing.assert_array_equal(kp[l, pt[b, pos // 4], :, pos % 4, :], kb[l, b, k])
                np.testing.assert_array_equal(vp[l, pt[b, pos // 4], :, pos % 4, :], vb[l, b, k])
    assert (kp != kp0).sum() > 0


def test_capacity_error_leaves_sequence_untouched():
    w = _w(batch=2, num_kv_heads=1, head_dim=8, block_k=4, context=6, page_size=4, vocab=13)
    c = make_cache(w)
    c["page_table"][1, 2:] = -1                     # sequence 1: positions 8.. are not mapped
    case = make_consensus_case(w, seed=4, n_acc=np.array([4, 4], np.int32))
    blk = make_block(w, seed=5)
    kp0, vp0 = c["k_pool"].copy(), c["v_pool"].copy()
    lens = c["seq_lens"].copy()
    with pytest.raises(RuntimeError):
        oracle.consensus_commit(case["ar_logits"], case["draft_tokens"], blk["k_blk"], blk["v_blk"],
                                c["k_pool"].copy(), c["v_pool"].copy(), c["page_table"], lens.copy())
    r = oracle.consensus_commit(case["ar_logits"], case["draft_tokens"], blk["k_blk"], blk["v_blk"],
                                c["k_pool"], c["v_pool"], c["page_table"], lens, allow_capacity_error=True)
    assert r["status"] == -4
    np.testing.assert_array_equal(lens, [10, 6])
    np.testing.assert_array_equal(r["num_committed"], [4, 0])
    np.testing.assert_array_equal(r["accept_len"], [4, 4])
    # sequence 1's pages are untouched
    for slot in range(2):
        pg = c["page_table"][1, slot]
        np.testing.assert_array_equal(c["k_pool"][pg], kp0[pg])
        np.testing.assert_array_equal(c["v_pool"][pg], vp0[pg])
