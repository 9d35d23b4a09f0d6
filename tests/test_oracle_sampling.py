"""Pins for the temperature > 0 consensus oracle (CPU only).

The accept/replace rule is checked against things other than the oracle itself:
  * a hand-worked three-token case (ratio 0.6, residual concentrated on one token);
  * the property the paper claims for it (Section 3.3: lossless sampling): over many independent
    trials the first emitted token is distributed exactly as the target row p_0, and the chance that
    the first draft is kept is sum_v min(p_0(v), q_0(v)) (the closed form of the published rule);
  * q == p keeps every draft; a draft outside the vocabulary is never kept;
  * the low-temperature limit with a one-hot draft distribution reproduces the greedy consensus
    (Eq. 8), i.e. the already pinned greedy oracle;
  * never more than K tokens, at least one, commit identical to the greedy commit for equal counts.
"""
import numpy as np
import pytest

import oracle
from orthrus_inputs import Workload, make_block, make_cache, make_sampling_case


def _logp(p):
    return np.log(np.asarray(p, np.float64)).astype(np.float32)


def test_hand_worked_ratio_and_residual():
    p = [0.5, 0.3, 0.2]
    q = [0.2, 0.5, 0.3]
    ar = _logp(p).reshape(1, 1, 3)
    df = _logp(q).reshape(1, 1, 3)
    draft = np.array([[1]], np.int32)                     # p/q = 0.6
    g = np.array([[0.0, 50.0, 50.0]], np.float32)         # noise cannot matter: only token 0 has p > q
    for u, kept in ((0.59, True), (0.61, False), (0.0, True), (0.999, False)):
        r = oracle.sampling_consensus_commit(ar, df, draft, np.array([[u]], np.float32), g, 1.0)
        assert (r["accept_len"][0] == 1) == kept
        assert r["num_committed"][0] == 1
        assert r["out_tokens"][0, 0] == (1 if kept else 0)
        assert r["next_anchor"][0] == r["out_tokens"][0, 0]
    # draft 0 has p/q = 2.5 > 1: kept for every u
    r = oracle.sampling_consensus_commit(ar, df, np.array([[0]], np.int32), np.array([[0.9999]], np.float32), g, 1.0)
    assert r["accept_len"][0] == 1 and r["out_tokens"][0, 0] == 0


def test_temperature_scales_logits():
    # logits 2*log p at T = 2 is the same distribution as log p at T = 1
    p = [0.5, 0.3, 0.2]; q = [0.2, 0.5, 0.3]
    ar = (2 * _logp(p)).reshape(1, 1, 3); df = (2 * _logp(q)).reshape(1, 1, 3)
    g = np.zeros((1, 3), np.float32)
    for u, kept in ((0.59, True), (0.61, False)):
        r = oracle.sampling_consensus_commit(ar, df, np.array([[1]], np.int32), np.array([[u]], np.float32), g, 2.0)
        assert (r["accept_len"][0] == 1) == kept


def test_first_emitted_token_follows_the_target_distribution():
    """Losslessness: P(first token = v) = p_0(v), and P(first draft kept) = sum min(p_0, q_0)."""
    V, K, N = 7, 3, 120000
    rng = np.random.default_rng(11)
    lp = rng.standard_normal(V) * 1.5
    lq = lp + rng.standard_normal(V) * 1.0
    T = 0.8
    p = np.exp(lp / T); p /= p.sum()
    q = np.exp(lq / T); q /= q.sum()
    ar = np.broadcast_to(lp.astype(np.float32), (N, K, V)).copy()
    df = np.broadcast_to(lq.astype(np.float32), (N, K, V)).copy()
    p = np.exp(ar[0, 0].astype(np.float64) / T); p /= p.sum()       # exactly what the fp32 logits encode
    q = np.exp(df[0, 0].astype(np.float64) / T); q /= q.sum()
    draft = rng.choice(V, size=(N, K), p=q).astype(np.int32)         # drafts drawn from q
    u = rng.random((N, K), dtype=np.float32)
    g = rng.gumbel(size=(N, V)).astype(np.float32)
    r = oracle.sampling_consensus_commit(ar, df, draft, u, g, T)
    first = r["out_tokens"][:, 0]
    freq = np.bincount(first, minlength=V) / N
    sigma = np.sqrt(p * (1 - p) / N)
    assert np.all(np.abs(freq - p) < 4.5 * sigma), (freq, p)
    # the draft distribution is visibly different, so the test cannot pass by echoing the drafts
    assert np.abs(q - p).max() > 20 * sigma.max()
    keep0 = np.mean(r["accept_len"] >= 1)
    want = np.minimum(p, q).sum()
    assert abs(keep0 - want) < 4.5 * np.sqrt(want * (1 - want) / N)
    # both rows kept with probability (sum min)^2: rows are independent here
    keep2 = np.mean(r["accept_len"] >= 2)
    assert abs(keep2 - want ** 2) < 4.5 * np.sqrt(want ** 2 * (1 - want ** 2) / N)
    assert np.all(r["num_committed"] == np.minimum(r["accept_len"] + 1, K))
    assert r["num_committed"].min() >= 1 and r["num_committed"].max() <= K


def test_equal_distributions_keep_everything_and_invalid_drafts_are_rejected():
    w = Workload(name="s", batch=6, num_q_heads=2, num_kv_heads=1, head_dim=8, block_k=5, context=4, vocab=50)
    c = make_sampling_case(w, seed=3, divergence=0.0)
    np.testing.assert_array_equal(c["ar_logits"], c["diff_logits"])
    r = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                         c["gumbel"], 1.0)
    assert np.all(r["accept_len"] == w.block_k) and np.all(r["num_committed"] == w.block_k)
    np.testing.assert_array_equal(r["out_tokens"], c["draft_tokens"])
    np.testing.assert_array_equal(r["next_anchor"], c["draft_tokens"][:, -1])
    for bad in (-1, 50, 10 ** 6):
        d = c["draft_tokens"].copy(); d[:, 2] = bad
        r = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], d, c["accept_u"], c["gumbel"], 1.0)
        assert np.all(r["accept_len"] == 2) and np.all(r["num_committed"] == 3)
        assert np.all((r["out_tokens"][:, 2] >= 0) & (r["out_tokens"][:, 2] < 50))
        assert np.all(r["out_tokens"][:, 3:] == -1)
        # residual is zero everywhere when p == q: the replacement is then a draw from p itself
        want = np.argmax(np.log(np.exp(c["ar_logits"][:, 2].astype(np.float64)) /
                                np.exp(c["ar_logits"][:, 2].astype(np.float64)).sum(-1, keepdims=True))
                         + c["gumbel"].astype(np.float64), axis=-1)
        np.testing.assert_array_equal(r["out_tokens"][:, 2], want)


def test_low_temperature_one_hot_drafts_reduce_to_greedy_consensus():
    """T -> 0 with a one-hot draft distribution: keep iff draft == argmax, replacement == argmax."""
    rng = np.random.default_rng(5)
    B, K, V = 8, 6, 40
    ar = rng.standard_normal((B, K, V)).astype(np.float32)
    am = np.argmax(ar, -1).astype(np.int32)
    draft = am.copy()
    for b in range(B):                                   # diverge at row b % (K+1) (none for the last value)
        j = b % (K + 1)
        if j < K:
            draft[b, j] = (am[b, j] + 1 + b) % V
    df = np.full((B, K, V), -30.0, np.float32)
    bi, ki = np.meshgrid(np.arange(B), np.arange(K), indexing="ij")
    df[bi, ki, draft] = 30.0                             # q is one-hot on the draft
    u = rng.random((B, K), dtype=np.float32) * 0.98 + 0.01
    g = rng.gumbel(size=(B, V)).astype(np.float32)
    rs = oracle.sampling_consensus_commit(ar, df, draft, u, g, 0.002)
    rg = oracle.consensus_commit(ar, draft)
    for key in ("accept_len", "num_committed", "out_tokens", "next_anchor"):
        np.testing.assert_array_equal(rs[key], rg[key], err_msg=key)


def test_commit_matches_greedy_commit_for_equal_counts():
    w = Workload(name="s", batch=4, num_q_heads=4, num_kv_heads=2, head_dim=8, block_k=4, context_range=(0, 9),
                 page_size=4, vocab=30, steps=1, seed=8)
    c = make_sampling_case(w, seed=4, divergence=1.0)
    cache = make_cache(w)
    blk = make_block(w, 9)
    kp, vp, lens = cache["k_pool"].copy(), cache["v_pool"].copy(), cache["seq_lens"].copy()
    r = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                         c["gumbel"], 1.0, blk["k_blk"], blk["v_blk"], kp, vp, cache["page_table"], lens)
    assert len(set(r["accept_len"].tolist())) > 1                    # a mix of outcomes
    np.testing.assert_array_equal(lens, cache["seq_lens"] + r["num_committed"])
    P = 4
    for b in range(w.batch):
        for k in range(int(r["num_committed"][b])):
            pos = int(cache["seq_lens"][b]) + k
            pg = cache["page_table"][b, pos // P]
            np.testing.assert_array_equal(kp[pg, :, pos % P, :], blk["k_blk"][b, k])
            np.testing.assert_array_equal(vp[pg, :, pos % P, :], blk["v_blk"][b, k])
    changed = (kp != cache["k_pool"]).any(axis=(1, 3)).sum()
    assert changed <= r["num_committed"].sum()


def test_margins_are_reported():
    w = Workload(name="s", batch=3, num_q_heads=2, num_kv_heads=1, head_dim=8, block_k=4, context=4, vocab=64)
    c = make_sampling_case(w, seed=1)
    r = oracle.sampling_consensus_commit(c["ar_logits"], c["diff_logits"], c["draft_tokens"], c["accept_u"],
                                         c["gumbel"], 1.0)
    for b in range(w.batch):
        n = int(r["accept_len"][b])
        examined = min(n + 1, w.block_k)
        assert np.all(r["margin_accept"][b, :examined] >= 0) and np.all(r["margin_accept"][b, examined:] == -1)
        assert (r["margin_draw"][b] >= 0) == (n < w.block_k)
