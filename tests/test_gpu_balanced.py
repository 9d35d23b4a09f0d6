"""GPU parity of the balanced partition (num_splits = ORTHRUS_SPLITS_BALANCED) on batches shaped to
reach its corner cases: more sequences than one wave scans at once, empty sequences, fewer tiles than
workgroups, several units per workgroup and units cut into many pieces.  Same bar as every attention
test: max-abs <= 2e-2 and mean-abs <= 2e-3 against the fp64 oracle, run-to-run bit identical.
"""
import numpy as np
import pytest

import oracle
from orthrus_inputs import Workload, make_block, make_cache

from test_gpu_parity import AR, DIFF, GpuCase, _check_attn, _oracle_attn

pytestmark = pytest.mark.gpu

BALANCED = -1


def _run(w, seq_lens, view, want_lse=False):
    cache = make_cache(w, seq_lens=np.asarray(seq_lens, np.int32))
    blk = make_block(w, w.seed + 5 + view)
    case = GpuCase(w, cache, num_splits=BALANCED, max_seq_len=max(int(np.max(seq_lens)), 1))
    got = case.attn(view, blk, want_lse=want_lse)
    again = case.attn(view, blk, want_lse=want_lse)
    return cache, blk, got, again


@pytest.mark.parametrize("view", [DIFF, AR])
def test_many_short_sequences(view):
    """150 sequences (three 64-wide scans), lengths 0..90: most workgroups hold several whole units."""
    rng = np.random.default_rng(901)
    lens = rng.integers(0, 91, size=150)
    lens[:3] = (0, 0, 90)
    w = Workload(name="bal_many", seed=902, batch=150, num_q_heads=4, num_kv_heads=2, head_dim=64, block_k=4,
                 context=90, page_size=16, paging="shuffled")
    cache, blk, (got, lse), (again, lse2) = _run(w, lens, view, want_lse=True)
    want, want_lse = _oracle_attn(view, w, blk, cache, want_lse=True)
    _check_attn(got, want, "many short view %d" % view)
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)
    np.testing.assert_array_equal(got, again)
    np.testing.assert_array_equal(lse, lse2)


@pytest.mark.parametrize("view", [DIFF, AR])
def test_one_long_among_short(view):
    """One 9000-token sequence among tiny ones: its units are cut into many pieces, the others are not."""
    lens = [40, 9000, 0, 333, 64, 31]
    w = Workload(name="bal_skew", seed=911, batch=6, num_q_heads=8, num_kv_heads=2, head_dim=128, block_k=16,
                 context=9000, page_size=16, paging="scattered")
    cache, blk, got, again = _run(w, lens, view)
    _check_attn(got, _oracle_attn(view, w, blk, cache), "skewed view %d" % view)
    np.testing.assert_array_equal(got, again)


def test_fewer_tiles_than_workgroups():
    """Three tiles in the whole launch: all but three workgroups leave at once."""
    w = Workload(name="bal_few", seed=921, batch=1, num_q_heads=7, num_kv_heads=1, head_dim=128, block_k=32,
                 context=50, page_size=16, paging="contiguous")
    cache, blk, got, again = _run(w, [50], AR)
    _check_attn(got, _oracle_attn(AR, w, blk, cache), "few tiles")
    np.testing.assert_array_equal(got, again)


def test_balanced_matches_fixed_splits_closely():
    """Both partitions merge fp32 partials of the same tiles: outputs differ by bf16 rounding at most."""
    rng = np.random.default_rng(931)
    lens = rng.integers(100, 3000, size=8)
    w = Workload(name="bal_cmp", seed=932, batch=8, num_q_heads=28, num_kv_heads=4, head_dim=128, block_k=32,
                 context=3000, page_size=16, paging="scattered")
    cache = make_cache(w, seq_lens=lens.astype(np.int32))
    blk = make_block(w, 933)
    outs = [GpuCase(w, cache, num_splits=s, max_seq_len=int(lens.max())).attn(DIFF, blk, want_lse=False) for s in (BALANCED, 2)]
    assert np.abs(outs[0] - outs[1]).max() <= 1e-2
    pick = [int(np.argmin(lens)), int(np.argmax(lens))]
    sb = {k: np.ascontiguousarray(v[pick]) for k, v in blk.items()}
    sc = dict(cache, page_table=np.ascontiguousarray(cache["page_table"][pick]),
              seq_lens=np.ascontiguousarray(cache["seq_lens"][pick]))
    _check_attn(outs[0][pick], _oracle_attn(DIFF, w, sb, sc), "balanced vs oracle")
