"""The arithmetic of the balanced partition, checked by brute force on the CPU.

The split kernel cuts the launch's tile sequence (head-major, per sequence ceil(L/32) cache tiles plus
the in-block tile) at floor(w * T / N); the merge kernel finds a unit's pieces again from closed forms
for the first and last workgroup that touch it.  This test restates both rules in a few lines of
Python and checks, against an explicit tile-by-tile assignment, that the closed forms name exactly the
workgroups that hold tiles of the unit, that a workgroup never needs more than its two partial slots,
and that "one workgroup holds the whole unit" is the same condition on both sides.
"""
import numpy as np
import pytest


def _cuts(total, n):
    n = min(n, total)
    return n, [w * total // n for w in range(n + 1)]


def _segments(lens, heads, n_wgs):
    """What the split kernel does: per workgroup a list of (unit, first tile, tiles, final?, slot)."""
    tiles = [(int(L) + 31) // 32 + 1 for L in lens]
    per_head = sum(tiles)
    total = per_head * heads
    n, c = _cuts(total, n_wgs)
    out = []
    for w in range(n):
        pos, left, segs = c[w], c[w + 1] - c[w], []
        g, r = divmod(pos, per_head)
        b = 0
        while r >= tiles[b]:
            r -= tiles[b]
            b += 1
        o = r
        while left > 0:
            take = min(tiles[b] - o, left)
            final = o == 0 and take == tiles[b]
            segs.append(((g, b), o, take, final, None if final else 2 * w + (1 if o == 0 else 0)))
            left -= take
            o = 0
            b += 1
            if b == len(tiles):
                b, g = 0, g + 1
        out.append(segs)
    return tiles, per_head, total, n, out


def _pieces(tiles, per_head, total, n, g, b):
    """What the merge kernel does for unit (g, b): None when the split kernel finished it, else its slots."""
    u0 = g * per_head + sum(tiles[:b])
    u1 = u0 + tiles[b]
    w_lo = ((u0 + 1) * n + total - 1) // total - 1
    w_hi = (u1 * n + total - 1) // total - 1
    if w_lo == w_hi:
        return None
    return [2 * w_lo + 1] + [2 * w for w in range(w_lo + 1, w_hi + 1)]


@pytest.mark.parametrize("seed", range(40))
def test_closed_forms_match_the_tile_by_tile_assignment(seed):
    rng = np.random.default_rng(seed)
    batch = int(rng.integers(1, 40))
    heads = int(rng.integers(1, 5))
    hi = int(rng.choice([40, 300, 3000, 9000]))
    lens = rng.integers(0, hi + 1, size=batch)
    n_wgs = int(rng.choice([1, 2, 7, 64, 256, 1536]))
    tiles, per_head, total, n, wgs = _segments(lens, heads, n_wgs)
    assert sum(t for segs in wgs for _, _, t, _, _ in segs) == total
    # equal shares: no workgroup has more than one tile above the average
    for segs in wgs:
        assert 1 <= sum(t for _, _, t, _, _ in segs) <= -(-total // n)
        slots = [s for *_, s in segs if s is not None]
        assert len(slots) == len(set(slots)) <= 2
    by_unit = {}
    for w, segs in enumerate(wgs):
        for unit, o, take, final, slot in segs:
            by_unit.setdefault(unit, []).append((o, take, final, slot))
    for g in range(heads):
        for b in range(batch):
            got = sorted(by_unit[(g, b)])
            # the pieces tile the unit without gap or overlap
            at = 0
            for o, take, _, _ in got:
                assert o == at
                at += take
            assert at == tiles[b]
            want = _pieces(tiles, per_head, total, n, g, b)
            if want is None:
                assert len(got) == 1 and got[0][2]
            else:
                assert not any(final for _, _, final, _ in got)
                assert [slot for *_, slot in got] == want


def test_more_workgroups_than_tiles():
    tiles, per_head, total, n, wgs = _segments([0, 5], 1, 256)
    assert total == 3 and n == 3 and all(len(s) == 1 for s in wgs)
