"""The bookkeeping of the balanced decode schedule, checked on the CPU by brute force.

The column-split attention kernel cuts one flat list of work units into equal ranges, one per
persistent workgroup: a sequence with live slots owns `run_cost` units (the fixed cost of a run)
followed by one unit per 16-slot tile.  Workgroup i stores the partial of its share of sequence b
as piece i + b.  The combine kernels never see that list: they recover a row's pieces from the
running unit counts alone, as first = (prefix[b] + run_cost) / share, last = (prefix[b + 1] - 1) / share.
Two independent statements of the same rule are compared here for many shapes: a walk over the
workgroups' ranges (what the attention kernel does) and the closed form (what the combine kernels
do).  They have to name the same pieces, every tile has to be covered exactly once, and no two
(workgroup, sequence) pairs may share a piece id.
"""
import numpy as np
import pytest

TILE = 16


def units_of(live, run_cost):
    return run_cost + (live + TILE - 1) // TILE if live > 0 else 0


def walk_ranges(lives, n_wg, run_cost):
    """Per workgroup: the (sequence, first slot, end slot) runs it streams, by walking its range."""
    prefix = np.concatenate([[0], np.cumsum([units_of(l, run_cost) for l in lives])])
    total = int(prefix[-1])
    share = -(-total // n_wg) if total else 1
    runs = []
    for i in range(n_wg):
        pos, end = i * share, min((i + 1) * share, total)
        mine = []
        p = pos
        while p < end:
            b = int(np.searchsorted(prefix, p, side="right") - 1)
            while prefix[b + 1] <= p:          # sequences without live slots own no unit
                b += 1
            org = int(prefix[b]) + run_cost    # unit of the sequence's first tile
            seg_end = min(end, int(prefix[b + 1]))
            if seg_end > org:                  # some tile of b lies inside the range
                k0 = (max(p, org) - org) * TILE
                k1 = min(lives[b], (seg_end - org) * TILE)
                mine.append((b, k0, k1))
            p = seg_end
        runs.append(mine)
    return runs, prefix, share


def pieces_closed_form(prefix, share, b, run_cost):
    p0, p1 = int(prefix[b]), int(prefix[b + 1])
    if p1 == p0:
        return 0, 0
    first, last = (p0 + run_cost) // share, (p1 - 1) // share
    return first + b, last - first + 1


@pytest.mark.parametrize("run_cost", [0, 1, 6, 16])
@pytest.mark.parametrize("seed", range(6))
def test_walk_and_closed_form_name_the_same_pieces(seed, run_cost):
    rng = np.random.default_rng(100 * run_cost + seed)
    B = int(rng.integers(1, 40))
    n_wg = int(rng.choice([1, 3, 8, 64, 256, 512]))
    top = int(rng.choice([1, 17, 200, 5000]))
    lives = [int(x) for x in rng.integers(0, top + 1, size=B)]
    if seed % 2:
        lives[:: 3] = [0] * len(lives[:: 3])
    runs, prefix, share = walk_ranges(lives, n_wg, run_cost)

    # every live slot of every sequence is streamed exactly once, in runs that start on tile boundaries
    cover = [np.zeros(max(l, 1), np.int32) for l in lives]
    ids = {}
    for i, mine in enumerate(runs):
        seqs = [b for b, _, _ in mine]
        assert seqs == sorted(set(seqs))       # at most one run per sequence and workgroup, in order
        for b, k0, k1 in mine:
            assert 0 <= k0 < k1 <= lives[b] and k0 % TILE == 0
            cover[b][k0:k1] += 1
            assert (i + b) not in ids          # piece ids are unique over (workgroup, sequence)
            ids[i + b] = (i, b)
    for b, l in enumerate(lives):
        assert np.all(cover[b][:l] == 1)

    # the closed form of the combine kernels finds exactly those pieces, contiguous per row
    for b, l in enumerate(lives):
        first, count = pieces_closed_form(prefix, share, b, run_cost)
        from_walk = sorted(i + b for i, mine in enumerate(runs) for bb, _, _ in mine if bb == b)
        assert from_walk == list(range(first, first + count))
        assert (count == 0) == (l == 0)
    assert len(ids) <= n_wg + B                # the workspace holds n_wg + batch pieces


def test_a_run_start_costs_the_workgroup_that_many_tiles():
    # two equal sequences over 4 workgroups, run cost 6: 2 * (6 + 50) = 112 units, 28 per workgroup;
    # the workgroups that start a sequence stream 22 tiles, the others 28
    runs, prefix, share = walk_ranges([800, 800], 4, 6)
    assert share == 28 and list(prefix) == [0, 56, 112]
    tiles = [[(k1 - k0 + TILE - 1) // TILE for _, k0, k1 in mine] for mine in runs]
    assert tiles == [[22], [28], [22], [28]]
