"""Pins of the batch-size pruning oracle (oracle/batch_prune.py) - CPU only.

The oracle is the pairwise definition.  It is pinned by a hand-worked example, by the textbook
sort-and-sweep construction of a two-criteria Pareto front (an independent algorithm), by the
special cases in which one criterion is constant, and by structural properties."""
from pathlib import Path

import numpy as np
import pytest

import oracle

GOLDEN = Path(__file__).resolve().parent / "golden" / "prune_worked_example.txt"


def test_hand_worked_example():
    rows = [l.split() for l in GOLDEN.read_text().splitlines() if l.strip() and not l.startswith("#")]
    sat = np.array([int(r[1]) for r in rows], dtype=np.uint32)
    lat = np.array([float(r[2]) for r in rows], dtype=np.float32)
    want = np.array([int(r[3]) for r in rows], dtype=np.uint8)
    keep, n_kept = oracle.batch_size_prune([0, len(rows)], sat, lat)
    assert keep.tolist() == want.tolist()
    assert n_kept.tolist() == [int(want.sum())]


def front_by_sort_and_sweep(sat, lat):
    """Textbook skyline of points (sat: larger is better, lat: smaller is better): visit the points by
    decreasing sat; a point is on the front iff its latency is below that of every point with strictly
    larger sat and not above that of any point with equal sat."""
    sat = np.asarray(sat, dtype=np.int64)
    lat = np.asarray(lat, dtype=np.float64)
    keep = np.zeros(len(sat), dtype=np.uint8)
    best_above = np.inf          # least latency among strictly larger sat values
    for s in sorted(set(sat.tolist()), reverse=True):
        idx = np.nonzero(sat == s)[0]
        level_min = lat[idx].min()
        if s != 0:
            for i in idx:
                if lat[i] == level_min and lat[i] < best_above:
                    keep[i] = 1
        best_above = min(best_above, level_min)
    return keep


@pytest.mark.parametrize("seed", range(12))
def test_equals_the_sort_and_sweep_front(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 60))
    # few distinct values: many ties in either criterion, and some candidates that serve nobody
    sat = rng.integers(0, 6, n).astype(np.uint32) * rng.integers(0, 2, n).astype(np.uint32) * 10
    lat = (rng.integers(0, 8, n) / 8.0).astype(np.float32)
    keep, n_kept = oracle.batch_size_prune([0, n], sat, lat)
    assert keep.tolist() == front_by_sort_and_sweep(sat, lat).tolist()
    assert int(n_kept[0]) == int(keep.sum())


@pytest.mark.parametrize("seed", range(8))
def test_structure_of_the_result(seed):
    rng = np.random.default_rng(200 + seed)
    n = int(rng.integers(2, 80))
    sat = rng.integers(0, 20, n).astype(np.uint32)
    lat = rng.random(n).astype(np.float32).round(1)
    keep, _ = oracle.batch_size_prune([0, n], sat, lat)
    kept = np.nonzero(keep == 1)[0]
    dom = oracle.batch_prune.dominates
    for i in kept:                       # the retained set: serves someone, nobody in it beats another
        assert sat[i] > 0
        assert not any(dom(sat[j], lat[j], sat[i], lat[i]) for j in range(n))
    for i in np.nonzero(keep == 0)[0]:   # every pruned candidate is beaten by a RETAINED one, or serves nobody
        assert sat[i] == 0 or any(dom(sat[j], lat[j], sat[i], lat[i]) for j in kept)
    # the order of the candidates inside the group does not matter
    perm = rng.permutation(n)
    keep_p, _ = oracle.batch_size_prune([0, n], sat[perm], lat[perm])
    assert keep_p.tolist() == keep[perm].tolist()
    # a candidate that is beaten changes nothing for the others
    worst = int(np.argmax(lat))
    sat2 = np.append(sat, max(int(sat.min()) - 1, 0)).astype(np.uint32)
    lat2 = np.append(lat, np.float32(lat[worst] + 1.0))
    keep2, _ = oracle.batch_size_prune([0, n + 1], sat2, lat2)
    assert keep2[:n].tolist() == keep.tolist() and keep2[n] == 0


def test_one_criterion_constant():
    sat = np.array([5, 9, 9, 3, 0, 9], dtype=np.uint32)
    same_lat = np.full(6, 0.25, dtype=np.float32)
    keep, _ = oracle.batch_size_prune([0, 6], sat, same_lat)   # only SLO satisfaction differs: the maxima stay
    assert keep.tolist() == [0, 1, 1, 0, 0, 1]
    lat = np.array([0.5, 0.2, 0.7, 0.2, 0.9], dtype=np.float32)
    keep, _ = oracle.batch_size_prune([0, 5], np.full(5, 7, np.uint32), lat)  # only latency differs: the minima stay
    assert keep.tolist() == [0, 1, 0, 1, 0]
    keep, n_kept = oracle.batch_size_prune([0, 3], np.zeros(3, np.uint32), np.zeros(3, np.float32))
    assert keep.tolist() == [0, 0, 0] and n_kept.tolist() == [0]   # nobody is served by anyone: nothing stays


def test_groups_are_independent_and_bad_groups_are_skipped():
    rng = np.random.default_rng(7)
    sat = rng.integers(0, 9, 30).astype(np.uint32)
    lat = rng.random(30).astype(np.float32)
    offsets = [0, 7, 7, 19, 30]
    keep, n_kept = oracle.batch_size_prune(offsets, sat, lat)
    for g in range(4):
        o0, o1 = offsets[g], offsets[g + 1]
        k, nk = oracle.batch_size_prune([0, o1 - o0], sat[o0:o1], lat[o0:o1])
        assert keep[o0:o1].tolist() == k.tolist() and n_kept[g] == nk[0]
    assert n_kept[1] == 0                                        # an empty group
    keep, n_kept = oracle.batch_size_prune([0, 10, 5, 40], sat, lat)  # backwards, then past the end
    assert n_kept.tolist()[1:] == [0, 0] and (keep[10:] == 255).all() and (keep[:10] != 255).all()
