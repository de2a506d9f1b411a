"""Oracle of the batch-size pruning that precedes Alg. 1.  TEST INFRASTRUCTURE ONLY.

Sec. IV-E ("Inference Batch Size Pruning"): for every parallelism configuration only the batch sizes
whose trade-off between latency and SLO satisfaction is Pareto-optimal are retained - batch sizes so
low that they add latency without serving more requests go, and so do batch sizes so high that no
request's SLO is met under load.

The definition written out, one pair of candidates at a time (plain Python loops; the groups are a
few dozen candidates): candidate i of a group goes when it meets no request's SLO, or when some
candidate j of the same group serves at least as many requests at no more latency and is strictly
better in one of the two.  Reading of the paper (it names the two criteria but prints no rule):
"SLO satisfaction" is the number of requests admitted, "latency" whatever response-latency figure
the caller evaluated the candidates with (lower is better); candidates that tie in both are all kept.
"""
from __future__ import annotations

import numpy as np


def dominates(sat_j, lat_j, sat_i, lat_i) -> bool:
    """j is at least as good as i in both respects and better in one."""
    return bool(sat_j >= sat_i and lat_j <= lat_i and (sat_j > sat_i or lat_j < lat_i))


def batch_size_prune(group_offsets, sat_count, latency):
    """Returns (keep [C] uint8, n_kept [G] uint32).  Candidates outside every group keep the value 255
    (not written); a group whose offsets run backwards or past the end is skipped with n_kept 0."""
    offsets = np.asarray(group_offsets, dtype=np.int64)
    sat = np.asarray(sat_count, dtype=np.int64)
    lat = np.asarray(latency, dtype=np.float32)
    keep = np.full(sat.shape[0], 255, dtype=np.uint8)
    n_kept = np.zeros(max(len(offsets) - 1, 0), dtype=np.uint32)
    for g in range(len(offsets) - 1):
        o0, o1 = int(offsets[g]), int(offsets[g + 1])
        if o0 > o1 or o1 > sat.shape[0]:
            continue
        for i in range(o0, o1):
            gone = sat[i] == 0
            for j in range(o0, o1):
                if dominates(sat[j], lat[j], sat[i], lat[i]):
                    gone = True
            keep[i] = 0 if gone else 1
            n_kept[g] += 0 if gone else 1
    return keep, n_kept
