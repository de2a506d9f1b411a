"""Pins of the oracle's Alg. 1 (instance configuration, single model), Alg. 2 (partition scan) and
the request split by SLO (Sec. IV-E)."""
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2509_06362_amd import workloads as W
from tests.test_oracle_window import read_golden, worked_example_workload

GOLDEN = Path(__file__).parent / "golden" / "partition_worked_example.txt"
WEIGHTS = (4.0, 0.3, 2048.0, 2.0)


def read_partition_golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split(":")
        out[k.strip()] = [float(x) for x in v.split()]
    return out


def test_hand_worked_greedy():
    g = read_partition_golden()
    w = worked_example_workload(read_golden())
    w = W.replace(w, tp_degree=np.array([1], dtype=np.uint32))
    r = oracle.ins_deploy(w, int(g["alg1_n_gpus"][0]), [0], [4], 4.0, 0.25, 128.0, 1.0, window=w.window)
    assert r["phi_star"] == pytest.approx(g["alg1_phi_star"], rel=1e-6)
    assert r["cnt_star"].tolist() == g["alg1_cnt_star"]
    assert r["cfg_star"].tolist() == [-1, 0, 0, -1, -1]
    assert r["n_evaluated"] == g["alg1_n_evaluated"][0]


def test_hand_worked_partition():
    g = read_partition_golden()
    n, rl, rr = int(g["alg2_n_gpus"][0]), int(g["alg2_n_req_l"][0]), int(g["alg2_n_req"][0])
    for key, hom in (("a", g["alg2_phi_h_star_a"]), ("b", g["alg2_phi_h_star_b"]), ("none", None)):
        r = oracle.resource_partition(n, g["alg2_phi_t_star"], g["alg2_phi_l_star"], hom, rl, rr)
        exp = g[f"alg2_expect_{key}"]
        assert [r["g_t"], r["g_l"], r["heterogeneous"], r["k_h"]] == exp[:4]
        assert r["phi_opt"] == exp[4]


def greedy_by_hand(w, n_gpus, cfg_tp, cfg_b, weights, window, max_inst=256):
    """Alg. 1 written a second time, in Python, on explicit candidate arrays scored one at a time."""
    phi_star = np.zeros(n_gpus + 1, np.float32)
    best = [None] * (n_gpus + 1)
    n_eval = 0
    for i, (t, b) in enumerate(zip(cfg_tp, cfg_b)):
        deg = int(w.tp_degree[t])
        n, phi = 0, np.float32(0.0)
        while n * deg < n_gpus:
            m = n + 1
            if m * deg > n_gpus or m > max_inst:
                break
            cand = W.replace(
                w, n_inst=np.array([m], np.uint32), tp_idx=np.full((1, m), t, np.uint8),
                max_batch=np.full((1, m), b, np.uint16), occ=np.zeros((1, m), np.int32),
                q_ticks=np.zeros((1, m), np.uint64))
            s = oracle.placement_score(cand, *weights, window=window)["score"][0]
            n_eval += 1
            if not s > phi:
                break
            n, phi = m, s
            if phi > phi_star[n * deg]:
                phi_star[n * deg] = phi
                best[n * deg] = (i, n)
    return phi_star, best, n_eval


@pytest.mark.parametrize("n_req,rate,n_gpus,window,max_inst", [
    (1500, 400.0, 16, 64, 256), (1200, 150.0, 12, 32, 5), (800, 900.0, 9, 0, 256), (0, 400.0, 8, 16, 256),
    (1500, 20.0, 16, 64, 256), (1500, 5.0, 16, 16, 256),
])
def test_greedy_matches_a_second_implementation(n_req, rate, n_gpus, window, max_inst):
    w = W.partition_case(n_req=max(n_req, 1), rate=rate, seed=11 + n_gpus)
    w = w.with_requests(0, n_req)
    tp, b = W.all_configs(batch_set=[4, 32, 128])
    r = oracle.ins_deploy(w, n_gpus, tp, b, *WEIGHTS, window=window, max_inst=max_inst)
    phi, best, n_eval = greedy_by_hand(w, n_gpus, tp, b, WEIGHTS, window, max_inst)
    assert np.array_equal(r["phi_star"], phi)
    assert r["n_evaluated"] == n_eval
    for k in range(n_gpus + 1):
        if best[k] is None:
            assert r["cfg_star"][k] == -1 and r["cnt_star"][k] == 0 and r["phi_star"][k] == 0
        else:
            assert (r["cfg_star"][k], r["cnt_star"][k]) == best[k]
            assert r["cnt_star"][k] * w.tp_degree[tp[r["cfg_star"][k]]] == k
    if n_req and window:
        assert np.count_nonzero(r["phi_star"]) > 3          # growth does happen in the windowed form
    if rate <= 20.0:                                         # light load: growth stops early
        assert n_eval < sum(min(n_gpus // int(w.tp_degree[t]), max_inst) for t in tp)


def test_static_scoring_never_grows_past_one_instance():
    """Without the state update identical fresh instances are indistinguishable: the second one
    changes nothing, so it is rejected.  (The reason the placer's growth needs the windowed form.)"""
    w = W.partition_case(n_req=600, seed=3)
    tp, b = W.all_configs(batch_set=[8, 64])
    r = oracle.ins_deploy(w, 16, tp, b, *WEIGHTS, window=0)
    assert set(r["cnt_star"].tolist()) <= {0, 1}
    assert r["n_evaluated"] == 2 * len(tp)


def partition_brute_force(n_gpus, pt, pl, ph, n_l, n):
    cap = 0 if n == 0 else (n_l * n_gpus) // n
    opt, k_h = np.float32(0), 0
    if ph is not None:
        k_h = int(np.argmax(ph)) if np.max(ph) > 0 else 0
        opt = np.float32(max(np.max(ph), 0))
    sums = [(np.float32(pt[n_gpus - g]) + np.float32(pl[g]), g) for g in range(1, min(cap, n_gpus) + 1)]
    better = [(s, g) for s, g in sums if s > opt]
    if better:
        top = max(s for s, _ in better)
        g = min(g for s, g in better if s == top)
        return dict(g_t=n_gpus - g, g_l=g, heterogeneous=1, k_h=k_h, phi_opt=float(top))
    return dict(g_t=k_h, g_l=0, heterogeneous=0, k_h=k_h, phi_opt=float(opt))


def test_partition_scan_against_brute_force():
    rng = np.random.default_rng(5)
    seen = set()
    for trial in range(400):
        n_gpus = int(rng.integers(0, 40))
        # coarse values so that equal sums are common
        pt = (rng.integers(0, 6, n_gpus + 1) * 0.5).astype(np.float32)
        pl = (rng.integers(0, 6, n_gpus + 1) * 0.5).astype(np.float32)
        ph = None if trial % 3 == 0 else (rng.integers(0, 9, n_gpus + 1) * 0.5).astype(np.float32)
        n = int(rng.integers(0, 50))
        n_l = int(rng.integers(0, n + 1))
        got = oracle.resource_partition(n_gpus, pt, pl, ph, n_l, n)
        assert got == partition_brute_force(n_gpus, pt, pl, ph, n_l, n), (trial, n_gpus, n_l, n)
        seen.add(got["heterogeneous"])
    assert seen == {0, 1}


def test_initial_share_is_the_exact_floor():
    # |R_l| / |R| * |G| with a quotient that binary floating point would round across an integer
    pt = np.zeros(50, np.float32)
    pl = np.arange(50, dtype=np.float32)     # prefers the largest allowed g_l
    for n_l, n, g, cap in ((1, 3, 3, 1), (29, 29, 49, 49), (2, 3, 49, 32), (7, 49, 49, 7), (0, 5, 49, 0),
                           (10**12 - 1, 10**12, 49, 48)):
        r = oracle.resource_partition(49, pt, pl, None, n_l, n) if g == 49 else \
            oracle.resource_partition(3, pt[:4], pl[:4], None, n_l, n)
        assert r["g_l"] == cap


def test_split_by_slo_is_a_stable_selection():
    w = W.random_small(91, 1, 4, 3000, n_slo=5)
    w = W.replace(w, arrival_ticks=W.poisson_arrivals(W.rng_for(91, 3), 500.0, 3000))
    t, l = oracle.split_by_slo(w, 0b01001)
    assert t.n_req + l.n_req == w.n_req and t.n_req and l.n_req
    assert set(np.unique(t.slo_class)) <= {0, 3} and not (set(np.unique(l.slo_class)) & {0, 3})
    assert np.all(np.diff(t.arrival_ticks.astype(np.int64)) >= 0)
    assert np.all(np.diff(l.arrival_ticks.astype(np.int64)) >= 0)
    # merging the two sides back by arrival order of the original positions restores the input
    pos_t = np.nonzero(np.isin(w.slo_class, [0, 3]))[0]
    pos_l = np.nonzero(~np.isin(w.slo_class, [0, 3]))[0]
    back = np.empty(w.n_req, np.uint32)
    back[pos_t], back[pos_l] = t.prompt_len, l.prompt_len
    assert np.array_equal(back, w.prompt_len)
