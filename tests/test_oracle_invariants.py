"""Invariants that hold for any input, checked on the oracle (CPU)."""
import numpy as np
import pytest

import oracle
from paper_2509_06362_amd import workloads as W


def stressed(seed, n_cand=24, i_pad=16, n_req=2000, **kw):
    return W.random_small(seed, n_cand, i_pad, n_req, **kw)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_threshold_route_gives_the_same_counts(seed):
    w = stressed(seed, n_cand=40, n_req=3000, pen_kappa=0.5 if seed == 3 else 0.0)
    s = oracle.placement_sweep(w)
    t = oracle.threshold_sweep(w)
    assert np.array_equal(s["sat_count"], t)
    assert 0 < t.min() < t.max() < w.n_req or len(np.unique(t)) > 5


def test_threshold_route_on_config_shapes():
    for w in (W.config1(n_cand=48, n_req=4096), W.config3(n_cand=48, n_req=4096),
              W.config4(n_cand=6, n_req=4096)):
        assert np.array_equal(oracle.placement_sweep(w)["sat_count"], oracle.threshold_sweep(w))
        tight = W.stressed(w, seed=3)
        c = oracle.placement_sweep(tight)["sat_count"]
        assert np.array_equal(c, oracle.threshold_sweep(tight))
        assert len(np.unique(c)) > 1


@pytest.mark.parametrize("which", ["d_ttft", "d_tbt"])
def test_loosening_a_deadline_never_lowers_satisfaction(which):
    w = stressed(4)
    base = oracle.placement_sweep(w)["sat_count"]
    for k in range(w.n_slo):
        d = getattr(w, which).copy()
        d[k] = np.float32(d[k] * 1.5)
        more = oracle.placement_sweep(W.replace(w, **{which: d}))["sat_count"]
        assert (more >= base).all()
    assert 0 < base.mean() < w.n_req


def test_adding_an_instance_never_lowers_satisfaction():
    w = stressed(5, i_pad=12)
    n0 = np.minimum(w.n_inst, 11).astype(np.uint32)
    a = oracle.placement_sweep(W.replace(w, n_inst=n0))
    b = oracle.placement_sweep(W.replace(w, n_inst=(n0 + 1).astype(np.uint32)))
    assert (b["sat_count"] >= a["sat_count"]).all()
    assert (b["sat_count"] > a["sat_count"]).any()
    # and the distributor's best slack per request can only go up
    w1 = W.replace(w, n_inst=n0)
    w2 = W.replace(w, n_inst=(n0 + 1).astype(np.uint32))
    c = int(np.argmax(n0 > 0))
    assert (oracle.score_assign(w2, c)["slack"] >= oracle.score_assign(w1, c)["slack"]).all()


def test_request_order_does_not_matter_for_counts():
    w = stressed(6)
    perm = np.random.default_rng(0).permutation(w.n_req)
    wp = W.replace(w, prompt_len=w.prompt_len[perm].copy(), out_len=w.out_len[perm].copy(),
                   slo_class=w.slo_class[perm].copy())
    assert np.array_equal(oracle.placement_sweep(w)["sat_count"],
                          oracle.placement_sweep(wp)["sat_count"])
    a, b = oracle.score_assign(w, 3), oracle.score_assign(wp, 3)
    assert np.array_equal(a["slack"][perm], b["slack"]) and np.array_equal(a["chosen"][perm], b["chosen"])


def test_instance_order_permutes_chosen_and_keeps_slack():
    w = stressed(7, n_cand=1, i_pad=10)
    w = W.replace(w, n_inst=np.array([10], np.uint32))
    perm = np.random.default_rng(1).permutation(10)
    wp = W.replace(w, tp_idx=w.tp_idx[:, perm].copy(), max_batch=w.max_batch[:, perm].copy(),
                   occ=w.occ[:, perm].copy(), q_ticks=w.q_ticks[:, perm].copy())
    a, b = oracle.score_assign(w), oracle.score_assign(wp)
    assert np.array_equal(a["slack"], b["slack"])
    st = oracle.stage(w)
    key = np.stack([st[k] for k in ("a", "p", "tbt", "wait")], axis=1)
    same = (key[perm[b["chosen"]]] == key[a["chosen"]]).all(axis=1)   # equal up to identical twins
    assert same.all()
    assert a["n_satisfied"] == b["n_satisfied"]


def test_padding_width_does_not_matter():
    w = stressed(8, i_pad=9)
    pad = lambda x, v: np.ascontiguousarray(np.pad(x, ((0, 0), (0, 23)), constant_values=v))
    wp = W.replace(w, tp_idx=pad(w.tp_idx, 3), max_batch=pad(w.max_batch, 1), occ=pad(w.occ, 99),
                   q_ticks=pad(w.q_ticks, 12345))
    a, b = oracle.placement_sweep(w), oracle.placement_sweep(wp)
    assert np.array_equal(a["sat_count"], b["sat_count"]) and a["best_cand"] == b["best_cand"]


def test_duplicated_candidate_and_tie_break():
    w = stressed(9, n_cand=6)
    s = oracle.placement_sweep(w)
    top = s["best_cand"]
    dup = lambda x: np.ascontiguousarray(np.concatenate([x[top:top + 1], x], axis=0))
    wd = W.replace(w, n_inst=dup(w.n_inst), tp_idx=dup(w.tp_idx), max_batch=dup(w.max_batch),
                   occ=dup(w.occ), q_ticks=dup(w.q_ticks))
    sd = oracle.placement_sweep(wd)
    assert np.array_equal(sd["sat_count"][1:], s["sat_count"])
    assert sd["sat_count"][0] == s["sat_count"][top] and sd["sat_ratio"][0] == s["sat_ratio"][top]
    assert sd["best_cand"] == 0                      # lowest index among equal counts
    # identical instances: the lowest index is chosen
    c = int(np.argmax(w.n_inst > 1))
    w2 = W.replace(w.with_candidates(c, c + 1))
    for arr in (w2.tp_idx, w2.max_batch, w2.occ, w2.q_ticks):
        arr[0, 1:] = arr[0, 0]
    assert (oracle.score_assign(w2)["chosen"] == 0).all()


def test_empty_candidate_and_empty_request_set():
    w = stressed(10, n_cand=4)
    w = W.replace(w, n_inst=np.array([0, 3, 0, 5], np.uint32))
    s = oracle.placement_sweep(w)
    assert s["sat_count"][0] == 0 and s["sat_count"][2] == 0
    r = oracle.score_assign(w, 0)
    assert (r["chosen"] == -1).all() and np.isneginf(r["slack"]).all() and r["n_satisfied"] == 0
    assert np.isnan(r["ttft"]).all()
    e = w.with_requests(0, 0)
    assert oracle.score_assign(e, 1)["n_satisfied"] == 0
    assert (oracle.placement_sweep(e)["sat_count"] == 0).all()


def test_subrange_sweep_matches_full_sweep():
    w = stressed(11)
    full = oracle.placement_sweep(w)
    part = oracle.placement_sweep(w, 5, 17)
    assert np.array_equal(part["sat_count"][5:17], full["sat_count"][5:17])
    assert (part["sat_count"][:5] == 0).all()
    assert part["best_cand"] == 5 + int(np.argmax(full["sat_count"][5:17]))


def test_a_fresh_instance_adds_no_wait_to_the_first_token_latency():
    """An instance with nothing queued and a free slot has a queue wait of exactly +0, and the
    first-token latency on it is the prefill time bit for bit (L_r = L_q + L_d with L_q = 0, Eq. 2):
    what allows a fast path that leaves the addition out for such instances."""
    w = W.config1(n_cand=6, n_req=64)
    rng = np.random.default_rng(7)
    for c in range(w.n_cand):
        st = oracle.stage(w, c)
        assert np.all(st["wait"] == 0.0) and not np.any(np.signbit(st["wait"]))
        for j in rng.choice(len(st["a"]), 3):
            for L in (0, 1, 17, 8192, 16777215):
                t = oracle.triple(st["a"][j], st["p"][j], st["tbt"][j], st["wait"][j], L, 100, 0.5, 0.05)
                pre = np.float32(np.float64(st["p"][j]) * np.float64(L) + np.float64(st["a"][j]))  # one rounding
                assert t["pre"] == pre and t["ttft"] == t["pre"] and t["pre"] > 0
    # with load it is not: queued prefill shows up in the wait
    loaded = W.stressed(w, seed=3)
    assert np.all(oracle.stage(loaded, 0)["wait"] > 0.0)
