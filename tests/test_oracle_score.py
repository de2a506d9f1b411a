"""Pins of the composite serving score (Eq. 6-8) as the oracle computes it."""
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2509_06362_amd import workloads as W
from tests.model64 import stage64, triple64
from tests.test_oracle_window import read_golden, worked_example_workload

GOLDEN = Path(__file__).parent / "golden" / "score_worked_example.txt"
TP = [1, 2, 4, 8]


def read_score_golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split(":")
        out[k.strip()] = float(v)
    return out


def test_hand_worked_score():
    g = read_score_golden()
    w = worked_example_workload(read_golden())
    r = oracle.placement_score(w, g["alpha"], g["beta"], g["gamma_t"], g["gamma_l"], window=w.window)
    assert r["sat_count"][0] == g["sat_count"]
    assert r["phi_t"][0] == g["phi_t"]
    assert r["phi_s"][0] == pytest.approx(g["phi_s"], rel=1e-6)
    assert r["phi_l"][0] == pytest.approx(g["phi_l"], rel=1e-6)
    assert r["score"][0] == pytest.approx(g["score"], rel=1e-6)


def score64(w, c, alpha, beta, gamma_t, gamma_l):
    """Static score of candidate c in float64, straight from the closed forms; also returns the
    smallest distance of any margin to zero or to a competing margin."""
    n = int(w.n_inst[c])
    st = [stage64(TP[w.tp_idx[c, j]], int(w.max_batch[c, j]), int(w.occ[c, j]), int(w.q_ticks[c, j]),
                  float(w.s_bar), float(w.pen_kappa)) for j in range(n)]
    used, waits, sat, clear = set(), 0.0, 0, np.inf
    for r in range(w.n_req):
        k = w.slo_class[r]
        m = [triple64(*st[j], float(w.prompt_len[r]), float(w.out_len[r]), float(w.d_ttft[k]),
                      float(w.d_tbt[k]))["slack"] for j in range(n)]
        if not m:
            continue
        order = np.argsort(m)[::-1]
        j = int(order[0])
        clear = min(clear, abs(m[j]), (m[j] - m[order[1]]) if n > 1 else np.inf)
        if m[j] >= 0:
            sat += 1; used.add(j); waits += st[j][3]
    ps = sat / w.n_req
    pt = sum(1.0 / st[j][2] for j in used)
    pl = waits / sat if sat else 0.0
    return dict(sat=sat, phi_s=ps, phi_t=pt, phi_l=pl, clear=clear,
                score=alpha * ps + beta * min(pt, gamma_t) / gamma_t
                + (1 - beta) * max(gamma_l - pl, 0) / gamma_l)


def test_static_score_matches_float64_definitions():
    w = W.random_small(71, 12, 6, 60, jitter=False, pen_kappa=0.5)
    w = W.replace(w, n_inst=np.maximum(w.n_inst, 1).astype(np.uint32))
    a, b, gt, gl = 4.0, 0.3, 300.0, 3.0
    r = oracle.placement_score(w, a, b, gt, gl)
    checked = 0
    for c in range(w.n_cand):
        m = score64(w, c, a, b, gt, gl)
        if m["clear"] < 1e-5:
            continue
        checked += 1
        assert r["sat_count"][c] == m["sat"]
        assert r["phi_s"][c] == pytest.approx(m["phi_s"], rel=1e-6)
        assert r["phi_t"][c] == pytest.approx(m["phi_t"], rel=1e-5)
        assert r["phi_l"][c] == pytest.approx(m["phi_l"], rel=1e-4, abs=2e-6)
        assert r["score"][c] == pytest.approx(m["score"], rel=1e-5)
    assert checked >= 8
    assert len(np.unique(r["sat_count"])) > 2


def test_score_structure():
    w = W.stressed(W.config1(n_cand=40, n_req=1500), seed=6)
    base = oracle.placement_score(w, 4.0, 0.3, 400.0, 2.0)
    sweep = oracle.placement_sweep(w)
    assert np.array_equal(base["sat_count"], sweep["sat_count"])
    assert np.array_equal(base["phi_s"], sweep["sat_ratio"])
    # one window over everything is the static score
    wa = W.replace(w, arrival_ticks=W.poisson_arrivals(W.rng_for(6, 3), 1000.0, w.n_req))
    one = oracle.placement_score(wa, 4.0, 0.3, 400.0, 2.0, window=w.n_req)
    for k in ("sat_count", "phi_s", "phi_t", "phi_l", "score"):
        assert np.array_equal(base[k], one[k]), k
    # alpha weighs the satisfaction ratio only
    more = oracle.placement_score(w, 5.0, 0.3, 400.0, 2.0)
    assert np.allclose(more["score"] - base["score"], base["phi_s"], atol=2e-6)
    # beta = 1 ignores the latency term, beta = 0 the throughput term
    b1 = oracle.placement_score(w, 4.0, 1.0, 400.0, 2.0)
    b1_other = oracle.placement_score(w, 4.0, 1.0, 400.0, 50.0)
    assert np.array_equal(b1["score"], b1_other["score"])
    b0 = oracle.placement_score(w, 4.0, 0.0, 400.0, 2.0)
    b0_other = oracle.placement_score(w, 4.0, 0.0, 9000.0, 2.0)
    assert np.array_equal(b0["score"], b0_other["score"])
    # normalised terms stay within [0, 1]
    assert (base["score"] <= 4.0 * base["phi_s"] + 1.0 + 1e-6).all()
    assert (base["score"] >= 4.0 * base["phi_s"] - 1e-6).all()
    # the best candidate is the first maximum
    assert base["best_cand"] == int(np.argmax(base["score"]))
    # an instance no request can use (its per-token latency misses every class) adds no throughput
    c = int(np.argmax(w.n_inst < w.i_pad))
    j = int(w.n_inst[c])
    slow = W.replace(w, n_inst=w.n_inst.copy(), tp_idx=w.tp_idx.copy(), max_batch=w.max_batch.copy(),
                     occ=w.occ.copy())
    slow.n_inst[c] += 1
    slow.tp_idx[c, j] = 0; slow.max_batch[c, j] = 128; slow.occ[c, j] = 127   # TP1 at batch 128: 58 ms
    s2 = oracle.placement_score(slow, 4.0, 0.3, 400.0, 2.0)
    assert s2["phi_t"][c] == base["phi_t"][c] and s2["score"][c] == base["score"][c]


def test_score_windowed_counts_match_the_windowed_sweep():
    w = W.stressed(W.config4(n_cand=6, n_req=4096), seed=2)
    a = oracle.placement_score(w, 4.0, 0.3, 3000.0, 5.0, window=512)
    b = oracle.placement_sweep_windowed(w, window=512)
    assert np.array_equal(a["sat_count"], b["sat_count"]) and np.array_equal(a["phi_s"], b["sat_ratio"])
    with pytest.raises(ValueError):
        oracle.placement_score(w, 4.0, 0.3, 0.0, 5.0)
