"""Pins of the oracle's arithmetic against closed forms in float64 and hand-checkable values."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2509_06362_amd import workloads as W
from tests.model64 import profile64, stage64, triple64

TP = [1, 2, 4, 8]


def one_instance(tp_i, B, occ, q=0, n_req=64, seed=11, kappa=0.0, b_cap=64):
    w = W.config0(n_req=n_req, seed=seed)
    a, p, t = W.profile_tables(b_cap)
    return W.replace(
        w, b_cap=b_cap, prefill_a=a, prefill_p=p, tbt=t,
        n_inst=np.array([1], np.uint32), tp_idx=np.array([[tp_i]], np.uint8),
        max_batch=np.array([[B]], np.uint16), occ=np.array([[occ]], np.int32),
        q_ticks=np.array([[q]], np.uint64), pen_kappa=np.float32(kappa))


def test_hand_values_of_the_synthetic_profile():
    # TP=1, one request in the batch: a = 0.02, p = 4e-5, tbt = 0.012 * 1.03.
    # A 1000-token prompt prefills in 0.02 + 0.04 = 0.06 s.
    w = one_instance(0, 8, 0)
    st = oracle.stage(w)
    assert st["a"][0] == np.float32(0.02) and st["p"][0] == np.float32(4e-5)
    assert st["tbt"][0] == np.float32(0.01236)
    assert st["wait"][0] == 0.0
    t = oracle.triple(st["a"][0], st["p"][0], st["tbt"][0], 0.0, 1000, 100, 0.5, 0.05)
    assert t["pre"] == pytest.approx(0.06, rel=1e-6)
    assert t["ttft"] == pytest.approx(0.06, rel=1e-6)
    assert t["e2e"] == pytest.approx(0.06 + 100 * 0.01236, rel=1e-6)       # 1.296 s
    assert t["s1"] == pytest.approx((0.5 - 0.06) / 0.5, rel=1e-5)            # 0.88
    assert t["s2"] == pytest.approx((0.05 - 0.01236) / 0.05, rel=1e-5)       # 0.7528
    assert t["s3"] == pytest.approx((5.5 - 1.296) / 5.5, rel=1e-5)           # De = 0.5 + 100*0.05
    assert t["slack"] == pytest.approx(0.7528, rel=1e-5)
    # TP=8 at batch 64: 8^0.8 = 2^2.4, 8^0.85 = 2^2.55, 8^0.7 = 2^2.1
    w = one_instance(3, 64, 63)
    st = oracle.stage(w)
    assert st["a"][0] == pytest.approx(0.02 / 2**2.4, rel=1e-6)
    assert st["p"][0] == pytest.approx(4e-5 / 2**2.55, rel=1e-6)
    assert st["tbt"][0] == pytest.approx(0.012 / 2**2.1 * (1 + 0.03 * 64), rel=1e-6)


@pytest.mark.parametrize("tp_i,B,occ", [(0, 8, 0), (0, 8, 7), (1, 16, 3), (2, 32, 31), (3, 64, 10),
                                         (3, 4, 2), (1, 1, 0)])
def test_single_instance_matches_closed_form(tp_i, B, occ):
    w = one_instance(tp_i, B, occ, n_req=256)
    r = oracle.score_assign(w)
    a, p, tbt, wait = stage64(TP[tp_i], B, occ, 0, float(w.s_bar))
    assert wait == 0.0
    for i in range(w.n_req):
        k = w.slo_class[i]
        m = triple64(a, p, tbt, wait, float(w.prompt_len[i]), float(w.out_len[i]),
                     float(w.d_ttft[k]), float(w.d_tbt[k]))
        assert r["chosen"][i] == 0
        assert r["ttft"][i] == pytest.approx(m["ttft"], rel=2e-6)
        assert r["e2e"][i] == pytest.approx(m["e2e"], rel=2e-6)
        assert r["tbt"][i] == pytest.approx(tbt, rel=2e-6)
        assert r["slack"][i] == pytest.approx(m["slack"], rel=1e-5, abs=2e-6)
    n_ok = sum(triple64(a, p, tbt, wait, float(L), float(S), float(w.d_ttft[k]),
                        float(w.d_tbt[k]))["slack"] >= 0
               for L, S, k in zip(w.prompt_len, w.out_len, w.slo_class))
    assert r["n_satisfied"] == n_ok


@pytest.mark.parametrize("occ,q,kappa,worst", [(9, 0, 0.0, False), (20, 0, 0.0, False),
                                                (3, 700_000, 0.0, False), (7, 123_457, 0.5, False),
                                                (30, 5_000_001, 0.5, False), (2, 0, 0.5, True),
                                                (5, 40_000_000, 0.0, True), (6, 0, 0.5, False)])
def test_queue_wait_penalty_and_worst_case_mode(occ, q, kappa, worst):
    # B = 8 on TP=2: occupancy past the cap queues, fill above 75 % is penalised,
    # worst-case mode reads the row of the full batch.
    B = 8
    w = one_instance(1, B, occ, q=q, n_req=128, kappa=kappa)
    st = oracle.stage(w, tbt_mode=1 if worst else 0)
    a, p, tbt, wait = stage64(2, B, occ, q, float(w.s_bar), kappa=kappa, worst=worst)
    assert st["a"][0] == pytest.approx(a, rel=1e-6)
    assert st["p"][0] == pytest.approx(p, rel=1e-6)
    assert st["tbt"][0] == pytest.approx(tbt, rel=1e-6)
    assert st["svc"][0] == pytest.approx(float(w.s_bar) * tbt, rel=1e-6)
    assert st["wait"][0] == pytest.approx(wait, rel=1e-6)
    r = oracle.score_assign(w, tbt_mode=1 if worst else 0)
    for i in range(w.n_req):
        k = w.slo_class[i]
        m = triple64(a, p, tbt, wait, float(w.prompt_len[i]), float(w.out_len[i]),
                     float(w.d_ttft[k]), float(w.d_tbt[k]))
        assert r["ttft"][i] == pytest.approx(m["ttft"], rel=2e-6)
        assert r["slack"][i] == pytest.approx(m["slack"], rel=1e-5, abs=2e-6)


def test_truncation_at_the_batch_cap():
    # Eq. 1 depends on min(B, W): beyond the cap the per-token latency stops changing,
    # only the queue wait grows.
    base = oracle.stage(one_instance(2, 16, 15))
    for occ in (16, 17, 40, 1000):
        st = oracle.stage(one_instance(2, 16, occ))
        assert st["tbt"][0] == base["tbt"][0] and st["a"][0] == base["a"][0]
        assert st["wait"][0] > 0
    w1 = oracle.stage(one_instance(2, 16, 17))["wait"][0]
    w2 = oracle.stage(one_instance(2, 16, 33))["wait"][0]
    assert w2 == pytest.approx(w1 * 18 / 2, rel=1e-6)  # (occ+1-B)/B: 2/16 vs 18/16


def test_end_to_end_margin_is_implied_by_the_other_two():
    # S*tbt + ttft <= S*Db + Dt whenever ttft <= Dt and tbt <= Db, and rounding is monotone.
    w = W.random_small(5, 8, 16, 512, pen_kappa=0.5)
    for c in range(w.n_cand):
        st = oracle.stage(w, c)
        for j, i in itertools.product(range(len(st["a"])), range(0, w.n_req, 7)):
            k = w.slo_class[i]
            t = oracle.triple(st["a"][j], st["p"][j], st["tbt"][j], st["wait"][j],
                              w.prompt_len[i], w.out_len[i], w.d_ttft[k], w.d_tbt[k])
            if t["s1"] >= 0 and t["s2"] >= 0:
                assert t["s3"] >= 0
            assert t["slack"] == min(t["s1"], t["s2"], t["s3"])
            assert (t["s1"] >= 0) == (t["ttft"] <= w.d_ttft[k])
            assert (t["s2"] >= 0) == (st["tbt"][j] <= w.d_tbt[k])


def test_equality_at_a_deadline_is_satisfied():
    # Eq. 3 uses <=.  Exactly representable numbers: a = 0.25, p = 2^-10, L = 256 -> ttft = 0.5.
    w = one_instance(0, 4, 0, n_req=2)
    a = np.full_like(w.prefill_a, 0.25); p = np.full_like(w.prefill_p, 2.0**-10)
    t = np.full_like(w.tbt, 2.0**-6)
    w = W.replace(w, prefill_a=a, prefill_p=p, tbt=t, prompt_len=np.array([256, 257], np.uint32),
                  out_len=np.array([64, 64], np.uint32), slo_class=np.array([0, 0], np.uint8),
                  d_ttft=np.array([0.5], np.float32), d_tbt=np.array([2.0**-6], np.float32))
    r = oracle.score_assign(w)
    assert r["ttft"][0] == 0.5 and r["slack"][0] == 0.0
    assert r["slack"][1] < 0 and r["chosen"][1] == 0       # best instance is reported even if blocked
    assert r["n_satisfied"] == 1
    s = oracle.placement_sweep(w)
    assert s["sat_count"][0] == 1 and s["sat_ratio"][0] == 0.5


def test_bad_profiles_are_rejected():
    w = one_instance(0, 4, 0)
    bad = w.tbt.copy(); bad[2, 5] = 0.0
    with pytest.raises(ValueError):
        oracle.score_assign(W.replace(w, tbt=bad))
    with pytest.raises(ValueError):
        oracle.placement_sweep(W.replace(w, d_ttft=np.array([0.5, np.inf, 1.0], np.float32)))
