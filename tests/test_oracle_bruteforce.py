"""Brute-force pins: every assignment of a tiny request set, every placement of a tiny budget."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2509_06362_amd import workloads as W
from tests.model64 import stage64, triple64

TP = [1, 2, 4, 8]
MARGIN = 1e-5  # cases closer than this to a deadline in float64 are regenerated


def tiny(seed, n_inst, n_req, tight=1.0):
    rng = np.random.default_rng(seed)
    a, p, t = W.profile_tables(16)
    d_ttft, d_tbt = W.slo_three_classes()
    tp_idx = rng.integers(0, 4, size=(1, n_inst)).astype(np.uint8)
    B = rng.choice([2, 4, 8, 16], size=(1, n_inst)).astype(np.uint16)
    occ = np.floor(rng.random((1, n_inst)) * B * 1.5).astype(np.int32)
    q = rng.integers(0, 1 << 19, size=(1, n_inst)).astype(np.uint64)
    out = W.log_uniform_int(rng, 8, 512, n_req)
    return W.Workload(
        name="tiny", seed=seed, tp_degree=W.TP_DEGREES.copy(), b_cap=16, prefill_a=a, prefill_p=p,
        tbt=t, d_ttft=(d_ttft * tight).astype(np.float32), d_tbt=(d_tbt * tight).astype(np.float32),
        prompt_len=W.log_uniform_int(rng, 16, 16384, n_req), out_len=out,
        slo_class=rng.integers(0, 3, size=n_req).astype(np.uint8), arrival_ticks=None,
        n_inst=np.array([n_inst], np.uint32), tp_idx=tp_idx, max_batch=B, occ=occ, q_ticks=q,
        s_bar=W.mean_out_len(out))


def margins64(w, c=0):
    """[R, I] float64 slack of every triple of candidate c, straight from the closed forms."""
    n = int(w.n_inst[c])
    m = np.empty((w.n_req, n))
    for j in range(n):
        a, p, tbt, wait = stage64(TP[w.tp_idx[c, j]], int(w.max_batch[c, j]), int(w.occ[c, j]),
                                  int(w.q_ticks[c, j]), float(w.s_bar), float(w.pen_kappa))
        for r in range(w.n_req):
            k = w.slo_class[r]
            m[r, j] = triple64(a, p, tbt, wait, float(w.prompt_len[r]), float(w.out_len[r]),
                               float(w.d_ttft[k]), float(w.d_tbt[k]))["slack"]
    return m


def clear_of_boundaries(m):
    if m.size == 0:
        return True
    srt = np.sort(m, axis=1)
    gaps_ok = True if m.shape[1] < 2 else (np.diff(srt, axis=1) > MARGIN).all()
    return (np.abs(m) > MARGIN).all() and gaps_ok


@pytest.mark.parametrize("seed", range(12))
def test_every_assignment_of_a_tiny_request_set(seed):
    n_inst, n_req = 1 + seed % 3, 3 + seed % 4
    w, m = None, None
    for attempt in range(20):
        w = tiny(1000 * attempt + seed, n_inst, n_req, tight=[1.0, 0.5, 0.2][seed % 3])
        m = margins64(w)
        if clear_of_boundaries(m):
            break
    else:
        pytest.fail("no clear case")
    ok = m >= 0
    best = -1
    # an assignment maps each request to one instance or to "blocked" (index n_inst)
    for assign in itertools.product(range(n_inst + 1), repeat=n_req):
        served = sum(1 for r, j in enumerate(assign) if j < n_inst and ok[r, j])
        best = max(best, served)
    r = oracle.score_assign(w)
    assert r["n_satisfied"] == best
    assert (r["chosen"] == m.argmax(axis=1)).all()
    assert np.allclose(r["slack"], m.max(axis=1), rtol=1e-4, atol=2e-6)
    assert oracle.placement_sweep(w)["sat_count"][0] == best


def multisets(budget, batch_sizes):
    """All multisets of (tp_idx, B) whose TP degrees sum to the budget."""
    kinds = [(t, b) for t in range(4) for b in batch_sizes]

    def rec(start, left):
        if left == 0:
            yield []
            return
        for i in range(start, len(kinds)):
            d = TP[kinds[i][0]]
            if d <= left:
                for rest in rec(i, left - d):
                    yield [kinds[i]] + rest
    return list(rec(0, budget))


@pytest.mark.parametrize("budget,seed", [(4, 0), (6, 1), (8, 2)])
def test_every_placement_of_a_tiny_budget(budget, seed):
    cands = multisets(budget, [4, 8])
    i_pad = budget
    rng = np.random.default_rng(seed)
    n_req = 24
    a, p, t = W.profile_tables(8)
    out = W.log_uniform_int(rng, 8, 2048, n_req)
    C = len(cands)
    tp_idx = np.zeros((C, i_pad), np.uint8); B = np.ones((C, i_pad), np.uint16)
    occ = np.zeros((C, i_pad), np.int32)
    for c, inst in enumerate(cands):
        for j, (ti, b) in enumerate(inst):
            tp_idx[c, j], B[c, j] = ti, b
            occ[c, j] = (7 * c + 3 * j) % (b + 3)          # some instances past their cap
    w = W.Workload(
        name="tiny_placements", seed=seed, tp_degree=W.TP_DEGREES.copy(), b_cap=8, prefill_a=a,
        prefill_p=p, tbt=t, d_ttft=np.array([0.12, 0.3, 1.5], np.float32),
        d_tbt=np.array([0.009, 0.0135, 0.05], np.float32),
        prompt_len=W.log_uniform_int(rng, 16, 16384, n_req), out_len=out,
        slo_class=rng.integers(0, 3, size=n_req).astype(np.uint8), arrival_ticks=None,
        n_inst=np.array([len(x) for x in cands], np.uint32), tp_idx=tp_idx, max_batch=B, occ=occ,
        q_ticks=np.zeros((C, i_pad), np.uint64), s_bar=W.mean_out_len(out))
    counts = np.zeros(C, np.int64)
    clear = np.ones(C, bool)
    for c in range(C):
        m = margins64(w, c)
        clear[c] = (np.abs(m) > MARGIN).all()
        counts[c] = (m >= 0).any(axis=1).sum()
    s = oracle.placement_sweep(w)
    assert clear.mean() > 0.9
    assert (s["sat_count"][clear] == counts[clear]).all()
    assert len(np.unique(counts)) > 1, "the case must discriminate between placements"
    if clear.all():
        assert s["best_cand"] == int(np.argmax(counts))       # first maximum = lowest index
    assert np.allclose(s["sat_ratio"], s["sat_count"] / n_req, rtol=1e-6)
    assert s["sat_count"][s["best_cand"]] == s["sat_count"].max()
    assert s["best_cand"] == int(np.argmax(s["sat_count"]))
