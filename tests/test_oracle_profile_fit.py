"""Pins of the oracle's least-squares fit of the throughput-decay function (Sec. IV-B, Eq. 1).

The oracle is the definition (the parameters that minimise the squared residual); what fixes it from
outside: noiseless samples return the parameters that generated them, no point of a brute-force grid
around the answer or over the whole box has a smaller residual, the residual at the generating
parameters is never below the fitted one, and the answer does not depend on where a search starts."""
import numpy as np
import pytest
from scipy.optimize import least_squares

import oracle
from oracle.profile_fit import fit_one
from paper_2509_06362_amd import workloads as W


def sse_of(params, w, y):
    t0, delta, eps = params
    return float(((t0 * (1.0 - delta * np.log(eps + w)) - y) ** 2).sum())


def samples_of(off, lv, th, t):
    return lv[off[t]:off[t + 1]].astype(np.float64), th[off[t]:off[t + 1]].astype(np.float64)


def test_noiseless_samples_give_the_parameters_back():
    off, lv, th, truth = W.throughput_samples(1, noise=0.0)
    params, tbt, ok = oracle.profile_fit(off, lv, th, 128)
    assert ok
    assert np.allclose(params[:, :3], truth, rtol=2e-5)       # samples are rounded to binary32
    b = np.arange(1, 129)
    for t in range(4):
        f = truth[t, 0] * (1 - truth[t, 1] * np.log(truth[t, 2] + b))
        assert np.allclose(tbt[t, 1:], 1.0 / f, rtol=1e-6)
    assert np.isnan(tbt[:, 0]).all()


def test_a_hand_made_exact_case():
    """Three samples on F(w) = 64 * (1 - 0.125 * log(1 + w)) at w = 1, 3, 7, i.e. log 2, 2 log 2, 3 log 2:
    y = 64 - 8 k log 2.  Three parameters, three points: the residual must vanish there."""
    w = np.array([1.0, 3.0, 7.0])
    y = 64.0 - 8.0 * np.log(2.0) * np.array([1.0, 2.0, 3.0])
    t0, delta, eps, res = fit_one(w, y, 2.0 ** -10, 2.0 ** 10)
    assert res < 1e-18
    assert np.allclose([t0, delta, eps], [64.0, 0.125, 1.0], rtol=1e-7)


@pytest.mark.parametrize("seed,noise", [(3, 0.02), (4, 0.05), (5, 0.002), (6, 0.1)])
def test_no_better_fit_exists(seed, noise):
    off, lv, th, truth = W.throughput_samples(seed, noise=noise, repeats=4)
    params, _, ok = oracle.profile_fit(off, lv, th, 64)
    assert ok
    rng = np.random.default_rng(seed)
    for t in range(len(off) - 1):
        w, y = samples_of(off, lv, th, t)
        t0, delta, eps, res = params[t]
        assert res == pytest.approx(sse_of((t0, delta, eps), w, y), rel=1e-12)
        # the generating parameters are one admissible point
        assert res <= sse_of(truth[t], w, y)
        # brute force, local: no neighbour on a 3-D grid of relative steps is better
        for step in (1e-2, 1e-4, 1e-6):
            for d0 in (-1, 0, 1):
                for d1 in (-1, 0, 1):
                    for d2 in (-1, 0, 1):
                        p = (t0 * (1 + d0 * step), delta * (1 + d1 * step), eps * (1 + d2 * step))
                        if 2.0 ** -10 <= p[2] <= 2.0 ** 10:           # eps is bounded
                            assert sse_of(p, w, y) >= res * (1 - 1e-12)
        # brute force, global: random points of the whole box, each polished in (T0, delta) by the
        # normal equations written out here
        for le in rng.uniform(np.log(2.0 ** -10), np.log(2.0 ** 10), 300):
            x = -np.log(np.exp(le) + w)
            n = len(w)
            sx, sy, sxx, sxy = x.sum(), y.sum(), (x * x).sum(), (x * y).sum()
            beta = (n * sxy - sx * sy) / (n * sxx - sx * sx)
            alpha = (sy - beta * sx) / n
            assert sse_of((alpha, beta / alpha, np.exp(le)), w, y) >= res * (1 - 1e-9)
        # a search started elsewhere does not end lower
        if 2.0 ** -10 * 1.01 < eps < 2.0 ** 10 * 0.99:
            fun = lambda p: p[0] * (1 - p[1] * np.log(p[2] + w)) - y  # noqa: E731
            for start in ([y.max(), 0.1, 1.0], [2 * y.max(), 0.05, 10.0]):
                other = least_squares(fun, start, bounds=([0, 0, 2.0 ** -10], [np.inf, 1, 2.0 ** 10]))
                assert 2 * other.cost >= res * (1 - 1e-9)


def test_eps_at_a_bound():
    """Samples whose best eps lies below the lower bound: the fit stays inside and lands on it."""
    off, lv, th, _ = W.throughput_samples(8, noise=0.0, truth=[[100.0, 0.1, 2.0 ** -14]])
    t0, delta, eps, res = fit_one(*samples_of(off, lv, th, 0), 2.0 ** -10, 2.0 ** 10)
    assert eps == pytest.approx(2.0 ** -10, rel=1e-9)
    assert np.allclose([t0, delta], [100.0, 0.1], rtol=1e-3)


def test_degenerate_inputs():
    # two samples cannot determine three parameters
    p = fit_one([1, 2], [10, 9], 2.0 ** -10, 2.0 ** 10)
    assert all(np.isnan(v) for v in p)
    # all samples at one level: no slope
    params, tbt, ok = oracle.profile_fit(np.array([0, 4], np.uint32), np.full(4, 8, np.float32),
                                         np.array([50, 51, 49, 50], np.float32), 8)
    assert not ok
    # a decay so steep that F(b) reaches zero inside the table
    off, lv, th, _ = W.throughput_samples(7, levels=(1, 2, 4, 8), noise=0.0, truth=[[100.0, 0.3, 1.0]])
    params, tbt, ok = oracle.profile_fit(off, lv, th, 64)       # 1 - 0.3 log(1 + 64) < 0
    assert not ok and (tbt[0, 1:9] > 0).all()
