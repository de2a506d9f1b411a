"""Pins of the oracle's least-squares fit of the throughput-decay function (Sec. IV-B, Eq. 1)."""
import numpy as np
import pytest
from scipy.optimize import least_squares

import oracle
from oracle.profile_fit import fit_one, line_fit
from paper_2509_06362_amd import workloads as W


def sse_of(params, w, y):
    t0, delta, eps = params
    return float(((t0 * (1.0 - delta * np.log(eps + w)) - y) ** 2).sum())


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


def test_line_fit_is_the_linear_least_squares_solution():
    rng = np.random.default_rng(2)
    w = rng.uniform(1, 128, 40)
    y = 100 * (1 - 0.1 * np.log(2.0 + w)) + rng.normal(0, 1, 40)
    for eps in (0.01, 2.0, 300.0):
        alpha, beta, sse = line_fit(w, y, eps)
        A = np.stack([np.ones_like(w), -np.log(eps + w)], axis=1)
        sol, res, *_ = np.linalg.lstsq(A, y, rcond=None)
        assert np.allclose([alpha, beta], sol, rtol=1e-9)
        assert sse == pytest.approx(float(res[0]), rel=1e-9)


@pytest.mark.parametrize("seed,noise", [(3, 0.02), (4, 0.05), (5, 0.002), (6, 0.1)])
def test_no_better_fit_exists(seed, noise):
    """The residual at the oracle's answer is a minimum: a dense scan over eps does not beat it, a
    three-parameter Gauss-Newton refinement started there does not move, and started elsewhere it
    does not end lower."""
    off, lv, th, _ = W.throughput_samples(seed, noise=noise, repeats=4)
    params, _, ok = oracle.profile_fit(off, lv, th, 64)
    assert ok
    for t in range(len(off) - 1):
        w = lv[off[t]:off[t + 1]].astype(np.float64)
        y = th[off[t]:off[t + 1]].astype(np.float64)
        t0, delta, eps, sse = params[t]
        assert sse == pytest.approx(sse_of((t0, delta, eps), w, y), rel=1e-9)
        dense = min(line_fit(w, y, e)[2] for e in np.exp(np.linspace(np.log(2.0 ** -10), np.log(2.0 ** 10), 20001)))
        assert sse <= dense * (1 + 1e-12)
        if 2.0 ** -10 * 1.01 < eps < 2.0 ** 10 * 0.99:           # interior minimum: stationary point
            res = lambda p: p[0] * (1 - p[1] * np.log(p[2] + w)) - y  # noqa: E731
            here = least_squares(res, [t0, delta, eps], xtol=1e-14, ftol=1e-14, gtol=1e-14)
            assert 2 * here.cost >= sse * (1 - 1e-9)
            assert np.allclose(here.x, [t0, delta, eps], rtol=1e-4)
            for start in ([y.max(), 0.1, 1.0], [2 * y.max(), 0.05, 10.0]):
                other = least_squares(res, start, bounds=([0, 0, 2.0 ** -10], [np.inf, 1, 2.0 ** 10]))
                assert 2 * other.cost >= sse * (1 - 1e-9)


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
