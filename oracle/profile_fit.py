"""CPU oracle of the profiler's least-squares fit.  TEST INFRASTRUCTURE ONLY.

Throughput-decay function (Sec. IV-B, Eq. 1): F(w) = T0 * (1 - delta * log(eps + w)), w = min(B, W).
The paper fits it to a limited set of throughput measurements by least squares.  This oracle is that
definition written out: the parameters (T0, delta, eps), eps within the given bounds, that minimise

    SSE(T0, delta, eps) = sum_i (F(w_i) - y_i)^2 .

How the minimum is found is of no concern to the definition; here: the residual with (T0, delta)
solved for by linear least squares (numpy.linalg.lstsq - for a fixed eps the model is linear in T0
and T0*delta) is scanned densely over log(eps) to find the basin of the global minimum, and the
three parameters are then refined together from there by scipy.optimize.least_squares on the
residual vector F(w_i) - y_i with its analytic Jacobian, eps bounded.  Plain numpy/scipy, binary64,
one strategy at a time.  The natural logarithm is taken ("logarithmic decay", base unstated).

With fewer than three samples, or samples at fewer than two distinct workload levels, the fit is
undefined (NaN).  With exactly two distinct levels the minimum is not unique in eps (every eps gives
the same residual), so a comparison with another implementation is meaningless there.
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import least_squares

SCAN_POINTS = 4001


def model(params, w):
    t0, delta, eps = params
    return t0 * (1.0 - delta * np.log(eps + w))


def sse(params, w, y):
    r = model(params, w) - y
    return float(r @ r)


def _linear_part(w, y, eps):
    """(T0, T0*delta) minimising the residual for a fixed eps, and that residual."""
    a = np.stack([np.ones_like(w), -np.log(eps + w)], axis=1)
    sol, *_ = np.linalg.lstsq(a, y, rcond=None)
    r = a @ sol - y
    return sol, float(r @ r)


def fit_one(w, y, eps_lo, eps_hi):
    """(T0, delta, eps, sse) of one strategy's samples."""
    w = np.asarray(w, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    if len(w) < 3 or len(np.unique(w)) < 2:
        return (np.nan,) * 4
    lo, hi = np.log(np.float64(eps_lo)), np.log(np.float64(eps_hi))
    scan = np.linspace(lo, hi, SCAN_POINTS)
    res = [_linear_part(w, y, np.exp(le)) for le in scan]
    i = int(np.argmin([r[1] for r in res]))
    (alpha, beta), _ = res[i]
    if not np.isfinite(alpha) or alpha == 0.0:
        return (np.nan,) * 4

    def residuals(p):                       # p = (T0, delta, log eps)
        return p[0] * (1.0 - p[1] * np.log(np.exp(p[2]) + w)) - y

    def jacobian(p):
        e = np.exp(p[2])
        lg = np.log(e + w)
        return np.stack([1.0 - p[1] * lg, -p[0] * lg, -p[0] * p[1] * e / (e + w)], axis=1)

    out = least_squares(residuals, np.array([alpha, beta / alpha, scan[i]]), jac=jacobian,
                        bounds=([-np.inf, -np.inf, lo], [np.inf, np.inf, hi]),
                        xtol=1e-15, ftol=1e-15, gtol=1e-15, x_scale="jac")
    t0, delta, le = out.x
    eps = float(np.exp(le))
    return float(t0), float(delta), eps, sse((t0, delta, eps), w, y)


def profile_fit(offsets, level, thr, b_cap, eps_lo=2.0 ** -10, eps_hi=2.0 ** 10):
    """All strategies: params [T, 4] float64 (T0, delta, eps, sse), tbt [T, b_cap + 1] float32 with
    tbt[t, b] = 1 / F_t(b) and column 0 NaN, ok (False when some F_t(b) <= 0 or a fit is undefined)."""
    n_tp = len(offsets) - 1
    params = np.full((n_tp, 4), np.nan)
    tbt = np.full((n_tp, b_cap + 1), np.nan, dtype=np.float32)
    ok = True
    b = np.arange(1, b_cap + 1, dtype=np.float64)
    for t in range(n_tp):
        s = slice(int(offsets[t]), int(offsets[t + 1]))
        t0, delta, eps, res = fit_one(level[s], thr[s], eps_lo, eps_hi)
        params[t] = (t0, delta, eps, res)
        if not np.isfinite(t0) or not t0 > 0:
            ok = False
            continue
        f = model((t0, delta, eps), b)
        ok = ok and bool((f > 0).all())
        with np.errstate(divide="ignore"):
            tbt[t, 1:] = (1.0 / f).astype(np.float32)
    return params, tbt, ok
