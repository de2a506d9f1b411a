"""CPU oracle of the profiler's least-squares fit.  TEST INFRASTRUCTURE ONLY.

Throughput-decay function (Sec. IV-B, Eq. 1): F(w) = T0 * (1 - delta * log(eps + w)), w = min(B, W).
The paper fits it to a limited set of throughput measurements by least squares and does not name a
method; the reading taken here: for a fixed eps the model is the straight line y = alpha - beta * x in
x = log(eps + w) (alpha = T0, beta = T0 * delta), fitted in closed form; eps minimises the remaining
residual and is found by nested grid search on log(eps) - 256 points between the bounds, keep the best
(lowest index on ties), continue between its two neighbours, 10 levels, answer = centre of the last
bracket.  Plain numpy, binary64, one strategy at a time.
"""
from __future__ import annotations

import numpy as np

GRID = 256
LEVELS = 10


def line_fit(w, y, eps):
    """Least-squares straight line through (log(eps + w_i), y_i): (alpha, beta, sse)."""
    x = np.log(eps + w)
    mx, my = x.sum() / len(x), y.sum() / len(y)
    dx, dy = x - mx, y - my
    sxx, sxy, syy = (dx * dx).sum(), (dx * dy).sum(), (dy * dy).sum()
    if not sxx > 0.0:
        return np.nan, np.nan, np.inf
    slope = sxy / sxx
    return my - slope * mx, -slope, syy - slope * sxy


def fit_one(w, y, eps_lo, eps_hi):
    """(T0, delta, eps, sse) of one strategy's samples."""
    w = np.asarray(w, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    if len(w) < 3:
        return (np.nan,) * 4
    lo, hi = np.log(np.float64(eps_lo)), np.log(np.float64(eps_hi))
    for _ in range(LEVELS):
        les = [lo + (hi - lo) * (i / (GRID - 1)) for i in range(GRID)]
        sse = [line_fit(w, y, np.exp(le))[2] for le in les]
        best = int(np.argmin(sse))              # first minimum
        lo, hi = les[max(best - 1, 0)], les[min(best + 1, GRID - 1)]
    eps = np.exp(0.5 * (lo + hi))
    alpha, beta, sse = line_fit(w, y, eps)
    return alpha, beta / alpha, eps, sse


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
        t0, delta, eps, sse = fit_one(level[s], thr[s], eps_lo, eps_hi)
        params[t] = (t0, delta, eps, sse)
        if not np.isfinite(t0) or not t0 > 0:
            ok = False
            continue
        f = t0 * (1.0 - delta * np.log(eps + b))
        ok = ok and bool((f > 0).all())
        with np.errstate(divide="ignore"):
            tbt[t, 1:] = (1.0 / f).astype(np.float32)
    return params, tbt, ok
