"""Float64 closed forms of the synthetic profile and of single-triple latencies.

Written straight from the definitions (no tables, no float32), so that it can pin the oracle's
table indexing, operand order and signs from the outside.  Used only by CPU tests.
"""
import numpy as np


def profile64(tp, b):
    """Synthetic profile: prefill = a + p*L, seconds per output token = d*(1+0.03 b)."""
    a = 0.02 / tp**0.8
    p = 4e-5 / tp**0.85
    tbt = (0.012 / tp**0.7) * (1.0 + 0.03 * b)
    return a, p, tbt


def stage64(tp, B, occ, q_ticks, s_bar, kappa=0.0, worst=False):
    w = B if worst else min(B, occ + 1)
    a, p, tbt = profile64(tp, w)
    tbt *= 1.0 + kappa * max(4 * w - 3 * B, 0) / B
    wait = q_ticks / 2.0**20 + max(occ + 1 - B, 0) / B * s_bar * tbt
    return a, p, tbt, wait


def triple64(a, p, tbt, wait, L, S, Dt, Db):
    ttft = wait + a + p * L
    e2e = ttft + S * tbt
    De = Dt + S * Db
    s = ((Dt - ttft) / Dt, (Db - tbt) / Db, (De - e2e) / De)
    return dict(ttft=ttft, e2e=e2e, s=s, slack=min(s))
