"""Plain reference of what the planner hands to the tuner (arXiv 1812.01776, Section 5,
"Initialization"): the traffic envelope of the sample trace and the per-model ratios.

TEST INFRASTRUCTURE ONLY: imported by tests/ and nothing else.

Envelope: window widths dT_i = T_s * 2^i while dT_i <= 60 s (at least dT_0); q_i = the largest number
of arrivals in any half-open window [t, t + dT_i).  Written as the definition: a window holding the
maximum can be slid right until it starts at an arrival, so only windows starting at arrivals are
counted, each by a plain scan.
"""
from fractions import Fraction

import numpy as np


def windows(service_time_us):
    w, out = int(service_time_us), []
    while not out or w <= 60_000_000:
        out.append(w)
        w *= 2
        if len(out) == 32:
            break
    return out


def envelope(arrival_us, service_time_us):
    a = [int(x) for x in np.asarray(arrival_us)]
    n = len(a)
    res = []
    for w in windows(service_time_us):
        best, end = 0, 0
        for j in range(n):
            if end < j:
                end = j
            while end < n and a[end] < a[j] + w:
                end += 1
            best = max(best, end - j)
        res.append(best)
    return res


def ratios(lat_us, arrival_us, visit_mask, cfg):
    """Per model (mu_m, rho_m) as exact fractions: mu_m = batch / latency(batch) in queries per second,
    rho_m = lambda * s_m / (replicas * mu_m) with lambda = n / (last - first arrival) and s_m the share
    of queries that visit the model; rho_m is None when the trace spans no time."""
    a = np.asarray(arrival_us)
    m = np.asarray(visit_mask)
    n = len(a)
    span = int(a[-1]) - int(a[0]) if n else 0
    out = []
    for s, (h, b, r) in enumerate(cfg):
        L = int(lat_us[s][h][b - 1])
        mu = Fraction(b * 1_000_000, L)
        visits = int(((m >> np.uint32(s)) & 1).sum()) if n else 0
        if span == 0:
            rho = None
        else:
            lam = Fraction(n * 1_000_000, span)
            rho = lam * Fraction(visits, n) / (r * mu)
        out.append((mu, rho))
    return out
