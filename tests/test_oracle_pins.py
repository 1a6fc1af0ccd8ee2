"""Pins for the CPU oracle: values fixed by hand traces, closed forms and textbook results.
Every check here is independent of the oracle's own code."""
import json
import os

import numpy as np
import pytest

from oracle import oracle
import refs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_traces.json")


def _examples():
    with open(GOLDEN) as f:
        return json.load(f)["examples"]


def _lat_table(L):
    """Ragged per-stage L lists -> [S][1][Bmax], padded by repeating the last entry."""
    Bmax = max(len(x) for x in L)
    return np.array([[list(x) + [x[-1]] * (Bmax - len(x))] for x in L], dtype=np.uint32)


@pytest.mark.parametrize("ex", _examples(), ids=lambda e: e["name"])
def test_hand_traces(ex):
    S = len(ex["parents"])
    lat = _lat_table(ex["L"])
    out = oracle.simulate(ex["parents"], lat, ex["arrival"], ex["mask"], [0] * S, ex["batch"],
                          ex["replicas"], want_stages=True)
    assert out["done"].tolist() == ex["done"]
    assert out["latency"].tolist() == ex["latency"]
    assert oracle.p99(out["latency"]) == ex["p99"]
    cost = np.full((S, 1), 1_000_000, dtype=np.uint64)
    r = oracle.run(ex["parents"], lat, cost, ex["arrival"], ex["mask"], [[0] * S], [ex["batch"]],
                   [ex["replicas"]], ex["slo"])
    assert int(r["p99_us"][0]) == ex["p99"]
    assert int(r["miss_count"][0]) == ex["miss_count"]
    assert int(r["cost_uusd_hr"][0]) == 1_000_000 * sum(ex["replicas"])


def test_lindley_recursion():
    """R=1, B=1, one stage is the single-server queue: done_i = max(done_{i-1}, t_i) + D."""
    rng = np.random.default_rng(11)
    for D in (1, 37, 5000):
        arr = np.cumsum(rng.integers(0, 2 * D + 2, size=5000)).astype(np.uint32)
        lat = np.full((1, 1, 1), D, dtype=np.uint32)
        out = oracle.simulate([[]], lat, arr, np.ones(5000, np.uint32), [0], [1], [1])
        ref = refs.lindley(arr, D) - arr.astype(np.int64)
        assert np.array_equal(out["latency"].astype(np.int64), ref)


def test_burst_closed_form():
    """All N queries at t=0, N a multiple of R*B: query i ends at (floor(i/(R*B))+1) * L(B)."""
    for (N, R, B, LB) in [(16, 2, 4, 9), (60, 3, 5, 17), (64, 1, 64, 100), (12, 4, 1, 3)]:
        lat = np.zeros((1, 1, B), dtype=np.uint32)
        lat[0, 0, :] = 1000 + np.arange(B)  # partial sizes never occur here
        lat[0, 0, B - 1] = LB
        out = oracle.simulate([[]], lat, np.zeros(N, np.uint32), np.ones(N, np.uint32), [0], [B], [R])
        want = (np.arange(N) // (R * B) + 1) * LB
        assert out["latency"].tolist() == want.tolist()


def test_no_contention_is_service_time():
    """With gaps longer than any stage latency every query sees an empty system: its latency is the
    sum of batch-1 latencies on its longest visited path (the planner's ServiceTime, Section 4.3)."""
    rng = np.random.default_rng(5)
    parents = [[], [0], [0], [1, 2], [3]]
    S = 5
    lat = rng.integers(10, 500, size=(S, 2, 4)).astype(np.uint32)
    n = 300
    arr = (np.arange(n) * 5000).astype(np.uint32)
    mask = np.zeros(n, np.uint32)
    for s in range(S):
        mask |= (rng.random(n) < 0.7).astype(np.uint32) << np.uint32(s)
    hw = rng.integers(0, 2, size=S)
    out = oracle.simulate(parents, lat, arr, mask, hw, [4] * S, [1] * S)
    for q in range(n):
        fin = [0] * S
        for s in range(S):
            r = max([fin[p] for p in parents[s]], default=0)
            fin[s] = r + (int(lat[s, hw[s], 0]) if (mask[q] >> s) & 1 else 0)
        assert int(out["latency"][q]) == fin[4]


@pytest.mark.parametrize("D,tol", [(500, 0.02), (800, 0.05)])
def test_md1_mean_wait(D, tol):
    """M/D/1 (Pollaczek-Khinchine with deterministic service): E[Wq] = rho*D / (2*(1-rho)).
    lambda = 1000 qps (so that 1e6 arrivals fit the 32-bit microsecond clock), N = 1e6 exponential
    gaps rounded to integer us, seed fixed.  Tolerance: 2% of E[Wq] at rho=0.5 (250 us -> 5 us,
    about 4 standard errors of the autocorrelated sample mean), 5% at rho=0.8 (1600 us -> 80 us)."""
    n = 1_000_000
    rng = np.random.default_rng(12345)
    gaps = np.rint(rng.exponential(1000.0, size=n)).astype(np.int64)
    arr = np.cumsum(gaps).astype(np.uint32)
    lat = np.full((1, 1, 1), D, dtype=np.uint32)
    out = oracle.simulate([[]], lat, arr, np.ones(n, np.uint32), [0], [1], [1])
    rho = D / 1000.0
    want = rho * D / (2 * (1 - rho))
    got = float(out["latency"].astype(np.float64).mean()) - D
    assert abs(got - want) <= tol * want, (got, want)


def test_p99_is_nearest_rank():
    rng = np.random.default_rng(3)
    for n in (1, 2, 99, 100, 101, 199, 200, 201, 1000, 12345):
        x = rng.integers(0, 10_000, size=n).astype(np.uint64)
        k = -(-99 * n // 100)
        assert oracle.p99(x) == int(np.sort(x)[k - 1])
    assert oracle.p99(np.zeros(0, np.uint64)) == 0
