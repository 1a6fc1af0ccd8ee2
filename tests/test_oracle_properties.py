"""Cross-checks and invariants for the CPU oracle on random tiny inputs."""
import numpy as np
import pytest

from oracle import oracle
from paper_1812_01776_amd import workloads
import refs


def _sim(w, c, **kw):
    return oracle.simulate(w.parents, w.lat_us, w.arrival_us, w.visit_mask, w.cfg_hw[c], w.cfg_batch[c],
                           w.cfg_replicas[c], **kw)


@pytest.mark.parametrize("seed", range(40))
def test_matches_tick_simulator(seed):
    """Brute force: a 1-us time-stepped simulator with polling, on tiny integer latencies."""
    rng = np.random.default_rng(seed)
    w = workloads.random_case(seed, S=int(rng.integers(1, 4)), n=int(rng.integers(1, 9)), C=2, max_b=3,
                              max_r=3, small_times=True)
    for c in range(w.n_configs):
        out = _sim(w, c, want_stages=True)
        lat, done = refs.tick_sim(w.parents, w.lat_us, w.arrival_us, w.visit_mask, w.cfg_hw[c],
                                  w.cfg_batch[c], w.cfg_replicas[c])
        assert out["latency"].astype(np.int64).tolist() == lat.tolist()
        assert out["done"].astype(np.int64).tolist() == done.tolist()


@pytest.mark.parametrize("seed", range(60))
def test_matches_per_stage_formulation(seed):
    """The event-queue simulation equals the per-stage sorted-scan formulation, per query and per
    stage, on random DAGs (half of the cases with many equal timestamps)."""
    w = workloads.random_case(1000 + seed, tie_heavy=(seed % 2 == 0))
    for c in range(w.n_configs):
        out = _sim(w, c, want_stages=True)
        lat, done = refs.stage_scan_sim(w.parents, w.lat_us, w.arrival_us, w.visit_mask, w.cfg_hw[c],
                                        w.cfg_batch[c], w.cfg_replicas[c])
        assert out["done"].astype(np.int64).tolist() == done.tolist()
        assert out["latency"].astype(np.int64).tolist() == lat.tolist()


@pytest.mark.parametrize("seed", range(30))
def test_structural_invariants(seed):
    w = workloads.random_case(2000 + seed, tie_heavy=(seed % 3 == 0))
    S, n = w.n_stages, w.n_queries
    for c in range(w.n_configs):
        out = _sim(w, c, want_stages=True, want_batches=True)
        ready, done, bl = out["ready"].astype(np.int64), out["done"].astype(np.int64), out["batches"].astype(np.int64)
        for s in range(S):
            visit = ((w.visit_mask >> s) & 1).astype(bool)
            B, R, h = int(w.cfg_batch[c, s]), int(w.cfg_replicas[c, s]), int(w.cfg_hw[c, s])
            bs = bl[bl[:, 0] == s]
            # every visiting query is in exactly one batch; sizes within [1, B]
            assert bs[:, 3].sum() == visit.sum()
            assert np.all((bs[:, 3] >= 1) & (bs[:, 3] <= B))
            # a batch lasts L(actual size)
            assert np.array_equal(bs[:, 2] - bs[:, 1], w.lat_us[s, h, bs[:, 3] - 1].astype(np.int64))
            # FIFO: batch start times never decrease in dispatch order
            assert np.all(np.diff(bs[:, 1]) >= 0)
            # at most R batches overlap
            ev = sorted([(int(b[1]), 1) for b in bs] + [(int(b[2]), -1) for b in bs], key=lambda e: (e[0], e[1]))
            run = 0
            for _, d in ev:
                run += d
                assert run <= R
            # skipped -> zero time; visited -> at least the fastest batch
            assert np.array_equal(done[s][~visit], ready[s][~visit])
            if visit.any():
                assert np.all(done[s][visit] >= ready[s][visit] + int(w.lat_us[s, h, :B].min()))
            # join by max / roots see the arrival
            if w.parents[s]:
                assert np.array_equal(ready[s], np.max(done[w.parents[s]], axis=0))
            else:
                assert np.array_equal(ready[s], w.arrival_us.astype(np.int64))
            # work conservation: a query waits only while all R replicas are busy
            for q in np.nonzero(visit)[0]:
                start = done[s][q] - int(w.lat_us[s, h, int(bs[(bs[:, 2] == done[s][q])][0, 3]) - 1])
                if start > ready[s][q]:
                    busy = np.sum((bs[:, 1] <= ready[s][q]) & (bs[:, 2] > ready[s][q]))
                    assert busy == R


@pytest.mark.parametrize("seed", range(10))
def test_shift_and_scale(seed):
    w = workloads.random_case(3000 + seed)
    for c in range(w.n_configs):
        base = _sim(w, c)["latency"]
        shifted = oracle.simulate(w.parents, w.lat_us, w.arrival_us + np.uint32(12345), w.visit_mask,
                                  w.cfg_hw[c], w.cfg_batch[c], w.cfg_replicas[c])["latency"]
        assert np.array_equal(base, shifted)
        scaled = oracle.simulate(w.parents, w.lat_us * np.uint32(7), w.arrival_us * np.uint32(7), w.visit_mask,
                                 w.cfg_hw[c], w.cfg_batch[c], w.cfg_replicas[c])["latency"]
        assert np.array_equal(base * np.uint64(7), scaled)


@pytest.mark.parametrize("seed", range(20))
def test_horizon_is_a_clamp(seed):
    """Saturating the clock at a small horizon equals clamping the unsaturated run's completion
    times at that horizon."""
    w = workloads.random_case(4000 + seed, max_r=2)
    for c in range(w.n_configs):
        free = _sim(w, c, want_stages=True)
        hz = int(w.arrival_us[-1]) + int(w.lat_us.max())  # lands in the middle of the busy period
        sat = _sim(w, c, want_stages=True, horizon=hz)
        assert np.array_equal(np.minimum(free["done"], np.uint64(hz)), sat["done"])


def test_p99_feasibility_relation():
    """miss_count <= N-k  <=>  p99 <= slo."""
    w = workloads.random_case(77, n=150, C=5)
    for slo in (50, 200, 400, 1000, 5000):
        r = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw, w.cfg_batch,
                       w.cfg_replicas, slo)
        k = -(-99 * 150 // 100)
        for c in range(5):
            assert (int(r["miss_count"][c]) <= 150 - k) == (int(r["p99_us"][c]) <= slo)
            cost = sum(int(w.cfg_replicas[c, s]) * int(w.cost_uusd_hr[s, w.cfg_hw[c, s]]) for s in range(w.n_stages))
            assert int(r["cost_uusd_hr"][c]) == cost
