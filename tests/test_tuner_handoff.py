"""Traffic envelope and per-model ratios handed from the planner to the tuner (Section 5).

oracle/envelope_oracle.py is the definition written out; it is pinned by a brute force over every
integer window start on tiny traces and by the closed form for evenly spaced arrivals.  The library
(estimator_tuner_handoff: one kernel over the trace plus exact integer ratios) must agree with it
exactly."""
from fractions import Fraction

import numpy as np
import pytest

import emu_lib
from oracle import envelope_oracle
from paper_1812_01776_amd import estimator as binding
from paper_1812_01776_amd import workloads


def test_window_widths_double_up_to_sixty_seconds():
    assert envelope_oracle.windows(1_000_000) == [1_000_000 * 2**i for i in range(6)]  # 32 s is the last <= 60 s
    assert envelope_oracle.windows(70_000_000) == [70_000_000]
    assert envelope_oracle.windows(3)[-1] <= 60_000_000 < 2 * envelope_oracle.windows(3)[-1]


def test_envelope_against_every_window_position():
    rng = np.random.default_rng(5)
    for _ in range(20):
        n = int(rng.integers(1, 40))
        a = np.sort(rng.integers(0, 60, size=n)).astype(np.uint32)
        ts = int(rng.integers(1, 9))
        got = envelope_oracle.envelope(a, ts)
        for w, q in zip(envelope_oracle.windows(ts), got):
            if w > 200:
                assert q == n  # wider than the whole trace
                continue
            brute = max(int(((a >= t) & (a < t + w)).sum()) for t in range(0, 61))
            assert q == brute


def test_envelope_of_evenly_spaced_arrivals():
    g, n = 250, 5000
    a = (np.arange(n) * g).astype(np.uint32)
    for w, q in zip(envelope_oracle.windows(1000), envelope_oracle.envelope(a, 1000)):
        assert q == min(n, -(-w // g))  # ceil(w / g) arrivals fit a half-open window of width w


def test_ratios_hand_computed():
    """mu_m and rho_m on numbers worked out by hand.  1,001 arrivals 1,000 us apart span exactly one
    second, so lambda = 1,001 queries/s.  Model 0: every query, batch 4 in 8,000 us (mu = 4 / 8 ms =
    500 queries/s) on 3 replicas: rho = 1001 / (3 * 500).  Model 1: every second query (501 of 1,001),
    batch 1 in 2,500 us (mu = 400/s) on 2 replicas: rho = 1001 * (501 / 1001) / (2 * 400) = 501 / 800.
    And the identity that gives the ratio its meaning (Section 5): at r = lambda the tuner's rule
    k_m = ceil(r s_m / (mu_m rho_m)) gives back the planned replicas."""
    n = 1001
    arr = (np.arange(n) * 1000).astype(np.uint32)
    mask = np.where(np.arange(n) % 2 == 0, 3, 1).astype(np.uint32)
    lat = np.zeros((2, 1, 4), np.uint32)
    lat[0, 0] = [5000, 6000, 7000, 8000]
    lat[1, 0] = [2500, 2600, 2700, 2800]
    cfg = [(0, 4, 3), (0, 1, 2)]
    (mu0, rho0), (mu1, rho1) = envelope_oracle.ratios(lat, arr, mask, cfg)
    assert (mu0, rho0) == (Fraction(500), Fraction(1001, 1500))
    assert (mu1, rho1) == (Fraction(400), Fraction(501, 800))
    lam = Fraction(1001)
    for (mu, rho), share, (_, _, replicas) in zip(((mu0, rho0), (mu1, rho1)), (Fraction(1), Fraction(501, 1001)), cfg):
        k = lam * share / (mu * rho)
        assert k == replicas and -(-k.numerator // k.denominator) == replicas
    # the same identity on a random pipeline, for every model
    w = workloads.random_case(47, S=4, n=500, C=1)
    triples = [(int(w.cfg_hw[0, s]), int(w.cfg_batch[0, s]), int(w.cfg_replicas[0, s])) for s in range(w.n_stages)]
    lam = Fraction(500 * 1_000_000, int(w.arrival_us[-1]) - int(w.arrival_us[0]))
    for s, ((mu, rho), (_, _, replicas)) in enumerate(zip(envelope_oracle.ratios(w.lat_us, w.arrival_us, w.visit_mask, triples), triples)):
        share = Fraction(int(((w.visit_mask >> s) & 1).sum()), 500)
        if share:
            k = lam * share / (mu * rho)
            assert -(-k.numerator // k.denominator) == replicas
    assert envelope_oracle.ratios(lat, arr[:1], mask[:1], cfg)[0][1] is None  # no time span, no rate


def _same_as_oracle(est, w, ts):
    cfg = binding.pack_configs(w.cfg_hw[:1], w.cfg_batch[:1], w.cfg_replicas[:1])[0]
    got = est.tuner_handoff(w.arrival_us, w.visit_mask, cfg, ts)
    assert got["window_us"] == envelope_oracle.windows(ts)
    assert got["max_queries"] == envelope_oracle.envelope(w.arrival_us, ts)
    triples = [(int(w.cfg_hw[0, s]), int(w.cfg_batch[0, s]), int(w.cfg_replicas[0, s])) for s in range(w.n_stages)]
    for (mu, rho), (mn, md), (rn, rd) in zip(envelope_oracle.ratios(w.lat_us, w.arrival_us, w.visit_mask, triples), got["mu"], got["rho"]):
        assert Fraction(mn, md) == mu
        assert (rho is None and rd == 0) or Fraction(rn, rd) == rho


@pytest.mark.parametrize("seed", range(4))
def test_library_handoff_matches_emulated(seed):
    w = workloads.random_case(40 + seed, S=3, n=400, C=2, tie_heavy=(seed % 2 == 0))
    _same_as_oracle(emu_lib.make(w), w, 7 + 13 * seed)


def test_handoff_rejects_bad_arguments():
    w = workloads.random_case(44, S=2, n=50, C=1)
    est = emu_lib.make(w)
    cfg = binding.pack_configs(w.cfg_hw[:1], w.cfg_batch[:1], w.cfg_replicas[:1])[0]
    with pytest.raises(binding.EstimatorError) as ei:
        est.tuner_handoff(w.arrival_us, w.visit_mask, cfg, 0)
    assert ei.value.code == binding.EST_EINVAL
    one = est.tuner_handoff(w.arrival_us[:1], w.visit_mask[:1], cfg, 5)  # a single query: no time span
    assert one["max_queries"][0] == 1 and all((rn, rd) == (0, 0) for rn, rd in one["rho"])


@pytest.mark.gpu
@pytest.mark.parametrize("name,n,ts", [("W3", 20000, 1500), ("W5", 30000, 40000), ("W2", 10000, 1)])
def test_library_handoff_matches(name, n, ts):
    w = workloads.WORKLOADS[name]()
    w = w.subset(cfg_index=[0], n_queries=min(n, w.n_queries))
    _same_as_oracle(binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr), w, ts)
