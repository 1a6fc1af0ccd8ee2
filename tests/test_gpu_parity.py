"""GPU parity: the HIP library against the CPU oracle, bit-exact (all values are integers: per-query
latency, P99, miss count, cost).  Everything goes through the C ABI of include/estimator.h."""
import hashlib
import json
import os

import numpy as np
import pytest

from oracle import oracle
from paper_1812_01776_amd import estimator as binding
from paper_1812_01776_amd import workloads

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(params=["1", "4", "2"], ids=["wave_per_candidate", "workgroup_per_candidate", "two_wavefronts_per_candidate"])
def waves(request, monkeypatch):
    """The ways a candidate is run: by one wavefront, or (what calls with few candidates get by default) by a
    workgroup of four, or of two, wavefronts that share its operations as a pipeline."""
    monkeypatch.setenv("EST_WAVES_PER_CANDIDATE", request.param)
    return int(request.param)


def _compare(w, latencies=True, est=None):
    own = est is None
    est = est or binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    got = est.run(w.arrival_us, w.visit_mask, cfg, w.slo_us)
    ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw, w.cfg_batch,
                     w.cfg_replicas, w.slo_us, want_latencies=latencies)
    assert np.array_equal(got["p99_us"].astype(np.uint64), ref["p99_us"])
    assert np.array_equal(got["miss_count"].astype(np.uint64), ref["miss_count"])
    assert np.array_equal(got["cost_uusd_hr"], ref["cost_uusd_hr"])
    if latencies:
        lat = est.run_latencies(w.arrival_us, w.visit_mask, cfg)
        assert np.array_equal(lat.astype(np.uint64), ref["latency"])
    if own:
        est.close()


def test_wave_primitive_lane_layout():
    """The data-parallel-primitive moves the kernels rely on (lane +-1, lane ^ 1/2/4/8) and the bitonic
    network built from them, checked lane by lane on the device (in-bounds, one wavefront)."""
    import ctypes
    import torch  # noqa: F401  (PyTorch's copy of the HIP runtime first, so that this library binds to the same instance)
    lib = ctypes.CDLL(os.path.join(os.path.dirname(__file__), "selftest", "libwave_selftest.so"))  # test-only library
    out = np.zeros((21, 64), np.uint32)
    assert lib.est_selftest_wave(ctypes.c_void_p(out.ctypes.data)) == 0
    ln = np.arange(64)
    v = 7 * ln + 3
    assert out[0].tolist() == [3] + v[:-1].tolist()
    assert out[1].tolist() == v[1:].tolist() + [int(v[63])]
    for row, j in ((2, 1), (3, 2), (4, 4), (5, 8)):
        assert out[row].tolist() == v[ln ^ j].tolist(), j
    scr = (ln * 37 + 11) & 63
    for i, width in enumerate((2, 4, 8, 16, 32, 64)):
        assert out[6 + i][:width].tolist() == sorted(scr[:width].tolist()), width
    m = 0xF0F0A5A5C3C3FF01
    assert out[12].tolist() == [bin(m & ((1 << i) - 1)).count("1") for i in range(64)]
    # the scalar-unit helpers
    assert out[13][:63].tolist() == v[1:].tolist()
    want = v.copy(); want[17] = 1000; want[41] = 1001
    assert out[14].tolist() == want.tolist()
    assert out[15].tolist() == [1000 + 0x200] * 64
    assert out[16].tolist() == [0xFFFFFFFF] * 64
    assert out[17].tolist() == [0b001010101] * 64
    assert out[18].tolist() == (1000 + ln).tolist()
    sq = scr * scr + 1
    assert out[19].tolist() == (np.cumsum(sq) - sq).tolist()
    assert out[20].tolist() == [int(sq.sum())] * 64


def _hand_examples():
    with open(os.path.join(GOLD, "hand_traces.json")) as f:
        return json.load(f)["examples"]


@pytest.mark.parametrize("ex", _hand_examples(), ids=lambda e: e["name"])
def test_hand_traces(ex, waves):
    S = len(ex["parents"])
    Bm = max(len(x) for x in ex["L"])
    lat = np.array([[list(x) + [x[-1]] * (Bm - len(x))] for x in ex["L"]], dtype=np.uint32)
    est = binding.Estimator(ex["parents"], lat, np.full((S, 1), 10**6, np.uint64))
    cfg = binding.pack_configs([[0] * S], [ex["batch"]], [ex["replicas"]])
    assert est.run_latencies(ex["arrival"], ex["mask"], cfg)[0].tolist() == ex["latency"]
    r = est.run(ex["arrival"], ex["mask"], cfg, ex["slo"])
    assert (int(r["p99_us"][0]), int(r["miss_count"][0]), int(r["cost_uusd_hr"][0])) == \
        (ex["p99"], ex["miss_count"], 10**6 * sum(ex["replicas"]))
    est.close()


@pytest.mark.parametrize("seed", range(60))
def test_random_dags(seed, waves):
    _compare(workloads.random_case(seed, tie_heavy=(seed % 2 == 0)))


@pytest.mark.parametrize("seed", range(56))
def test_backlog_lockstep_and_horizon_cases(seed, waves):
    """Overloaded pipelines: full batches in rotation, replicas in lock step (tied completions), maximum
    batch size 1 with ties out of query order, queueing that runs into the horizon."""
    _compare(workloads.backlog_case(seed))


@pytest.mark.parametrize("seed", range(6))
def test_wide_batches_many_replicas_ties(seed, waves):
    """R up to 16, B up to 64, several thousand queries (bounded rings wrap, ragged tails), times on a
    10-us grid so that batches complete together."""
    _compare(workloads.random_case(100 + seed, S=4, n=6000 + 37 * seed, C=24, max_b=64, max_r=16, tie_heavy=True,
                                   dag="linear" if seed % 2 else "random"))


@pytest.mark.parametrize("seed", range(20))
def test_bursts_of_large_groups(seed, waves):
    """Queries that become ready in groups of 4..48, large batches whose service time is several times the
    gap between groups, many batches in flight at once (the light-load step for large groups), with ties
    on a 100-us grid, the fork-join shape, and stages that are short of replicas for part of the trace."""
    _compare(workloads.grouped_case(seed))


@pytest.mark.parametrize("seed", range(16))
def test_small_in_ring(seed, monkeypatch):
    """The scans' LDS in-ring at 128 keys instead of 256 (what the host picks when that lets a sixth wavefront
    share a SIMD, as on W4 and W5): refills of uneven length, with and without a filter."""
    monkeypatch.setenv("EST_SCAN_RING", "128")
    _compare([workloads.random_case, workloads.backlog_case, workloads.grouped_case, workloads.provisioned_case][seed % 4](seed + 100))


@pytest.mark.parametrize("seed", range(24))
def test_provisioned_small_batches_with_tied_completions(seed, waves):
    """Pipelines at 80-100 % utilisation with small batches on many replicas downstream of a batching stage
    (the regime around the SLO boundary): groups are cut into several batches that start at the same
    instant, completions tie and leave merged by query index."""
    _compare(workloads.provisioned_case(seed))


def test_replica_and_batch_limits(waves):
    """R = 64 and B = 64, the largest the interface allows."""
    w = workloads.random_case(7, S=2, n=5000, C=4, max_b=64, max_r=4, dag="linear")
    w.cfg_replicas[:] = np.array([[64, 1], [64, 64], [1, 64], [33, 17]], np.uint16)
    w.cfg_batch[:] = np.array([[64, 64], [1, 64], [64, 1], [63, 2]], np.uint8)
    _compare(w)


def test_degenerate_inputs(waves):
    w = workloads.random_case(3, S=3, n=40, C=3, dag="linear")
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    r = est.run(np.zeros(0, np.uint32), np.zeros(0, np.uint32), cfg, 100)
    assert r["p99_us"].tolist() == [0, 0, 0] and r["miss_count"].tolist() == [0, 0, 0]
    assert est.run(w.arrival_us, w.visit_mask, cfg[:0], 100)["p99_us"].shape == (0,)
    # one query; all queries at the same instant; nobody visits any stage; a stage nobody visits
    for arr, mask in ((np.array([5], np.uint32), np.array([7], np.uint32)),
                      (np.full(300, 9, np.uint32), np.full(300, 7, np.uint32)),
                      (np.arange(50, dtype=np.uint32), np.zeros(50, np.uint32)),
                      (np.arange(200, dtype=np.uint32) * 3, np.full(200, 5, np.uint32))):
        w2 = workloads.Workload("deg", w.parents, w.lat_us, w.cost_uusd_hr, arr, mask, w.cfg_hw, w.cfg_batch, w.cfg_replicas, 100)
        _compare(w2, est=est)
    with pytest.raises(binding.EstimatorError) as ei:
        bad = w.arrival_us.copy(); bad[3] = bad[2] - 1
        est.run(bad, w.visit_mask, cfg, 100)
    assert ei.value.code == binding.EST_EINVAL
    est.close()


def test_clock_saturates_at_the_horizon(waves):
    rng = np.random.default_rng(1)
    n = 4000
    arr = (np.uint64(3_000_000_000) + np.cumsum(rng.integers(0, 2000, size=n)).astype(np.uint64)).astype(np.uint32)
    lat = np.zeros((3, 1, 4), np.uint32)
    lat[:] = np.array([900_000, 1_000_000, 1_100_000, 1_200_000], np.uint32)
    lat[1] = lat[1] // 3
    mask = (rng.integers(0, 8, size=n) | 1).astype(np.uint32)
    w = workloads.Workload("sat", [[], [0], [0, 1]], lat, np.full((3, 1), 5, np.uint64), arr, mask,
                           np.zeros((3, 3), np.uint8), np.array([[1, 1, 1], [2, 4, 1], [4, 2, 3]], np.uint8),
                           np.array([[1, 1, 1], [2, 1, 2], [1, 3, 2]], np.uint16), 1000)
    _compare(w)


def test_w1_full():
    _compare(workloads.w1())


@pytest.mark.production_rings
def test_w2_full():
    _compare(workloads.w2())


def test_device_pointer_entry_points_and_tiling():
    """estimator_run_dev / estimator_run_latencies_dev with torch-owned memory, the torch stream, and a
    caller workspace small enough that the candidates share a few scratch slots."""
    import torch
    w = workloads.w2().subset(cfg_index=np.arange(0, 1024, 4))
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    dev = torch.device("cuda:0")
    arr_t = torch.from_numpy(w.arrival_us.view(np.int32)).to(dev)
    msk_t = torch.from_numpy(w.visit_mask.view(np.int32)).to(dev)
    cfg_t = torch.from_numpy(cfg.view(np.uint8).reshape(-1)).to(dev)
    ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw, w.cfg_batch,
                     w.cfg_replicas, w.slo_us, want_latencies=True)
    ws = torch.empty(6_000_000, dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        got = est.run_dev(arr_t, msk_t, cfg_t, w.n_configs, w.slo_us, workspace_t=ws)
        lat = est.run_latencies_dev(arr_t, msk_t, cfg_t, w.n_configs, workspace_t=ws)
    assert est.stats()["n_slots"] < w.n_configs
    assert np.array_equal(got["p99_us"].cpu().numpy().view(np.uint32).astype(np.uint64), ref["p99_us"])
    assert np.array_equal(got["miss_count"].cpu().numpy().view(np.uint32).astype(np.uint64), ref["miss_count"])
    assert np.array_equal(got["cost_uusd_hr"].cpu().numpy().view(np.uint64), ref["cost_uusd_hr"])
    assert np.array_equal(lat.cpu().numpy().view(np.uint32).astype(np.uint64), ref["latency"])
    est.close()


# ----------------------------------------------------------------------------- the large workloads

def _expected(name):
    with open(os.path.join(GOLD, "expected_%s.json" % name.lower())) as f:
        return json.load(f)


def _check_rows(w, exp, p99, miss, cost, est, lat_rows):
    """p99/miss/cost: full arrays over all configurations of the sweep; per-query latencies are
    recomputed for lat_rows of the sampled configurations and compared by SHA-256."""
    for row in exp["rows"]:
        c = row["config"]
        assert int(p99[c]) == row["p99_us"], (c, int(p99[c]), row["p99_us"])
        assert int(miss[c]) == row["miss_count"], c
        assert int(cost[c]) == row["cost_uusd_hr"], c
    rows = exp["rows"][:lat_rows]
    idx = [r["config"] for r in rows]
    cfg = binding.pack_configs(w.cfg_hw[idx], w.cfg_batch[idx], w.cfg_replicas[idx])
    lat = est.run_latencies(w.arrival_us, w.visit_mask, cfg)
    for i, row in enumerate(rows):
        assert hashlib.sha256(lat[i].astype("<u4").tobytes()).hexdigest() == row["latency_sha256"], row["config"]


@pytest.mark.production_rings
def test_w3_full_sweep_sampled_against_oracle():
    """All 8,192 configurations x 100,000 queries in one call (the launch shape the benchmark uses);
    48 sampled configurations are compared with stored oracle results (P99, misses, cost, and every
    per-query latency through its SHA-256), and all configurations with the live oracle on the first
    2,000 queries."""
    w = workloads.w3()
    exp = _expected("W3")
    assert exp["n_queries"] == w.n_queries and exp["n_configs"] == w.n_configs
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    got = est.run(w.arrival_us, w.visit_mask, cfg, w.slo_us)
    _check_rows(w, exp, got["p99_us"], got["miss_count"], got["cost_uusd_hr"], est, lat_rows=48)
    # cost of every configuration has a closed form
    want_cost = (w.cfg_replicas.astype(np.uint64) * w.cost_uusd_hr[np.arange(5)[None, :], w.cfg_hw]).sum(axis=1)
    assert np.array_equal(got["cost_uusd_hr"], want_cost)
    est.close()
    _compare(w.subset(cfg_index=np.arange(0, 8192, 8), n_queries=2000), latencies=False)


def _dev_inputs(w):
    import torch
    dev = torch.device("cuda:0")
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    return (torch.from_numpy(w.arrival_us.view(np.int32)).to(dev), torch.from_numpy(w.visit_mask.view(np.int32)).to(dev),
            torch.from_numpy(cfg.view(np.uint8).reshape(-1)).to(dev))


def _run_sweep_dev(est, w, arr_t, msk_t, cfg_t, per_call):
    """The whole sweep through estimator_run_dev, per_call candidates at a time (the benchmark's call shape)."""
    S = w.n_stages
    p99, miss, cost = [], [], []
    for lo in range(0, w.n_configs, per_call):
        hi = min(lo + per_call, w.n_configs)
        print("%s candidates %d..%d" % (w.name, lo, hi), flush=True)
        r = est.run_dev(arr_t, msk_t, cfg_t[lo * S * 4:hi * S * 4], hi - lo, w.slo_us)
        p99.append(r["p99_us"].cpu().numpy().view(np.uint32)); miss.append(r["miss_count"].cpu().numpy().view(np.uint32))
        cost.append(r["cost_uusd_hr"].cpu().numpy().view(np.uint64))
    return np.concatenate(p99), np.concatenate(miss), np.concatenate(cost)


@pytest.mark.production_rings
def test_w4_full_sweep_sampled_against_oracle():
    """All 65,536 configurations x 1,000,000 queries, called the way the benchmark calls the library
    (device pointers, 32,768 candidates per call); the 64 sampled configurations (the 16 with the least
    head-room at their bottleneck, the 16 with the most, 32 random) are compared with the stored oracle
    results: P99, misses, cost, and every per-query latency through its SHA-256."""
    w = workloads.w4()
    exp = _expected("W4")
    assert exp["n_queries"] == w.n_queries and exp["n_configs"] == w.n_configs and len(exp["rows"]) == 64
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    arr_t, msk_t, cfg_t = _dev_inputs(w)
    p99, miss, cost = _run_sweep_dev(est, w, arr_t, msk_t, cfg_t, 32768)
    _check_rows(w, exp, p99, miss, cost, est, lat_rows=64)
    S = w.n_stages
    want_cost = (w.cfg_replicas.astype(np.uint64) * w.cost_uusd_hr[np.arange(S)[None, :], w.cfg_hw]).sum(axis=1)
    assert np.array_equal(cost, want_cost)
    est.close()


@pytest.mark.production_rings
def test_w3_workgroup_per_candidate_long_trace(monkeypatch):
    """64 candidates of W3 at the full 100,000 queries, each run by a workgroup of four wavefronts (fork, three
    branches, join): every per-query latency, P99, misses and cost against the live oracle."""
    monkeypatch.setenv("EST_WAVES_PER_CANDIDATE", "4")
    w = workloads.w3().subset(cfg_index=np.arange(3, 8192, 128))
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    _compare(w, est=est)
    assert est.stats()["waves_per_candidate"] == 4
    est.close()


@pytest.mark.production_rings
def test_w4_pipeline_provisioned_candidates_full_trace():
    """W4's pipeline and full trace with 16 candidates provisioned around the SLO boundary (from slightly
    overloaded to comfortably feasible: the regime a planner's search works in): P99, misses, cost and
    every per-query latency (SHA-256) against stored oracle results."""
    w = workloads.w4_provisioned()
    exp = _expected("W4p")
    assert exp["n_queries"] == w.n_queries and exp["n_configs"] == w.n_configs == len(exp["rows"])
    assert sum(1 for r in exp["rows"] if r["p99_us"] <= w.slo_us) >= 8  # feasible ones are really among them
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    got = est.run(w.arrival_us, w.visit_mask, cfg, w.slo_us)
    assert est.stats()["waves_per_candidate"] == 4  # (a call this small gives every candidate a workgroup)
    _check_rows(w, exp, got["p99_us"], got["miss_count"], got["cost_uusd_hr"], est, lat_rows=16)
    est.close()


@pytest.mark.production_rings
def test_w5_sampled_configs_full_trace():
    """64 sampled configurations of the largest sweep (least head-room, most, random) at its full trace
    length (2,000,000 queries): P99, misses, cost and every per-query latency (SHA-256) against stored
    oracle results."""
    w = workloads.w5()
    exp = _expected("W5")
    assert exp["n_queries"] == w.n_queries and exp["n_configs"] == w.n_configs and len(exp["rows"]) == 64
    idx = [r["config"] for r in exp["rows"]]
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = binding.pack_configs(w.cfg_hw[idx], w.cfg_batch[idx], w.cfg_replicas[idx])
    got = est.run(w.arrival_us, w.visit_mask, cfg, w.slo_us)
    lat = est.run_latencies(w.arrival_us, w.visit_mask, cfg)
    for i, row in enumerate(exp["rows"]):
        assert int(got["p99_us"][i]) == row["p99_us"], row["config"]
        assert int(got["miss_count"][i]) == row["miss_count"], row["config"]
        assert int(got["cost_uusd_hr"][i]) == row["cost_uusd_hr"], row["config"]
        assert hashlib.sha256(lat[i].astype("<u4").tobytes()).hexdigest() == row["latency_sha256"], row["config"]
    est.close()


@pytest.mark.parametrize("name", ["W4", "W5"])
def test_w4_w5_all_configs_trace_prefix(name):
    """EVERY configuration of each 10-stage sweep on the first 2,000 queries of its trace: P99 and miss
    count of all 65,536 / 262,144 candidates against the stored oracle results (SHA-256 of the arrays,
    and 32 spot values that name a culprit when the hashes differ), cost against its closed form."""
    w = workloads.WORKLOADS[name]()
    exp = _expected(name)["prefix"]
    w = w.subset(n_queries=exp["n_queries"])
    est = binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    arr_t, msk_t, cfg_t = _dev_inputs(w)
    p99, miss, cost = _run_sweep_dev(est, w, arr_t, msk_t, cfg_t, 65536)
    est.close()
    for c, p, m in zip(exp["probe_configs"], exp["probe_p99_us"], exp["probe_miss_count"]):
        assert (int(p99[c]), int(miss[c])) == (p, m), c
    assert hashlib.sha256(p99.astype("<u4").tobytes()).hexdigest() == exp["p99_sha256"]
    assert hashlib.sha256(miss.astype("<u4").tobytes()).hexdigest() == exp["miss_sha256"]
    S = w.n_stages
    want_cost = (w.cfg_replicas.astype(np.uint64) * w.cost_uusd_hr[np.arange(S)[None, :], w.cfg_hw]).sum(axis=1)
    assert np.array_equal(cost, want_cost)


def test_diagnostics_variant_gives_the_same_results(tmp_path, monkeypatch):
    """EST_DEBUG_TICKS=<file> launches the kernel variant compiled with step counters and dumps them:
    per candidate the wavefront's run time, then per candidate and stage sixteen counters."""
    w = workloads.random_case(21, S=4, n=1500, C=6, max_b=8, max_r=4)
    dump = tmp_path / "ticks.bin"
    monkeypatch.setenv("EST_DEBUG_TICKS", str(dump))
    _compare(w)
    d = np.fromfile(dump, dtype=np.uint64)
    assert d.size == w.n_configs * (1 + 16 * 32)
    assert (d[:w.n_configs] > 0).all()
