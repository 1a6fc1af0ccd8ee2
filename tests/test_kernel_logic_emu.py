"""Host-side checks of the kernel logic and of the host planner.

The device source (paper_1812_01776_amd/csrc/est_device.h) is compiled for the CPU against a lock-step
emulation of the 64-lane wavefront primitives (tests/emu) with its consistency checks switched on, and
driven through the same C ABI and host planner as the GPU library.  This finds indexing and protocol
mistakes before anything runs on a GPU, and exercises every host-reachable error code.  It is a check
of the code's logic, not a product path: the GPU parity tests are in test_gpu_parity.py.
"""
import ctypes
import json
import os

import numpy as np
import pytest

import emu_lib
from oracle import oracle
from paper_1812_01776_amd import estimator as binding
from paper_1812_01776_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_traces.json")


def _compare(w, est=None):
    est = est or emu_lib.make(w)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    lat = est.run_latencies(w.arrival_us, w.visit_mask, cfg)
    got = est.run(w.arrival_us, w.visit_mask, cfg, w.slo_us)
    ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw, w.cfg_batch,
                     w.cfg_replicas, w.slo_us, want_latencies=True)
    assert np.array_equal(lat.astype(np.uint64), ref["latency"])
    assert np.array_equal(got["p99_us"].astype(np.uint64), ref["p99_us"])
    assert np.array_equal(got["miss_count"].astype(np.uint64), ref["miss_count"])
    assert np.array_equal(got["cost_uusd_hr"], ref["cost_uusd_hr"])


def _hand_examples():
    with open(GOLDEN) as f:
        return json.load(f)["examples"]


@pytest.mark.parametrize("ex", _hand_examples(), ids=lambda e: e["name"])
def test_hand_traces(ex):
    S = len(ex["parents"])
    Bm = max(len(x) for x in ex["L"])
    lat = np.array([[list(x) + [x[-1]] * (Bm - len(x))] for x in ex["L"]], dtype=np.uint32)
    est = binding.Estimator(ex["parents"], lat, np.full((S, 1), 10**6, np.uint64), _lib=emu_lib.lib())
    cfg = binding.pack_configs([[0] * S], [ex["batch"]], [ex["replicas"]])
    assert est.run_latencies(ex["arrival"], ex["mask"], cfg)[0].tolist() == ex["latency"]
    r = est.run(ex["arrival"], ex["mask"], cfg, ex["slo"])
    assert (int(r["p99_us"][0]), int(r["miss_count"][0])) == (ex["p99"], ex["miss_count"])


@pytest.mark.parametrize("seed", range(24))
def test_random_dags_match_oracle(seed):
    _compare(workloads.random_case(seed, tie_heavy=(seed % 2 == 0)))


@pytest.mark.parametrize("seed", range(28))
def test_backlog_lockstep_and_horizon_cases_match_oracle(seed):
    # long queues: full batches in rotation, replicas in lock step (tied completions), maximum batch
    # size 1 with ties out of query order, queueing that runs into the horizon
    _compare(workloads.backlog_case(seed))


@pytest.mark.parametrize("seed", range(10))
def test_bursts_of_large_groups_match_oracle(seed, tmp_path, monkeypatch):
    # groups of queries that become ready together, large batches, many of them in flight at once; the
    # step counters confirm that the light-load step for large groups is the one that ran
    w = workloads.grouped_case(seed, n=1200)
    dump = tmp_path / "ticks.bin"
    monkeypatch.setenv("EST_DEBUG_TICKS", str(dump))
    _compare(w)
    d = np.fromfile(dump, dtype=np.uint64)[w.n_configs:].reshape(w.n_configs, 32, 16)
    assert d[:, :w.n_stages, 4].sum() > 0


@pytest.mark.parametrize("seed", range(12))
def test_provisioned_small_batches_with_tied_completions_match_oracle(seed):
    # 80-100 % utilisation, small batches on many replicas downstream of a batching stage: groups cut into
    # several batches that start together, so completions tie and leave merged by query index
    _compare(workloads.provisioned_case(seed, n=1500))


@pytest.mark.parametrize("seed,nw", [(s, 4) for s in range(12)] + [(s, 2) for s in range(0, 12, 2)])
def test_several_wavefronts_per_candidate_match_oracle(seed, nw, monkeypatch):
    # the candidate's operations dealt out to four (or two) wavefronts that run as a pipeline through the rings
    monkeypatch.setenv("EST_WAVES_PER_CANDIDATE", str(nw))
    w = [workloads.random_case, workloads.backlog_case, workloads.grouped_case, workloads.provisioned_case][seed % 4](seed)
    if w.n_queries > 1500:
        w = w.subset(n_queries=1500)
    est = emu_lib.make(w)
    _compare(w, est=est)
    assert est.stats()["waves_per_candidate"] == nw


@pytest.mark.parametrize("seed", range(12))
def test_small_in_ring_matches_oracle(seed, monkeypatch):
    # the scans' LDS in-ring at 128 keys (what the host picks when that lets a sixth wavefront share a SIMD):
    # refills of uneven length, with and without a filter
    monkeypatch.setenv("EST_SCAN_RING", "128")
    w = [workloads.random_case, workloads.backlog_case, workloads.grouped_case, workloads.provisioned_case][seed % 4](seed + 100)
    if w.n_queries > 900:
        w = w.subset(n_queries=900)
    _compare(w)


def test_wide_batches_many_replicas_and_ring_wrap():
    """R up to 16, B up to 64 and enough queries for the bounded rings to wrap several times; every
    time a multiple of 10 so that batches complete together and have to be merged by query index."""
    _compare(workloads.random_case(5, S=3, n=2500, C=2, max_b=64, max_r=16, tie_heavy=True, dag="linear"))


def test_clock_saturates_at_the_horizon():
    rng = np.random.default_rng(1)
    n = 1500
    arr = (np.uint64(3_500_000_000) + np.cumsum(rng.integers(0, 2000, size=n)).astype(np.uint64)).astype(np.uint32)
    lat = np.zeros((3, 1, 4), np.uint32)
    lat[:] = np.array([900_000, 1_000_000, 1_100_000, 1_200_000], np.uint32)
    lat[1] = lat[1] // 3
    mask = (rng.integers(0, 8, size=n) | 1).astype(np.uint32)
    w = workloads.Workload("sat", [[], [0], [0, 1]], lat, np.full((3, 1), 5, np.uint64), arr, mask,
                           np.zeros((2, 3), np.uint8), np.array([[1, 1, 1], [4, 2, 3]], np.uint8),
                           np.array([[1, 1, 1], [1, 3, 2]], np.uint16), 1000)
    ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw, w.cfg_batch,
                     w.cfg_replicas, w.slo_us, want_latencies=True)
    assert int((ref["latency"][0] + arr.astype(np.uint64) == 2**32 - 1).sum()) > 100  # the case does saturate
    _compare(w)


# ----------------------------------------------------------------------------- host planner / error codes

def _small():
    return workloads.random_case(3, S=3, n=40, C=3, dag="linear")


def test_empty_inputs_succeed():
    w = _small()
    est = emu_lib.make(w)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    r = est.run(np.zeros(0, np.uint32), np.zeros(0, np.uint32), cfg, 100)
    assert r["p99_us"].tolist() == [0, 0, 0] and r["miss_count"].tolist() == [0, 0, 0]
    want = [sum(int(w.cfg_replicas[c, s]) * int(w.cost_uusd_hr[s, w.cfg_hw[c, s]]) for s in range(3)) for c in range(3)]
    assert r["cost_uusd_hr"].tolist() == want
    r = est.run(w.arrival_us, w.visit_mask, cfg[:0], 100)
    assert r["p99_us"].shape == (0,)


def test_run_rejects_bad_inputs_and_leaves_outputs_alone():
    w = _small()
    est = emu_lib.make(w)
    lib = emu_lib.lib()
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)

    def expect(code, arrival=w.arrival_us, mask=w.visit_mask, cfg=cfg, slo=w.slo_us):
        with pytest.raises(binding.EstimatorError) as ei:
            est.run(arrival, mask, cfg, slo)
        assert ei.value.code == code
        assert lib.estimator_last_error(est._h) != b""

    bad = w.arrival_us.copy(); bad[10] = bad[9] - 1
    expect(binding.EST_EINVAL, arrival=bad)                                   # arrivals decrease
    for field, val in (("hw", 7), ("batch", 0), ("batch", 200), ("replicas", 0), ("replicas", 65)):
        c2 = cfg.copy(); c2[1, 2][field] = val
        expect(binding.EST_EINVAL, cfg=c2)
    late = (w.arrival_us.astype(np.uint64) + np.uint64(2**32 - 1 - int(w.arrival_us[-1]) - 5)).astype(np.uint32)
    expect(binding.EST_EINVAL, arrival=late)                                  # too close to the horizon
    # outputs untouched on error
    p99 = np.full(3, 77, np.uint32); miss = np.full(3, 78, np.uint32); cost = np.full(3, 79, np.uint64)
    c2 = cfg.copy(); c2[0, 0]["batch"] = 0
    tr = binding._Trace(w.n_queries, ctypes.c_void_p(w.arrival_us.ctypes.data), ctypes.c_void_p(w.visit_mask.ctypes.data))
    res = binding._Result(ctypes.c_void_p(p99.ctypes.data), ctypes.c_void_p(miss.ctypes.data), ctypes.c_void_p(cost.ctypes.data))
    rc = lib.estimator_run(est._h, ctypes.byref(tr), ctypes.c_void_p(c2.ctypes.data), ctypes.c_uint64(3), ctypes.c_uint32(10), ctypes.byref(res))
    assert rc == binding.EST_EINVAL and p99.tolist() == [77] * 3 and miss.tolist() == [78] * 3 and cost.tolist() == [79] * 3
    # NULL pointers
    assert lib.estimator_run(est._h, None, ctypes.c_void_p(cfg.ctypes.data), ctypes.c_uint64(3), ctypes.c_uint32(10), ctypes.byref(res)) == binding.EST_EINVAL
    assert lib.estimator_run(est._h, ctypes.byref(tr), None, ctypes.c_uint64(3), ctypes.c_uint32(10), ctypes.byref(res)) == binding.EST_EINVAL
    assert lib.estimator_run(est._h, ctypes.byref(tr), ctypes.c_void_p(cfg.ctypes.data), ctypes.c_uint64(3), ctypes.c_uint32(10), None) == binding.EST_EINVAL
    assert lib.estimator_run(None, ctypes.byref(tr), ctypes.c_void_p(cfg.ctypes.data), ctypes.c_uint64(3), ctypes.c_uint32(10), ctypes.byref(res)) == binding.EST_EINVAL
    # the device-side checks used by the device-pointer entry point (host memory plays the device here)
    rc = lib.estimator_run_dev(est._h, ctypes.byref(tr), ctypes.c_void_p(c2.ctypes.data), ctypes.c_uint64(3), ctypes.c_uint32(10),
                               ctypes.byref(res), None, ctypes.c_uint64(0), None)
    assert rc == binding.EST_EINVAL and p99.tolist() == [77] * 3
    trb = binding._Trace(w.n_queries, ctypes.c_void_p(bad.ctypes.data), ctypes.c_void_p(w.visit_mask.ctypes.data))
    rc = lib.estimator_run_dev(est._h, ctypes.byref(trb), ctypes.c_void_p(cfg.ctypes.data), ctypes.c_uint64(3), ctypes.c_uint32(10),
                               ctypes.byref(res), None, ctypes.c_uint64(0), None)
    assert rc == binding.EST_EINVAL and p99.tolist() == [77] * 3


def test_too_many_input_streams_is_unsupported():
    """A sink fed by more than EST_MAX_MERGE_SOURCES conditional stages."""
    S = 10
    parents = [[]] + [[0]] * 9
    rng = np.random.default_rng(0)
    lat = rng.integers(5, 50, size=(S, 1, 2)).astype(np.uint32)
    n = 400
    mask = (rng.integers(0, 2**S, size=n) | 1).astype(np.uint32)
    arr = np.cumsum(rng.integers(0, 30, size=n)).astype(np.uint32)
    est = binding.Estimator(parents, lat, np.ones((S, 1), np.uint64), _lib=emu_lib.lib())
    cfg = binding.pack_configs(np.zeros((1, S)), np.ones((1, S)), np.ones((1, S)))
    with pytest.raises(binding.EstimatorError) as ei:
        est.run(arr, mask, cfg, 100)
    assert ei.value.code == binding.EST_EUNSUPPORTED


def test_caller_workspace_limits_the_scratch_slots():
    """With a small caller-provided workspace fewer wavefronts (scratch slots) than candidates share the
    work; too small a workspace is EST_ENOMEM."""
    w = workloads.random_case(9, S=3, n=300, C=7, dag="linear")
    lib = emu_lib.lib()
    est = emu_lib.make(w)
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw, w.cfg_batch,
                     w.cfg_replicas, w.slo_us)
    tr = binding._Trace(w.n_queries, ctypes.c_void_p(w.arrival_us.ctypes.data), ctypes.c_void_p(w.visit_mask.ctypes.data))
    p99 = np.zeros(7, np.uint32); miss = np.zeros(7, np.uint32); cost = np.zeros(7, np.uint64)
    res = binding._Result(ctypes.c_void_p(p99.ctypes.data), ctypes.c_void_p(miss.ctypes.data), ctypes.c_void_p(cost.ctypes.data))
    raw = np.zeros(200_000 + 256, np.uint8)
    base = (raw.ctypes.data + 255) // 256 * 256
    rc = lib.estimator_run_dev(est._h, ctypes.byref(tr), ctypes.c_void_p(cfg.ctypes.data), ctypes.c_uint64(7), ctypes.c_uint32(w.slo_us),
                               ctypes.byref(res), ctypes.c_void_p(base), ctypes.c_uint64(90_000), None)
    assert rc == 0, lib.estimator_last_error(est._h)
    st = est.stats()
    assert st["n_slots"] < 7
    assert np.array_equal(p99.astype(np.uint64), ref["p99_us"]) and np.array_equal(miss.astype(np.uint64), ref["miss_count"])
    assert np.array_equal(cost, ref["cost_uusd_hr"])
    rc = lib.estimator_run_dev(est._h, ctypes.byref(tr), ctypes.c_void_p(cfg.ctypes.data), ctypes.c_uint64(7), ctypes.c_uint32(w.slo_us),
                               ctypes.byref(res), ctypes.c_void_p(base), ctypes.c_uint64(20_000), None)
    assert rc == binding.EST_ENOMEM
    assert est.workspace_bytes(300, 7) > 90_000


def test_diagnostics_variant_gives_the_same_results(tmp_path, monkeypatch):
    w = workloads.random_case(21, S=4, n=300, C=3, max_b=8, max_r=4)
    dump = tmp_path / "ticks.bin"
    monkeypatch.setenv("EST_DEBUG_TICKS", str(dump))
    _compare(w)
    d = np.fromfile(dump, dtype=np.uint64)
    assert d.size == w.n_configs * (1 + 16 * 32)
