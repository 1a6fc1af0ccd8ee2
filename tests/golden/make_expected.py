"""Writes tests/golden/expected_w{3,4,5,4p}.json: what the CPU oracle computes for the large workloads.

  W3            48 seeded configurations at the full trace length
  W4, W5        64 configurations each at the full trace length: the 16 with the least head-room at their
                bottleneck stage, the 16 with the most, 32 seeded random ones; and for ALL configurations
                of the sweep the P99 and miss count on the first 2,000 queries of the same trace (stored
                as SHA-256 of the uint32 little-endian arrays, plus a few sampled values)
  W4p           W4's pipeline with 16 candidates provisioned around the SLO boundary, full trace length

Per configuration at full length: P99, miss count, cost, and a SHA-256 of the per-query latency array
(uint32 little endian, query order).

Calls only the oracle (oracle/) and the seeded input generators; nothing here comes from the GPU path.
Run from the repository root:  python tests/golden/make_expected.py [W3 W4 W5 W4p]
"""
import hashlib
import json
import multiprocessing
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle  # noqa: E402
from paper_1812_01776_amd import workloads  # noqa: E402

PREFIX = 2000
MAKERS = {"W3": workloads.w3, "W4": workloads.w4, "W5": workloads.w5, "W4p": workloads.w4_provisioned}


def headroom(w):
    """Per configuration: the smallest ratio over stages of capacity R * B / L(B) to the share of the
    trace's queries that visit the stage (a common factor, the arrival rate, does not change the order)."""
    S = w.n_stages
    share = np.array([float(((w.visit_mask >> s) & 1).mean()) for s in range(S)])
    st = np.arange(S)[None, :]
    lat = w.lat_us[st, w.cfg_hw, w.cfg_batch.astype(np.int64) - 1].astype(np.float64)
    cap = w.cfg_replicas.astype(np.float64) * w.cfg_batch.astype(np.float64) / lat
    return (cap / np.maximum(share, 1e-9)[None, :]).min(axis=1)


def sample_indices(name, w):
    n_configs = w.n_configs
    if name == "W4p":
        return list(range(n_configs))
    if name == "W3":
        rng = np.random.default_rng(31)
        idx = set([0, n_configs - 1])
        idx.update(int(i) for i in rng.choice(n_configs, size=46, replace=False))
        return sorted(idx)
    rng = np.random.default_rng({"W4": 41, "W5": 51}[name])
    order = np.argsort(headroom(w), kind="stable")
    idx = set(int(i) for i in order[:16]) | set(int(i) for i in order[-16:])
    rest = np.array([i for i in range(n_configs) if i not in idx])
    idx.update(int(i) for i in rng.choice(rest, size=32, replace=False))
    return sorted(idx)


_W = None


def _init(name):
    global _W
    _W = MAKERS[name]()


def _full_row(c):
    w = _W
    r = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw[c:c + 1],
                   w.cfg_batch[c:c + 1], w.cfg_replicas[c:c + 1], w.slo_us, want_latencies=True)
    lat = r["latency"][0]
    assert int(lat.max()) < 2**32
    return {"config": int(c), "p99_us": int(r["p99_us"][0]), "miss_count": int(r["miss_count"][0]),
            "cost_uusd_hr": int(r["cost_uusd_hr"][0]),
            "latency_sha256": hashlib.sha256(lat.astype("<u4").tobytes()).hexdigest()}


def _prefix_chunk(span):
    w = _W
    lo, hi = span
    r = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us[:PREFIX], w.visit_mask[:PREFIX], w.cfg_hw[lo:hi],
                   w.cfg_batch[lo:hi], w.cfg_replicas[lo:hi], w.slo_us)
    return lo, r["p99_us"].astype(np.uint32), r["miss_count"].astype(np.uint32)


def main():
    names = sys.argv[1:] or ["W3", "W4", "W5", "W4p"]
    procs = min(8, os.cpu_count() or 1)
    for name in names:
        w = MAKERS[name]()
        idx = sample_indices(name, w)
        with multiprocessing.Pool(procs, initializer=_init, initargs=(name,)) as pool:
            rows = pool.map(_full_row, idx, chunksize=1)
            out = {"_about": "CPU-oracle results for %s; written by tests/golden/make_expected.py, which calls only "
                             "oracle/ and the seeded generators." % name,
                   "workload": name, "n_queries": w.n_queries, "n_configs": w.n_configs, "rows": rows}
            if name in ("W4", "W5"):
                step = 2048
                spans = [(lo, min(lo + step, w.n_configs)) for lo in range(0, w.n_configs, step)]
                p99 = np.zeros(w.n_configs, np.uint32)
                miss = np.zeros(w.n_configs, np.uint32)
                for lo, p, m in pool.imap_unordered(_prefix_chunk, spans):
                    p99[lo:lo + p.shape[0]] = p
                    miss[lo:lo + m.shape[0]] = m
                probe = list(range(0, w.n_configs, w.n_configs // 32))
                out["prefix"] = {"n_queries": PREFIX,
                                 "p99_sha256": hashlib.sha256(p99.astype("<u4").tobytes()).hexdigest(),
                                 "miss_sha256": hashlib.sha256(miss.astype("<u4").tobytes()).hexdigest(),
                                 "probe_configs": probe, "probe_p99_us": [int(p99[i]) for i in probe],
                                 "probe_miss_count": [int(miss[i]) for i in probe]}
        for r in rows:
            print(name, r["config"], r["p99_us"], r["miss_count"], flush=True)
        with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "expected_%s.json" % name.lower()), "w") as f:
            json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
