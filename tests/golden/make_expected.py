"""Writes tests/golden/expected_w{3,4,5}.json: for seeded samples of the candidate configurations of
the three large workloads, what the CPU oracle computes at the full trace length -- P99, miss count,
cost, and a SHA-256 of the per-query latency array (uint32 little endian, query order).

Calls only the oracle (oracle/) and the seeded input generators; nothing here comes from the GPU path.
Run from the repository root:  python tests/golden/make_expected.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle  # noqa: E402
from paper_1812_01776_amd import workloads  # noqa: E402

SAMPLES = {"W3": 48, "W4": 12, "W5": 12}


def sample_indices(name, n_configs):
    rng = np.random.default_rng({"W3": 31, "W4": 41, "W5": 51}[name])
    k = SAMPLES[name]
    idx = set([0, n_configs - 1])
    idx.update(int(i) for i in rng.choice(n_configs, size=k - 2, replace=False))
    return sorted(idx)


def main():
    for name in ("W3", "W4", "W5"):
        w = workloads.WORKLOADS[name]()
        idx = sample_indices(name, w.n_configs)
        rows = []
        for c in idx:
            r = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw[c:c + 1],
                           w.cfg_batch[c:c + 1], w.cfg_replicas[c:c + 1], w.slo_us, want_latencies=True)
            lat = r["latency"][0]
            assert int(lat.max()) < 2**32
            rows.append({"config": c, "p99_us": int(r["p99_us"][0]), "miss_count": int(r["miss_count"][0]),
                         "cost_uusd_hr": int(r["cost_uusd_hr"][0]),
                         "latency_sha256": hashlib.sha256(lat.astype("<u4").tobytes()).hexdigest()})
            print(name, c, rows[-1]["p99_us"], rows[-1]["miss_count"], flush=True)
        out = {"_about": "CPU-oracle results at full trace length for sampled configurations of %s; written by "
                         "tests/golden/make_expected.py, which calls only oracle/ and the seeded generators." % name,
               "workload": name, "n_queries": w.n_queries, "n_configs": w.n_configs, "rows": rows}
        with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "expected_%s.json" % name.lower()), "w") as f:
            json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
