#!/usr/bin/env python3
"""Benchmark of the batched Estimator on one MI355X.

One step = one pass of the whole hot path (trace scan, per-stage batch-queue scans, merges/joins,
latencies + miss counts, P99 selection, cost) over every candidate configuration of the workload,
with all inputs already resident in GPU memory.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload W5]
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak

# HBM bytes per launch of est_sim_kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes summarised in
# profiles/est_sim_kernel_W4.md, keyed by (workload, candidates per call).  Valid for the kernel those
# passes profiled; an entry is removed when the kernel changes and put back after re-profiling.
MEASURED_TRAFFIC_BYTES = {("W4", 65536): 1.5719e13}

# The kernel is bound by vector-instruction issue, not by HBM, so the line also says how full the
# VALU issue slots are: SQ_INSTS_VALU per launch from the same profile (same validity rule), against
# 256 CUs x 4 SIMDs x 2.4 GHz / 4 cycles per wave64 instruction on a 16-lane SIMD.
MEASURED_VALU_INSTS = {("W4", 65536): 5.2901e12}
VALU_PEAK_GINST_S = 256 * 4 * 2.4 / 4.0  # 614.4 G wavefront instructions / s


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=0)
    ap.add_argument("--workload", default="W4", choices=["W1", "W2", "W3", "W4", "W5"])
    ap.add_argument("--chunk", type=int, default=65536, help="candidates per library call (a progress line is printed after each)")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="configs timed on the CPU oracle (0 = skip)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="before the timed region, copy this many MiB device to device once (a kernel of known "
                         "traffic, to scale hardware counters read under rocprofv3)")
    ap.add_argument("--planner", action="store_true",
                    help="instead of the sweep, time the greedy planner (estimator_plan) on the workload's pipeline, trace and SLO")
    ap.add_argument("--handoff", action="store_true",
                    help="instead of the sweep, time estimator_tuner_handoff (traffic envelope + per-model ratios) on the workload's trace")
    ap.add_argument("--shared", action="store_true",
                    help="instead of the hot path with every candidate simulated on its own: the same candidates through "
                         "estimator_run_shared_dev, upstream stages shared with a base configuration (W4, W5)")
    ap.add_argument("--shared-bases-per-call", type=int, default=0, help="bases per library call (0 = 4096 on W4, 2048 on W5; the library takes them in rounds that fit the memory)")
    ap.add_argument("--shared-configs", type=int, default=0, help="only the first this many candidates (0 = all)")
    ap.add_argument("--planner-queries", type=int, default=50000, help="trace prefix the planner works on")
    ap.add_argument("--planner-max-replicas", type=int, default=32)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: candidate configurations are independent, so more GPUs would each take "
              "a slice of the configurations, but this build runs and reports a single MI355X (--gpus 1).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1812_01776_amd import estimator, workloads
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    w = workloads.WORKLOADS[args.workload]()
    est = estimator.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
    cfg = estimator.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    digest = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]  # which inputs this line was measured on
    input_sha256 = {"arrival_us": digest(w.arrival_us), "visit_mask": digest(w.visit_mask), "configs": digest(cfg),
                    "lat_us": digest(w.lat_us), "cost_uusd_hr": digest(w.cost_uusd_hr)}
    arr_t = torch.from_numpy(w.arrival_us.view(np.int32)).to(dev)
    msk_t = torch.from_numpy(w.visit_mask.view(np.int32)).to(dev)
    cfg_t = torch.from_numpy(cfg.view(np.uint8).reshape(-1)).to(dev)
    torch.cuda.synchronize()

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib * (1 << 20) // 4, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.handoff:
        # traffic envelope of the whole trace (one kernel) + per-model ratios (host arithmetic)
        est = estimator.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
        cfg = estimator.pack_configs(w.cfg_hw[:1], w.cfg_batch[:1], w.cfg_replicas[:1])[0]
        ts = int(sum(int(w.lat_us[s, w.cfg_hw[0, s], 0]) for s in range(w.n_stages)))  # a service time: every stage at batch 1
        est.tuner_handoff(w.arrival_us, w.visit_mask, cfg, ts)
        reps = 5
        t0 = time.perf_counter()
        for _ in range(reps):
            out = est.tuner_handoff(w.arrival_us, w.visit_mask, cfg, ts)
        dt = (time.perf_counter() - t0) / reps
        print(json.dumps({"metric": "tuner hand-off (traffic envelope + ratios) wall time, host buffers in, on 1 MI355X", "value": dt, "unit": "s",
                          "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": dt * 1e3, "higher_is_better": False, "scaling": "weak",
                          "vs_baseline": None, "dtype": "u32", "data": "synthetic",
                          "config": {"workload": args.workload + " trace", "n_queries": w.n_queries, "service_time_us": ts,
                                     "windows": len(out["window_us"]), "max_queries": out["max_queries"]}}))
        return

    if args.planner:
        # the step above the hot path: Algorithms 1 and 2 driving the batched Estimator
        n = min(args.planner_queries, w.n_queries)
        est = estimator.Estimator(w.parents, w.lat_us, w.cost_uusd_hr)
        t0 = time.perf_counter()
        plan = est.plan(w.arrival_us[:n], w.visit_mask[:n], w.slo_us, max_replicas=args.planner_max_replicas)
        t1 = time.perf_counter()
        line = {"metric": "greedy planner wall time on 1 MI355X", "value": t1 - t0, "unit": "s", "n_gpus": 1, "steps": 1, "warmup": 0,
                "ms_per_step": (t1 - t0) * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u32",
                "data": "synthetic",
                "config": {"workload": args.workload + " pipeline, first %d queries, SLO %d us" % (n, w.slo_us), "max_replicas": args.planner_max_replicas,
                           "feasible": plan is not None}}
        if plan is not None:
            line["config"].update({"accepted_steps": plan["n_steps"], "estimator_calls": plan["estimator_calls"],
                                   "candidates_simulated": plan["candidates"], "cost_uusd_hr": plan["cost_uusd_hr"], "p99_us": plan["p99_us"],
                                   "plan": [[int(x) for x in c] for c in plan["config"].tolist()],
                                   "simulations_per_s": plan["candidates"] * n / (t1 - t0)})
        print(json.dumps(line))
        return

    S = w.n_stages
    if args.shared:
        # The same candidates with shared upstream stages.  W5's candidates are 64-member neighbourhoods, the
        # first member being the base; a grid (W4) is cut along its most downstream swept stage: the base of a
        # candidate is the candidate with that stage at the grid's first value.
        words = cfg.view(np.uint32).reshape(w.n_configs, S)
        if args.workload == "W5":
            base_rows, base_of = words[::64].copy(), (np.arange(w.n_configs) // 64).astype(np.int64)
        else:
            varies = [s_ for s_ in range(S) if (words[:, s_] != words[0, s_]).any()]
            key = words.copy()
            if varies:
                key[:, max(varies)] = words[0, max(varies)]
            base_rows, base_of = np.unique(key, axis=0, return_inverse=True)
            base_of = base_of.reshape(-1)
        C = args.shared_configs if args.shared_configs > 0 else w.n_configs
        per_call = args.shared_bases_per_call or (2048 if args.workload == "W5" else 4096)
        order = np.argsort(base_of[:C], kind="stable")  # candidates grouped by base, results put back in place
        p99 = np.zeros(C, np.uint32); miss = np.zeros(C, np.uint32)
        sim_ms = cap_ms = 0.0; frac = []; calls = 0
        used = np.unique(base_of[:C])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for lo in range(0, len(used), per_call):
            bsel = used[lo:lo + per_call]
            remap = np.full(len(base_rows), -1, np.int64); remap[bsel] = np.arange(len(bsel))
            csel = order[np.isin(base_of[:C][order], bsel)]
            b_t = torch.from_numpy(np.ascontiguousarray(base_rows[bsel]).view(np.uint8).reshape(-1)).to(dev)
            c_t = torch.from_numpy(np.ascontiguousarray(words[csel]).view(np.uint8).reshape(-1)).to(dev)
            o_t = torch.from_numpy(remap[base_of[:C][csel]].astype(np.int32)).to(dev)
            r = est.run_shared_dev(arr_t, msk_t, b_t, len(bsel), c_t, o_t, len(csel), w.slo_us)
            st = est.stats()
            p99[csel] = r["p99_us"].cpu().numpy().view(np.uint32); miss[csel] = r["miss_count"].cpu().numpy().view(np.uint32)
            sim_ms += st["sim_ms"]; cap_ms += st["capture_ms"]; frac.append(st["ops_run_fraction"] * len(csel)); calls += 1
            print("[bench] shared: bases %d..%d of %d (%d candidates) done, kernels %.1f ms of which bases %.1f ms, scratch %.1f GB"
                  % (lo, lo + len(bsel), len(used), len(csel), st["sim_ms"], st["capture_ms"], st["workspace_bytes"] / 1e9), file=sys.stderr, flush=True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # a seeded sample against the oracle, which simulates each candidate on its own
        from oracle import oracle
        n_sample = args.cpu_sample if args.cpu_sample >= 0 else 8
        idx = np.sort(np.random.default_rng(7).choice(C, size=min(n_sample, C), replace=False))
        ok = None; cpu = None
        if len(idx):
            c0 = time.perf_counter()
            ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw[idx], w.cfg_batch[idx], w.cfg_replicas[idx], w.slo_us)
            c1 = time.perf_counter()
            ok = bool(np.array_equal(ref["p99_us"], p99[idx].astype(np.uint64)) and np.array_equal(ref["miss_count"], miss[idx].astype(np.uint64)))
            cpu = {"value": len(idx) * w.n_queries / (c1 - c0), "unit": "config*query simulations/s", "cores": 1, "kind": "oracle",
                   "sample": "%d seeded configurations of %s at the full %d queries, one thread, each simulated on its own" % (len(idx), args.workload, w.n_queries),
                   "matches_gpu": ok}
        print(json.dumps({"metric": "config*query simulations/s with shared upstream stages on 1 MI355X", "value": C * w.n_queries / (t1 - t0),
                          "unit": "config*query simulations/s", "n_gpus": 1, "steps": 1, "warmup": 0, "ms_per_step": (t1 - t0) * 1e3,
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
                          "config": {"workload": args.workload, "n_configs": C, "n_queries": w.n_queries, "bases": int(len(used)), "library_calls": calls,
                                     "kernel_ms": sim_ms, "kernel_ms_bases": cap_ms, "operations_run_fraction": float(sum(frac) / C),
                                     "feasible_configs": int((p99 <= w.slo_us).sum())},
                          "cpu_baseline": cpu}))
        return

    stats = {"sim_ms": 0.0, "launches": 0}

    def one_pass(tag, timed):
        """The whole hot path over every candidate, a chunk of candidates per library call."""
        parts = []
        for lo in range(0, w.n_configs, args.chunk):
            hi = min(lo + args.chunk, w.n_configs)
            parts.append(est.run_dev(arr_t, msk_t, cfg_t[lo * S * 4:hi * S * 4], hi - lo, w.slo_us))
            st = est.stats()  # HIP-event durations of this call's kernels, on the stream they ran on
            if timed:
                stats["sim_ms"] += st["sim_ms"]; stats["launches"] += st["n_launches"]
            stats["last"] = st
            print("[bench] %s: candidates %d..%d of %d done, simulation kernel %.1f ms" % (tag, lo, hi, w.n_configs, st["sim_ms"]),
                  file=sys.stderr, flush=True)
        return {k: torch.cat([p_[k] for p_ in parts]) for k in parts[0]}

    for i in range(args.warmup):
        one_pass("warmup %d" % i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        res = one_pass("step %d" % i, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    st = stats["last"]
    sim_ms, launches = stats["sim_ms"], stats["launches"]
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sims = w.n_configs * w.n_queries
    value = sims / (ms_per_step * 1e-3)

    # roofline of the dominant kernel (the simulation kernel): algorithmic bytes = 8 B per stage visit
    # (one ready time in, one completion time out), per candidate, per launch
    visits = st["stage_visits"]
    cfgs_per_launch = w.n_configs * args.steps / launches
    alg_bytes_per_launch = 8.0 * visits * cfgs_per_launch
    avg_launch_s = sim_ms * 1e-3 / launches
    achieved = alg_bytes_per_launch / avg_launch_s / 1e9

    valu = None
    insts = MEASURED_VALU_INSTS.get((args.workload, min(args.chunk, w.n_configs)))
    if insts is not None and launches == args.steps:  # one launch per step, as profiled
        g = insts / avg_launch_s / 1e9
        valu = {"insts_per_launch": insts, "achieved": g, "peak": VALU_PEAK_GINST_S, "unit": "G wave64 VALU instructions/s",
                "frac": g / VALU_PEAK_GINST_S}

    p99 = res["p99_us"].cpu().numpy().view(np.uint32)
    feasible = int((p99 <= w.slo_us).sum())

    # CPU baseline: the oracle as it stands, single thread, on a bounded sample of the same workload
    n_sample = args.cpu_sample if args.cpu_sample >= 0 else {"W1": 16, "W2": 1024, "W3": 160, "W4": 16, "W5": 8}[args.workload]
    cpu = None
    if n_sample > 0:
        from oracle import oracle
        rng = np.random.default_rng(7)
        idx = np.sort(rng.choice(w.n_configs, size=min(n_sample, w.n_configs), replace=False))
        c0 = time.perf_counter()
        ref = oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw[idx], w.cfg_batch[idx],
                         w.cfg_replicas[idx], w.slo_us)
        c1 = time.perf_counter()
        ok = (np.array_equal(ref["p99_us"], p99[idx].astype(np.uint64)) and
              np.array_equal(ref["miss_count"], res["miss_count"].cpu().numpy().view(np.uint32)[idx].astype(np.uint64)))
        cpu = {"value": len(idx) * w.n_queries / (c1 - c0), "unit": "config*query simulations/s", "cores": 1, "kind": "oracle",
               "sample": "%d seeded configurations of %s at the full %d queries, one thread" % (len(idx), args.workload, w.n_queries),
               "matches_gpu": bool(ok)}

    out = {
        "metric": "config x query simulations/sec on 1 MI355X",
        "value": value, "unit": "config*query simulations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": args.workload, "n_configs": w.n_configs, "n_queries": w.n_queries, "n_stages": w.n_stages,
                   "stage_visits_per_config": visits, "scratch_slots": st["n_slots"], "candidates_per_call": min(args.chunk, w.n_configs),
                   "feasible_configs": feasible, "input_sha256": input_sha256},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, min(args.chunk, w.n_configs))),
                     "kernel": "est_sim_kernel", "avg_launch_ms": avg_launch_s * 1e3, "valu_issue": valu},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
