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
VALU_PEAK_GINST_S = 256 * 4 * 2.4 / 4.0  # 614.4 G wave64 vector instructions / s: 256 CUs x 4 SIMDs x 2.4 GHz / 4 cycles each
SALU_PEAK_GINST_S = 256 * 2.4            # 614.4 G scalar instructions / s: one scalar unit per CU, one instruction per cycle

# Hardware-counter figures per launch of est_sim_kernel, from the rocprofv3 passes summarised under profiles/
# (FETCH_SIZE + WRITE_SIZE scaled by a copy kernel of known size; SQ_INSTS_VALU; SQ_INSTS_SALU), keyed by
# (workload, candidates per call).  Each entry names the SHA-256 (first 16 hex digits) of the kernel sources it
# was taken on; the line below prints it only while the sources in the tree still hash to that, else null.
PROFILED = {
    ("W4", 65536): {"csrc_sha16": "3f0eef93ac58c684", "traffic_bytes": 1.65695e13, "valu_insts": 4.43262e12, "salu_insts": 4.74188e12,
                    "source": "profiles/est_sim_kernel_W4.md"},
    ("W5", 262144): {"csrc_sha16": "3f0eef93ac58c684", "traffic_bytes": 1.38932e14, "valu_insts": 3.55471e13, "salu_insts": 4.16431e13,
                    "source": "profiles/est_sim_kernel_W5.md"},
}


def csrc_sha16():
    d = os.path.join(ROOT, "paper_1812_01776_amd", "csrc")
    h = hashlib.sha256()
    for f in sorted(os.listdir(d)):
        if f.endswith((".h", ".hip")) or f == "est_host.cpp":  # what the kernels are compiled from, and the host code that lays out their operations and streams
            h.update(f.encode()); h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def oracle_legs(w, idx, threads):
    """The CPU oracle as it stands on a seeded sample: one thread, then the same kind of sample fanned out over
    `threads` host threads (one configuration at a time per thread; the oracle itself stays single-threaded and
    ctypes releases the interpreter lock during the call).  Returns (single, parallel, results of the first leg)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import oracle

    def one(c):
        return oracle.run(w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, w.cfg_hw[c:c + 1], w.cfg_batch[c:c + 1],
                          w.cfg_replicas[c:c + 1], w.slo_us)

    t0 = time.perf_counter()
    ref = [one(int(c)) for c in idx]
    t1 = time.perf_counter()
    single = len(idx) * w.n_queries / (t1 - t0)
    par = None
    if threads > 1:
        rng = np.random.default_rng(11)
        idx2 = rng.choice(w.n_configs, size=min(w.n_configs, max(threads, int(len(idx) * threads * 0.6))), replace=False)
        t2 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, [int(c) for c in idx2]))
        t3 = time.perf_counter()
        par = (len(idx2) * w.n_queries / (t3 - t2), len(idx2))
    return single, par, ref


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=0)
    ap.add_argument("--workload", default="W4", choices=["W1", "W2", "W3", "W4", "W5"])
    ap.add_argument("--chunk", type=int, default=0, help="candidates per library call, 0 = the whole sweep in one call (a progress line is printed after each call)")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="configs timed on the CPU oracle (0 = skip)")
    ap.add_argument("--copy-mib", type=int, default=1024,
                    help="size of the device-to-device copy that measures the copy bandwidth before the timed region (0 = skip); "
                         "under rocprofv3 the same copy kernel, of known traffic, scales the hardware counters")
    ap.add_argument("--regime-sample", type=int, default=512, help="candidates run once more with step counters for config.regime_mix (0 = skip)")
    ap.add_argument("--largest-sweep", default="auto", choices=["auto", "always", "never"],
                    help="with --workload W4: also time one pass of W5 after the timed steps (auto: when it fits --budget-s)")
    ap.add_argument("--provisioned", type=int, default=6144,
                    help="with --workload W4: also time one call of this many candidates provisioned around the SLO boundary (0 = skip)")
    ap.add_argument("--budget-s", type=int, default=540, help="wall time the default run allows itself before it leaves out the W5 pass")
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
              "a slice of the configurations, but the benchmark runs and reports a single MI355X (--gpus 1).", file=sys.stderr)
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
                                     "sharing": ("the library simulated every candidate on its own: the rounds the memory forces were estimated slower "
                                                 "(EST_SHARED_ALWAYS=1 forces them)") if sum(frac) >= C else "upstream stages shared",
                                     "feasible_configs": int((p99 <= w.slo_us).sum())},
                          "cpu_baseline": cpu}))
        return

    def chunk_of(wl):
        return min(args.chunk, wl.n_configs) if args.chunk > 0 else wl.n_configs

    def run_pass(wl, est_, arr, msk, cfgt, tag, acc=None):
        """The whole hot path over every candidate of wl, a chunk of candidates per library call."""
        parts = []
        S_ = wl.n_stages
        chunk = chunk_of(wl)
        for lo in range(0, wl.n_configs, chunk):
            hi = min(lo + chunk, wl.n_configs)
            parts.append(est_.run_dev(arr, msk, cfgt[lo * S_ * 4:hi * S_ * 4], hi - lo, wl.slo_us))
            st_ = est_.stats()  # HIP-event durations of this call's kernels, on the stream they ran on
            if acc is not None:
                acc["sim_ms"] += st_["sim_ms"]; acc["launches"] += st_["n_launches"]; acc["last"] = st_
            print("[bench] %s %s: candidates %d..%d of %d done, simulation kernel %.1f ms" % (wl.name, tag, lo, hi, wl.n_configs, st_["sim_ms"]),
                  file=sys.stderr, flush=True)
        return {k: torch.cat([p_[k] for p_ in parts]) for k in parts[0]}

    def roofline_of(wl, acc, passes):
        """Dominant kernel = the simulation kernel: algorithmic bytes = 8 B per stage visit (one ready time in, one
        completion time out) x candidates per launch, over the launch's HIP-event duration."""
        visits = acc["last"]["stage_visits"]
        launches = acc["launches"]
        per_launch = wl.n_configs * passes / launches
        avg_s = acc["sim_ms"] * 1e-3 / launches
        achieved = 8.0 * visits * per_launch / avg_s / 1e9
        r = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
             "kernel": "est_sim_kernel", "avg_launch_ms": avg_s * 1e3, "algorithmic_bytes_per_launch": 8.0 * visits * per_launch,
             "limited_by": "vector and scalar instruction issue, not memory bandwidth (profiles/)"}
        prof = PROFILED.get((wl.name, chunk_of(wl)))
        if prof is not None and per_launch == chunk_of(wl):  # (one launch per library call of that many candidates)
            if prof["csrc_sha16"] == csrc_sha16():
                r["traffic"] = prof["traffic_bytes"]
                for key, peak, unit in (("valu", VALU_PEAK_GINST_S, "G wave64 vector instructions/s"), ("salu", SALU_PEAK_GINST_S, "G scalar instructions/s")):
                    g = prof[key + "_insts"] / avg_s / 1e9
                    r[key + "_issue"] = {"insts_per_launch": prof[key + "_insts"], "achieved": g, "peak": peak,
                                         "unit": unit, "frac": g / peak, "source": prof["source"]}
            else:
                r["profile_note"] = "counters in %s were taken on other kernel sources (%s): not repeated here" % (prof["source"], prof["csrc_sha16"])
        return r

    # device copy bandwidth, measured: the second yardstick beside the published peak
    copy_gbs = None
    if args.copy_mib > 0:
        src = torch.ones(args.copy_mib * (1 << 20) // 4, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9  # bytes read + bytes written
        del src, dst

    t_all = time.perf_counter()
    for i in range(args.warmup):
        run_pass(w, est, arr_t, msk_t, cfg_t, "warmup %d" % i)
    stats = {"sim_ms": 0.0, "launches": 0}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        res = run_pass(w, est, arr_t, msk_t, cfg_t, "step %d" % i, stats)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    st = stats["last"]
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sims = w.n_configs * w.n_queries
    value = sims / (ms_per_step * 1e-3)
    roof = roofline_of(w, stats, args.steps)
    if copy_gbs is not None:
        roof["copy_bandwidth_measured"] = {"value": copy_gbs, "unit": "GB/s (read + write, %d MiB device to device)" % args.copy_mib,
                                           "frac": roof["achieved"] / copy_gbs}
    p99 = res["p99_us"].cpu().numpy().view(np.uint32)
    miss_gpu = res["miss_count"].cpu().numpy().view(np.uint32)
    feasible = int((p99 <= w.slo_us).sum())

    # which kind of step carried the stage visits (the kernel variant with step counters, on a spread of candidates),
    # and how many queries end clamped at the horizon (per-query latencies of a few candidates)
    regime = None
    if args.regime_sample > 0:
        import tempfile
        k = min(args.regime_sample, w.n_configs)
        sel = np.sort(np.random.default_rng(13).choice(w.n_configs, size=k, replace=False))  # (a stride would alias with a grid sweep)
        sub_t = torch.from_numpy(np.ascontiguousarray(cfg[sel]).view(np.uint8).reshape(-1)).to(dev)
        with tempfile.TemporaryDirectory() as td:
            os.environ["EST_DEBUG_TICKS"] = os.path.join(td, "ticks.bin")
            try:
                est.run_dev(arr_t, msk_t, sub_t, len(sel), w.slo_us)
            finally:
                del os.environ["EST_DEBUG_TICKS"]
            d = np.fromfile(os.path.join(td, "ticks.bin"), dtype=np.uint64)
        rec = d[len(sel):].reshape(len(sel), 32, 16).astype(np.float64)
        stg, oth = rec[:, :S, :], rec[:, 31, :]
        fast, gen = stg[:, :, 3].sum(), oth[:, 7].sum()
        tot = fast + gen
        named = stg[:, :, 4:8].sum(axis=(0, 1))
        lsel = sel[:: max(len(sel) // 8, 1)][:8]
        lcfg_t = torch.from_numpy(np.ascontiguousarray(cfg[lsel]).view(np.uint8).reshape(-1)).to(dev)
        lat = est.run_latencies_dev(arr_t, msk_t, lcfg_t, len(lsel)).cpu().numpy().view(np.uint32)
        clamped = float((lat.astype(np.uint64) + w.arrival_us.astype(np.uint64)[None, :] == 2**32 - 1).mean())
        ticks = stg[:, :, 1].sum() + oth[:, 0].sum() + oth[:, 1].sum() + oth[:, 2].sum()
        regime = {"sample": "%d seeded random candidates of the sweep (step counters), %d of them for the clamped share" % (len(sel), len(lsel)),
                  "stage_visits_by_step": {"light_load_large_groups": named[0] / tot, "light_load": named[1] / tot, "one_query_per_batch": named[2] / tot,
                                           "block_of_batches": named[3] / tot, "backlog_and_horizon": (fast - named.sum()) / tot, "general_one_batch": gen / tot},
                  "queries_per_step": tot / (stg[:, :, 2].sum() + stg[:, :, 0].sum()),
                  "wavefront_time_share": {"scans": stg[:, :, 1].sum() / ticks, "merges": oth[:, 0].sum() / ticks, "latency_sink": oth[:, 1].sum() / ticks,
                                           "p99_selection": oth[:, 2].sum() / ticks},
                  "queries_clamped_at_horizon": clamped}

    # CPU baseline: the oracle as it stands on a bounded seeded sample of the same workload, on this machine's host
    # cores: one thread, and fanned out over the host threads available (at most 16)
    n_sample = args.cpu_sample if args.cpu_sample >= 0 else {"W1": 16, "W2": 1024, "W3": 96, "W4": 8, "W5": 4}[args.workload]
    cpu = None
    if n_sample > 0:
        rng = np.random.default_rng(7)
        idx = np.sort(rng.choice(w.n_configs, size=min(n_sample, w.n_configs), replace=False))
        threads = max(1, min(16, len(os.sched_getaffinity(0)), os.cpu_count() or 1))
        single, par, ref = oracle_legs(w, idx, threads)
        ok = all(int(r["p99_us"][0]) == int(p99[c]) and int(r["miss_count"][0]) == int(miss_gpu[c]) for r, c in zip(ref, idx))
        cpu = {"value": par[0] if par else single, "unit": "config*query simulations/s", "cores": threads if par else 1, "kind": "oracle",
               "sample": ("%d seeded configurations of %s at the full %d queries on %d threads (one configuration per thread at a time)"
                          % (par[1], args.workload, w.n_queries, threads)) if par else
                         "%d seeded configurations of %s at the full %d queries, one thread" % (len(idx), args.workload, w.n_queries),
               "host_cores_visible": os.cpu_count(),
               "single_thread": {"value": single, "cores": 1, "sample": "%d seeded configurations at the full %d queries" % (len(idx), w.n_queries)},
               "matches_gpu": bool(ok)}

    # the largest sweep (W5): one pass of it after the timed steps when that fits the time this run may take;
    # a pass of W5 does about 8.9 x the work of a pass of W4 (8 x the simulations, a few more visits per query)
    largest = None
    # the regime a planner's search visits (W4's pipeline and trace, candidates provisioned around the SLO boundary):
    # one call, timed like the sweep, reported beside it
    provisioned = None
    if args.workload == "W4" and args.provisioned > 0:
        wp = workloads.w4_provisioned(n=w.n_queries, n_configs=args.provisioned, base=w)
        cp = torch.from_numpy(estimator.pack_configs(wp.cfg_hw, wp.cfg_batch, wp.cfg_replicas).view(np.uint8).reshape(-1)).to(dev)
        torch.cuda.synchronize()
        q0 = time.perf_counter()
        rp = est.run_dev(arr_t, msk_t, cp, wp.n_configs, wp.slo_us)
        torch.cuda.synchronize()
        q1 = time.perf_counter()
        sp = est.stats()
        pp = rp["p99_us"].cpu().numpy().view(np.uint32)
        provisioned = {"workload": "W4p", "n_configs": wp.n_configs, "n_queries": wp.n_queries, "ms": (q1 - q0) * 1e3, "kernel_ms": sp["sim_ms"],
                       "value": wp.n_configs * wp.n_queries / (q1 - q0), "unit": "config*query simulations/s",
                       "feasible_configs": int((pp <= wp.slo_us).sum()),
                       "roofline_frac": 8.0 * sp["stage_visits"] * wp.n_configs / (sp["sim_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if args.workload == "W5":
        largest = "this line"
    elif args.workload == "W4" and args.largest_sweep != "never":
        est_w5_s = 9.0 * ms_per_step * 1e-3
        spent = time.perf_counter() - t_all
        if args.largest_sweep == "always" or spent + est_w5_s + 60 <= args.budget_s:
            est.close()  # (its cached scratch and W5's do not fit side by side)
            w5 = workloads.w5()
            est5 = estimator.Estimator(w5.parents, w5.lat_us, w5.cost_uusd_hr)
            cfg5 = estimator.pack_configs(w5.cfg_hw, w5.cfg_batch, w5.cfg_replicas)
            a5 = torch.from_numpy(w5.arrival_us.view(np.int32)).to(dev); m5 = torch.from_numpy(w5.visit_mask.view(np.int32)).to(dev)
            c5 = torch.from_numpy(cfg5.view(np.uint8).reshape(-1)).to(dev)
            acc5 = {"sim_ms": 0.0, "launches": 0}
            # (untimed: one candidate per resident wavefront, so that the handle allocates its scratch, 233 GB, before the pass)
            est5.run_dev(a5, m5, c5[:6144 * w5.n_stages * 4], 6144, w5.slo_us)
            torch.cuda.synchronize()
            q0 = time.perf_counter()
            r5 = run_pass(w5, est5, a5, m5, c5, "pass", acc5)
            torch.cuda.synchronize()
            q1 = time.perf_counter()
            p5 = r5["p99_us"].cpu().numpy().view(np.uint32)
            largest = {"workload": "W5", "n_configs": w5.n_configs, "n_queries": w5.n_queries, "passes": 1, "ms_per_pass": (q1 - q0) * 1e3,
                       "value": w5.n_configs * w5.n_queries / (q1 - q0), "unit": "config*query simulations/s",
                       "stage_visits_per_config": acc5["last"]["stage_visits"], "feasible_configs": int((p5 <= w5.slo_us).sum()),
                       "roofline": roofline_of(w5, acc5, 1)}
            est5.close()
        else:
            largest = ("W5 not timed: %d warm-up + %d timed passes of W4 took %.0f s and one pass of W5 needs about %.0f s more, beyond the %d s "
                       "this run allows itself (--budget-s); `python bench.py --workload W5 --steps 1` times it alone"
                       % (args.warmup, args.steps, spent, est_w5_s, args.budget_s))

    out = {
        "metric": "config x query simulations/sec on 1 MI355X",
        "value": value, "unit": "config*query simulations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": args.workload, "n_configs": w.n_configs, "n_queries": w.n_queries, "n_stages": w.n_stages,
                   "stage_visits_per_config": st["stage_visits"], "scratch_slots": st["n_slots"], "candidates_per_call": chunk_of(w),
                   "feasible_configs": feasible, "kernel_sources_sha16": csrc_sha16(), "input_sha256": input_sha256, "largest_sweep": largest,
                   "provisioned_regime": provisioned, "regime_mix": regime},
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
