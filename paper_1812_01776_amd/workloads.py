"""Seeded synthetic inputs for the batched Estimator.

This module only *draws inputs* (traces, profiles, DAGs, candidate configurations); it holds
none of the Estimator's arithmetic and is the one module shared by the CPU oracle's tests and
the GPU library's tests and benchmark.

The shapes follow the paper's workload description (arXiv 1812.01776, Section 6 "Workload
Setup"): inter-arrival times are Gamma distributed with mean 1/lambda and a given CV, a
time-varying workload moves between Gamma distributions over time, batching raises both
throughput and latency of a model profile (Section 2.1, model-profile figure), and some
pipeline branches are taken conditionally (Section 2).  The paper defines
CV = sigma^2 / mu^2 (Section 2.1), so the Gamma shape is k = 1/CV and the scale is CV/lambda.
The five workloads W1..W5 are the five benchmark configurations of this repository; each
function's docstring states its recipe.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class Workload:
    name: str
    parents: list            # per stage, list of parent stage indices (parents precede children)
    lat_us: np.ndarray       # uint32 [S][H][Bmax], entry b-1 = latency of a batch of b
    cost_uusd_hr: np.ndarray  # uint64 [S][H], micro-dollars per replica-hour
    arrival_us: np.ndarray   # uint32 [N], non-decreasing
    visit_mask: np.ndarray   # uint32 [N], bit s = query visits stage s
    cfg_hw: np.ndarray       # uint8  [C][S]
    cfg_batch: np.ndarray    # uint8  [C][S]
    cfg_replicas: np.ndarray  # uint16 [C][S]
    slo_us: int

    @property
    def n_stages(self):
        return len(self.parents)

    @property
    def n_queries(self):
        return int(self.arrival_us.shape[0])

    @property
    def n_configs(self):
        return int(self.cfg_hw.shape[0])

    def stage_visits(self):
        """Total number of (query, stage) visits: sum over stages of N_s."""
        S = self.n_stages
        return int(sum(int(((self.visit_mask >> s) & 1).sum()) for s in range(S)))

    def subset(self, cfg_index=None, n_queries=None):
        idx = slice(None) if cfg_index is None else np.asarray(cfg_index)
        nq = self.n_queries if n_queries is None else int(n_queries)
        return Workload(self.name, self.parents, self.lat_us, self.cost_uusd_hr,
                        self.arrival_us[:nq].copy(), self.visit_mask[:nq].copy(),
                        np.ascontiguousarray(self.cfg_hw[idx]), np.ascontiguousarray(self.cfg_batch[idx]),
                        np.ascontiguousarray(self.cfg_replicas[idx]), self.slo_us)


# ----------------------------------------------------------------------------- traces

def gamma_trace(n, rate_qps, cv, seed):
    """n arrivals; gaps ~ Gamma(shape 1/cv, scale cv/rate) seconds, rounded to integer us."""
    rng = np.random.default_rng(seed)
    gaps_s = rng.gamma(1.0 / cv, cv / rate_qps, size=n)
    gaps_us = np.rint(gaps_s * 1e6).astype(np.int64)
    arr = np.cumsum(gaps_us)
    assert arr[-1] < 2**32 - 1
    return arr.astype(np.uint32)


def ramp_trace(n, rate_lo, rate_hi, ramp_windows, cv, seed):
    """Time-varying trace: the rate is constant inside each 1 s window, rising linearly from
    rate_lo to rate_hi over the first `ramp_windows` windows and staying at rate_hi after.
    Each gap is drawn from the Gamma of the window that holds the previous arrival."""
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.int64)
    filled = 0
    t = 0  # integer us
    w = 0
    while filled < n:
        rate = rate_lo + (rate_hi - rate_lo) * w / ramp_windows if w < ramp_windows else rate_hi
        wend = (w + 1) * 1_000_000
        if t >= wend:
            w += 1
            continue
        m = int(rate * 1.5) + 64
        gaps = np.rint(rng.gamma(1.0 / cv, cv / rate, size=m) * 1e6).astype(np.int64)
        times = t + np.cumsum(gaps)
        # gap i was drawn while standing at times[i-1] (or t): keep it if that instant is in this window
        prev = np.concatenate(([t], times[:-1]))
        keep = int(np.searchsorted(prev, wend, side="left"))  # prev < wend
        keep = min(keep, n - filled)
        out[filled:filled + keep] = times[:keep]
        filled += keep
        t = int(times[keep - 1]) if keep > 0 else t
        if keep < m:
            w += 1
    assert out[-1] < 2**32 - 1
    return out.astype(np.uint32)


# ----------------------------------------------------------------------------- profiles

def linear_profiles(S, H, Bmax, seed, quadratic=False):
    """L(b) = a + c*b (+ d*b^2) us with a~U{2000..20000}, c~U{100..3000}, d~U{0..20}, and a
    per-replica price ~U[0.1, 3.0] $/hr stored as integer micro-dollars."""
    rng = np.random.default_rng(seed)
    a = rng.integers(2000, 20001, size=(S, H))
    c = rng.integers(100, 3001, size=(S, H))
    d = rng.integers(0, 21, size=(S, H)) if quadratic else np.zeros((S, H), dtype=np.int64)
    b = np.arange(1, Bmax + 1, dtype=np.int64)
    lat = a[:, :, None] + c[:, :, None] * b[None, None, :] + d[:, :, None] * b[None, None, :] ** 2
    cost = np.rint(rng.uniform(0.1, 3.0, size=(S, H)) * 1e6).astype(np.uint64)
    return lat.astype(np.uint32), cost


def branch_masks(n, S, always, branches, seed):
    """visit masks: stages in `always` are visited by every query; each entry of `branches` is a
    (stages, probability) pair drawn once per query (Bernoulli), all its stages sharing the draw."""
    rng = np.random.default_rng(seed)
    mask = np.zeros(n, dtype=np.uint32)
    for s in always:
        mask |= np.uint32(1 << s)
    for stages, p in branches:
        take = rng.random(n) < p
        bits = np.uint32(sum(1 << s for s in stages))
        mask[take] |= bits
    return mask


# ----------------------------------------------------------------------------- the five workloads

def w1():
    """Linear 2-stage pipeline, 1,000 Poisson arrivals at 100 qps, 16 configs."""
    S, H, Bmax = 2, 1, 8
    lat, cost = linear_profiles(S, H, Bmax, seed=1001)
    arr = gamma_trace(1000, 100.0, 1.0, seed=0)
    mask = np.full(1000, 3, dtype=np.uint32)
    hw, bt, rp = [], [], []
    for b in (1, 2, 4, 8):
        for r in (1, 2, 3, 4):
            hw.append([0, 0]); bt.append([b, 4]); rp.append([r, 2])
    return Workload("W1", [[], [0]], lat, cost, arr, mask, np.array(hw, np.uint8),
                    np.array(bt, np.uint8), np.array(rp, np.uint16), 150_000)


def w2():
    """Linear 3-stage pipeline, 10,000 arrivals (CV=1, 500 qps), 1,024 random configs."""
    S, H, Bmax = 3, 3, 32
    lat, cost = linear_profiles(S, H, Bmax, seed=1002)
    arr = gamma_trace(10_000, 500.0, 1.0, seed=1)
    mask = np.full(10_000, 7, dtype=np.uint32)
    rng = np.random.default_rng(2002)
    C = 1024
    hw = rng.integers(0, H, size=(C, S)).astype(np.uint8)
    bt = (1 << rng.integers(0, 6, size=(C, S))).astype(np.uint8)
    rp = rng.integers(1, 9, size=(C, S)).astype(np.uint16)
    return Workload("W2", [[], [0], [1]], lat, cost, arr, mask, hw, bt, rp, 200_000)


def w3():
    """5-stage fan-out DAG: 0 -> {1,2,3} -> 4 (join by max), 100,000 bursty arrivals (CV=4,
    1,000 qps); each branch taken per query with its own seeded probability in [0.3,1.0]."""
    S, H, Bmax = 5, 3, 64
    n = 100_000
    lat, cost = linear_profiles(S, H, Bmax, seed=1003)
    arr = gamma_trace(n, 1000.0, 4.0, seed=2)
    prng = np.random.default_rng(1003 + 500)
    probs = prng.uniform(0.3, 1.0, size=3)
    mask = branch_masks(n, S, always=[0, 4], branches=[([1], probs[0]), ([2], probs[1]), ([3], probs[2])],
                        seed=1003 + 700)
    rng = np.random.default_rng(2003)
    C = 8192
    hw = rng.integers(0, H, size=(C, S)).astype(np.uint8)
    bt = rng.integers(1, 65, size=(C, S)).astype(np.uint8)
    rp = rng.integers(1, 17, size=(C, S)).astype(np.uint16)
    return Workload("W3", [[], [0], [0], [0], [1, 2, 3]], lat, cost, arr, mask, hw, bt, rp, 300_000)


W45_PARENTS = [[], [0], [1], [2], [3], [2], [5], [4, 6], [7], [8]]
"""10 stages: 0 -> 1 -> 2, then branch A = 3 -> 4 and branch B = 5 -> 6 in parallel, joined at 7,
then 7 -> 8 -> 9."""


def _w45_masks(n, seed):
    prng = np.random.default_rng(seed)
    pa, pb = prng.uniform(0.3, 1.0, size=2)
    mask = branch_masks(n, 10, always=[0, 1, 2, 7, 8, 9], branches=[([3, 4], pa), ([5, 6], pb)],
                        seed=seed + 200)
    return mask, (pa, pb)


def _visit_prob(s, pa, pb):
    return pa if s in (3, 4) else pb if s in (5, 6) else 1.0


def _fixed_stage(lat, s, demand_qps, rng):
    """A seeded (hw, B, R) for a stage that is not swept, with capacity R * B / L(B) >= 1.5 x the
    stage's demand: the (hardware type, batch size) pairs are tried in a seeded random order and the
    first that reaches the capacity with at most 16 replicas is taken; if none does, the pair with the
    largest capacity at 16 replicas."""
    H = lat.shape[1]
    pairs = [(h, b) for h in range(H) for b in (8, 16, 32, 64)]
    best = None
    for i in rng.permutation(len(pairs)):
        hw, b = pairs[int(i)]
        per_replica = b / (float(lat[s, hw, b - 1]) * 1e-6)
        r = int(np.ceil(1.5 * demand_qps / per_replica))
        if r <= 16:
            return hw, b, max(r, 1)
        if best is None or per_replica > best[0]:
            best = (per_replica, hw, b)
    return best[1], best[2], 16


def w4(n=1_000_000):
    """10-stage DAG, 1,000,000 arrivals (CV=2, 5,000 qps), quadratic profiles, 65,536 configs =
    a 16-point (B, R) grid on each of the 4 most expensive stages, the other stages fixed."""
    S, H, Bmax = 10, 3, 64
    lat, cost = linear_profiles(S, H, Bmax, seed=1004, quadratic=True)
    arr = gamma_trace(n, 5000.0, 2.0, seed=3)
    mask, (pa, pb) = _w45_masks(n, seed=1004 + 500)
    rng = np.random.default_rng(2004)
    swept = sorted(np.argsort(-cost.min(axis=1).astype(np.int64), kind="stable")[:4].tolist())
    base_hw = np.zeros(S, np.uint8); base_b = np.zeros(S, np.uint8); base_r = np.zeros(S, np.uint16)
    for s in range(S):
        if s in swept:
            base_hw[s] = int(np.argmin(lat[s, :, 0]))  # the hardware with the lowest batch-1 latency
        else:
            base_hw[s], base_b[s], base_r[s] = _fixed_stage(lat, s, 5000.0 * _visit_prob(s, pa, pb), rng)
    grid = [(b, r) for b in (1, 4, 16, 64) for r in (2, 4, 8, 16)]
    C = 16 ** 4
    hw = np.tile(base_hw, (C, 1)); bt = np.tile(base_b, (C, 1)); rp = np.tile(base_r, (C, 1))
    idx = np.arange(C)
    for k, s in enumerate(swept):
        g = (idx // (16 ** k)) % 16
        bt[:, s] = np.array([grid[i][0] for i in range(16)], np.uint8)[g]
        rp[:, s] = np.array([grid[i][1] for i in range(16)], np.uint16)[g]
    return Workload("W4", W45_PARENTS, lat, cost, arr, mask, hw, bt, rp, 250_000)


def w4_provisioned(n=1_000_000, n_configs=16, seed=2404, base=None):
    """W4's pipeline, profiles, trace and masks with candidates that are provisioned for the load
    (the regime a planner's search spends its time in, around the SLO boundary): per stage a seeded
    batch size in {1, 2, 4, 8}, the hardware type with the lowest latency at that batch size, and
    replicas = ceil(f x demand / (B / L(B))) with a seeded head-room f in [0.9, 1.3], up to the 64
    replicas the interface allows.  The head-room grows with the candidate index, so the set runs
    from slightly overloaded through barely stable to comfortably feasible.  (base: W4 as already generated, to
    save generating it again.)"""
    w = base if base is not None else w4(n=n)
    S = w.n_stages
    prng = np.random.default_rng(1004 + 500)
    pa, pb = prng.uniform(0.3, 1.0, size=2)  # the branch probabilities w4() drew
    rng = np.random.default_rng(seed)
    hw = np.zeros((n_configs, S), np.uint8); bt = np.zeros((n_configs, S), np.uint8); rp = np.zeros((n_configs, S), np.uint16)
    for c in range(n_configs):
        lo = 0.9 + 0.3 * c / max(n_configs - 1, 1)
        for s in range(S):
            b = int(rng.choice([1, 2, 4, 8]))
            h = int(np.argmin(w.lat_us[s, :, b - 1]))
            f = float(rng.uniform(lo, lo + 0.1))
            per_replica = b / (float(w.lat_us[s, h, b - 1]) * 1e-6)
            r = int(np.ceil(f * 5000.0 * _visit_prob(s, pa, pb) / per_replica))
            hw[c, s] = h; bt[c, s] = b; rp[c, s] = min(max(r, 1), 64)
    return Workload("W4p", w.parents, w.lat_us, w.cost_uusd_hr, w.arrival_us, w.visit_mask, hw, bt, rp, w.slo_us)


def w5(n=2_000_000, n_base=4096):
    """Same DAG under a time-varying trace (1,000 -> 8,000 qps over 160 one-second windows, then
    flat; CV=4 inside each window); configs are the 64-member neighbourhoods of seeded bases:
    the base, 50 single-stage moves (replicas +1/-1, batch x2, the two other hardware types)
    and 13 seeded two-stage moves."""
    S, H, Bmax = 10, 3, 64
    lat, cost = linear_profiles(S, H, Bmax, seed=1005, quadratic=True)
    arr = ramp_trace(n, 1000.0, 8000.0, 160, 4.0, seed=4)
    mask, (pa, pb) = _w45_masks(n, seed=1005 + 500)
    rng = np.random.default_rng(2005)
    hw_l, bt_l, rp_l = [], [], []

    def move(cfg, s, kind):
        h, b, r = cfg
        h = h.copy(); b = b.copy(); r = r.copy()
        if kind == 0:
            r[s] = min(r[s] + 1, 16)
        elif kind == 1:
            r[s] = max(r[s] - 1, 1)
        elif kind == 2:
            b[s] = min(b[s] * 2, 64)
        elif kind == 3:
            h[s] = (h[s] + 1) % 3
        else:
            h[s] = (h[s] + 2) % 3
        return h, b, r

    for _ in range(n_base):
        h = rng.integers(0, H, size=S).astype(np.int64)
        b = (1 << rng.integers(0, 7, size=S)).astype(np.int64)
        r = rng.integers(1, 17, size=S).astype(np.int64)
        base = (h, b, r)
        members = [base]
        for s in range(S):
            for kind in range(5):
                members.append(move(base, s, kind))
        for _ in range(13):
            s1, s2 = rng.choice(S, size=2, replace=False)
            k1, k2 = rng.integers(0, 5, size=2)
            members.append(move(move(base, int(s1), int(k1)), int(s2), int(k2)))
        for (mh, mb, mr) in members:
            hw_l.append(mh); bt_l.append(mb); rp_l.append(mr)
    return Workload("W5", W45_PARENTS, lat, cost, arr, mask, np.array(hw_l, np.uint8),
                    np.array(bt_l, np.uint8), np.array(rp_l, np.uint16), 200_000)


WORKLOADS = {"W1": w1, "W2": w2, "W3": w3, "W4": w4, "W5": w5}


def random_case(seed, S=None, n=None, C=None, max_b=8, max_r=4, H=2, small_times=False, dag="random",
                tie_heavy=False):
    """A small random DAG / trace / config set for property and parity tests."""
    rng = np.random.default_rng(seed)
    S = int(rng.integers(1, 7)) if S is None else S
    n = int(rng.integers(1, 200)) if n is None else n
    C = int(rng.integers(1, 6)) if C is None else C
    parents = []
    for s in range(S):
        if s == 0 or dag == "roots":
            parents.append([])
        elif dag == "linear":
            parents.append([s - 1])
        else:
            k = int(rng.integers(0, min(s, 3) + 1))
            parents.append(sorted(rng.choice(s, size=k, replace=False).tolist()) if k else [])
    Bmax = max_b
    if small_times:
        lat = rng.integers(1, 9, size=(S, H, Bmax)).astype(np.uint32)
        gaps = rng.integers(0, 4, size=n)
    else:
        a = rng.integers(20, 200, size=(S, H)); c = rng.integers(1, 40, size=(S, H))
        lat = (a[:, :, None] + c[:, :, None] * np.arange(1, Bmax + 1)[None, None, :]).astype(np.uint32)
        if tie_heavy:
            lat = (lat // 10 * 10).astype(np.uint32)
            gaps = rng.integers(0, 3, size=n) * 10
        else:
            gaps = rng.integers(0, 120, size=n)
    arr = np.cumsum(gaps).astype(np.uint32)
    mask = np.zeros(n, dtype=np.uint32)
    for s in range(S):
        p = 1.0 if rng.random() < 0.5 else rng.uniform(0.2, 1.0)
        mask |= (rng.random(n) < p).astype(np.uint32) << np.uint32(s)
    cost = rng.integers(100_000, 3_000_000, size=(S, H)).astype(np.uint64)
    hw = rng.integers(0, H, size=(C, S)).astype(np.uint8)
    bt = rng.integers(1, Bmax + 1, size=(C, S)).astype(np.uint8)
    rp = rng.integers(1, max_r + 1, size=(C, S)).astype(np.uint16)
    slo = int(lat.max()) * 2
    return Workload("rand%d" % seed, parents, lat, cost, arr, mask, hw, bt, rp, slo)


def neighbourhood_case(seed, n=None, n_bases=None, per_base=None, **kw):
    """random_case whose candidates are neighbours of a few base configurations (the call pattern of
    the planner's search, Section 4.3): each candidate copies its base and re-draws 0, 1 or 2 stages.
    Returns the workload plus (base hw, batch, replicas arrays [n_bases][S], base_of [C])."""
    rng = np.random.default_rng(10_000 + seed)
    nb = int(rng.integers(1, 4)) if n_bases is None else n_bases
    pb = int(rng.integers(2, 9)) if per_base is None else per_base
    w = random_case(seed, n=n, C=nb, **kw)
    S, H, Bmax = w.lat_us.shape
    max_r = kw.get("max_r", 4)
    b_hw, b_bt, b_rp = w.cfg_hw.copy(), w.cfg_batch.copy(), w.cfg_replicas.copy()
    hw, bt, rp, base_of = [], [], [], []
    for b in range(nb):
        for _ in range(pb):
            h, t, r = b_hw[b].copy(), b_bt[b].copy(), b_rp[b].copy()
            for s in rng.choice(S, size=min(S, int(rng.integers(0, 3))), replace=False):
                h[s] = rng.integers(0, H); t[s] = rng.integers(1, Bmax + 1); r[s] = rng.integers(1, max_r + 1)
            hw.append(h); bt.append(t); rp.append(r); base_of.append(b)
    order = rng.permutation(len(base_of))  # candidates of one base need not be adjacent
    w.cfg_hw = np.array(hw, np.uint8)[order]
    w.cfg_batch = np.array(bt, np.uint8)[order]
    w.cfg_replicas = np.array(rp, np.uint16)[order]
    return w, (b_hw, b_bt, b_rp), np.array(base_of, np.uint32)[order]


def backlog_case(seed):
    """A small overloaded pipeline: service times far above the arrival gaps, so queues stay long,
    batches run full and replicas rotate.  Every fourth seed quantises all times (replicas fall
    into lock step and completions tie), every seventh starts so late that queueing runs into the
    2^32-1 us horizon, every third has stages with maximum batch size 1."""
    rng = np.random.default_rng(1000 + seed)
    S = int(rng.integers(1, 4))
    n = int(rng.integers(500, 3000))
    C, H, Bmax = 4, 1, 32
    if seed % 4 == 3:
        parents = [[], [0], [0], [1, 2]]
        S = 4
    else:
        parents = [[]] + [[s - 1] for s in range(1, S)]
    quantum = [1, 10, 100, 1000][seed % 4] if seed % 2 == 0 else 1
    a = rng.integers(50, 3000, size=(S, H))
    c = rng.integers(1, 200, size=(S, H))
    lat = (a[:, :, None] + c[:, :, None] * np.arange(1, Bmax + 1)[None, None, :]).astype(np.uint32)
    lat = np.maximum(lat // quantum * quantum, quantum).astype(np.uint32)
    g = int(rng.integers(2, 400))
    gaps = rng.integers(0, g, size=n)
    if quantum > 1 and rng.random() < 0.5:
        gaps = gaps // quantum * quantum
    base = 0
    if seed % 7 == 3:
        base = 2**32 - 2 - int(gaps.sum()) - 2 * S * int(lat.max()) - 1
    arr = (base + np.cumsum(gaps)).astype(np.uint32)
    mask = np.zeros(n, np.uint32)
    for s in range(S):
        p = 1.0 if rng.random() < 0.6 else rng.uniform(0.3, 1.0)
        mask |= (rng.random(n) < p).astype(np.uint32) << np.uint32(s)
    cost = np.full((S, H), 5, np.uint64)
    hw = np.zeros((C, S), np.uint8)
    sizes = [2, 2, 3, 4, 4, 5, 8, 8, 16, 32] if seed % 3 else [1, 1, 1, 2, 4, 16]
    bt = rng.choice(sizes, size=(C, S)).astype(np.uint8)
    rp = rng.choice([1, 1, 2, 2, 3, 4, 5, 8], size=(C, S)).astype(np.uint16)
    return Workload("backlog%d" % seed, parents, lat, cost, arr, mask, hw, bt, rp, int(lat.max()))


def grouped_case(seed, n=None):
    """A small pipeline under bursts: queries arrive in groups of 4..48 at the same microsecond, the stages
    take large batches whose service time is several times the gap between groups, on enough replicas
    that every group finds one idle -- many batches are in flight at once and leave in completion order.
    Every second seed puts all times on a 100-us grid (completions tie), every third seed is the W4/W5
    fork-join shape, every fifth gives some stage too few replicas for part of the trace."""
    rng = np.random.default_rng(3000 + seed)
    n = int(rng.integers(2000, 5000)) if n is None else n
    C, H, Bmax = 4, 2, 64
    if seed % 3 == 2:
        parents = [[], [0], [1], [1], [2, 3], [4]]
    else:
        parents = [[]] + [[s - 1] for s in range(1, int(rng.integers(2, 5)))]
    S = len(parents)
    quantum = 100 if seed % 2 == 0 else 1
    a = rng.integers(8000, 40000, size=(S, H))
    c = rng.integers(50, 800, size=(S, H))
    lat = (a[:, :, None] + c[:, :, None] * np.arange(1, Bmax + 1)[None, None, :]).astype(np.uint32)
    lat = np.maximum(lat // quantum * quantum, quantum).astype(np.uint32)
    sizes = rng.integers(4, 49, size=n)
    starts = np.cumsum(rng.integers(1500, 7000, size=n) // quantum * quantum)
    arr = np.repeat(starts, sizes)[:n].astype(np.uint32)
    mask = np.zeros(n, np.uint32)
    for s in range(S):
        p = 1.0 if (rng.random() < 0.6 or s == 0 or s == S - 1) else rng.uniform(0.4, 1.0)
        mask |= (rng.random(n) < p).astype(np.uint32) << np.uint32(s)
    cost = np.full((S, H), 5, np.uint64)
    hw = rng.integers(0, H, size=(C, S)).astype(np.uint8)
    bt = rng.choice([48, 64, 64, 32], size=(C, S)).astype(np.uint8)
    rp = rng.integers(12, 17, size=(C, S)).astype(np.uint16)
    if seed % 5 == 4:
        rp[:, int(rng.integers(0, S))] = rng.integers(2, 6, size=C)
    return Workload("grouped%d" % seed, parents, lat, cost, arr, mask, hw, bt, rp, int(lat.max()) * 2)


def provisioned_case(seed, n=None):
    """A small pipeline provisioned at 80-100 % utilisation with small batches on many replicas (the
    regime around the SLO boundary): an upstream stage batches, so the next stages see groups of queries
    that become ready together and cut them into several batches started at the same instant on
    different replicas -- completions tie all the time and have to be merged by query index.  Service
    times are set from the utilisation; every third seed is a fork-join, every second quantises times."""
    rng = np.random.default_rng(4000 + seed)
    n = int(rng.integers(3000, 7000)) if n is None else n
    C, H, Bmax = 4, 1, 16
    if seed % 3 == 2:
        parents = [[], [0], [0], [1, 2], [3]]
    else:
        parents = [[]] + [[s - 1] for s in range(1, int(rng.integers(2, 5)))]
    S = len(parents)
    rate = 5000.0
    quantum = 10 if seed % 2 == 0 else 1
    gaps = np.rint(rng.gamma(0.5, 2.0 / rate, size=n) * 1e6).astype(np.int64) // quantum * quantum
    arr = np.cumsum(gaps).astype(np.uint32)
    bt = rng.choice([1, 2, 2, 4, 8], size=(C, S)).astype(np.uint8)
    rp = rng.integers(6, 33, size=(C, S)).astype(np.uint16)
    lat = np.zeros((S, H, Bmax), np.uint32)
    for s in range(S):
        b, r = int(bt[0, s]), int(rp[0, s])
        lb = r * b * float(rng.uniform(0.8, 1.0)) / rate * 1e6   # L(b) for that utilisation under the first candidate
        a = 0.6 * lb
        c = (lb - a) / b
        lat[s, 0, :] = np.maximum(np.rint(a + c * np.arange(1, Bmax + 1)) // quantum * quantum, quantum)
    mask = np.zeros(n, np.uint32)
    for s in range(S):
        p = 1.0 if (rng.random() < 0.7 or s == 0 or s == S - 1) else rng.uniform(0.5, 1.0)
        mask |= (rng.random(n) < p).astype(np.uint32) << np.uint32(s)
    cost = np.full((S, H), 5, np.uint64)
    hw = np.zeros((C, S), np.uint8)
    return Workload("prov%d" % seed, parents, lat, cost, arr, mask, hw, bt, rp, int(lat.max()) * 3)


def planner_case(seed, n=1500):
    """A small pipeline for the greedy planner: three hardware types per stage (fast and expensive,
    medium, slow and cheap -- in seeded index order), batching that amortises a fixed cost, an
    SLO of a few service times, a Poisson-like trace that needs several replicas at batch 1."""
    rng = np.random.default_rng(3000 + seed)
    S = int(rng.integers(1, 5))
    H, Bmax = 3, 16
    if S >= 3 and seed % 2 == 0:
        parents = [[], [0], [0]] + ([[1, 2]] if S == 4 else [])
    else:
        parents = [[]] + [[s - 1] for s in range(1, S)]
    speed = np.array([1.0, 2.2, 5.0])
    price = np.array([900_000, 300_000, 60_000], dtype=np.uint64)
    lat = np.zeros((S, H, Bmax), np.uint32)
    cost = np.zeros((S, H), np.uint64)
    for s in range(S):
        order = rng.permutation(H)
        fixed = float(rng.integers(300, 2000))
        per = float(rng.integers(20, 300))
        for k, h in enumerate(order):
            lat[s, h, :] = np.maximum(1, (speed[k] * (fixed + per * np.arange(1, Bmax + 1)))).astype(np.uint32)
            cost[s, h] = price[k] + int(rng.integers(0, 1000))
    gap = float(rng.integers(150, 900))
    arr = np.cumsum(rng.exponential(gap, size=n)).astype(np.uint32)
    mask = np.zeros(n, np.uint32)
    for s in range(S):
        p = 1.0 if (s == 0 or rng.random() < 0.5) else rng.uniform(0.3, 0.9)
        mask |= (rng.random(n) < p).astype(np.uint32) << np.uint32(s)
    fast = np.array([lat[s, :, 0].min() for s in range(S)], dtype=np.float64)
    slo = int(fast.sum() * float(rng.uniform(2.0, 8.0)))
    hw = np.zeros((1, S), np.uint8)
    return Workload("plan%d" % seed, parents, lat, cost, arr, mask, hw, np.ones((1, S), np.uint8), np.ones((1, S), np.uint16), slo)

