"""Plain sequential reference of the greedy low-frequency planner (arXiv 1812.01776, Section 4.3,
Algorithms 1 and 2), one Estimator call per candidate, every call answered by the CPU oracle.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing else); the library's own planner
(estimator_plan) shares no code with it.

What the paper fixes and what is read into it (the same readings are stated in the design notes):
  * Feasible(config)      <=>  nearest-rank P99 of the Estimator's latencies <= SLO (Section 2, 4.3).
  * BestHardware(model)   = the hardware type with the smallest batch-1 latency (lowest index on ties).
  * ServiceTime(pipeline) = sum of batch-1 latencies along the longest path of the DAG (Section 4.3);
                            the SLO is unattainable when it exceeds the SLO.
  * FindMinThru           = the stage with the smallest sustainable pipeline throughput
                            replicas * batch / latency(batch) / scale factor, scale factor = fraction of
                            the trace's queries that visit the stage (Section 4.1); exact rational
                            comparison, lowest index on ties; stages nobody visits are ignored.
  * IncreaseBatch doubles the maximum batch size (Section 4.3), RemoveReplica removes one replica,
    DowngradeHW moves the model to the next cheaper hardware type (the most expensive among the
    strictly cheaper ones, lowest index on ties), restarts that model at batch 1 / 1 replica, adds
    replicas to it until the pipeline is feasible again, then greedily applies IncreaseBatch /
    RemoveReplica to that model alone while they stay feasible; it is rejected unless the result
    is strictly cheaper than the configuration it started from.
  * One iteration of Algorithm 2 takes, among all feasible results of the 3 actions on every model,
    the cheapest one (the first in (model, action) order on ties; actions in the order IncreaseBatch,
    RemoveReplica, DowngradeHW), and the search ends when no action yields a feasible result.
"""
import numpy as np

from . import oracle


class PlannerOracle:
    def __init__(self, parents, lat_us, cost_uusd_hr, arrival_us, visit_mask, slo_us, max_replicas=64):
        self.parents = [list(p) for p in parents]
        self.lat = np.asarray(lat_us, dtype=np.uint32)
        self.price = np.asarray(cost_uusd_hr, dtype=np.uint64)
        self.arr = np.asarray(arrival_us, dtype=np.uint32)
        self.mask = np.asarray(visit_mask, dtype=np.uint32)
        self.slo = int(slo_us)
        self.rmax = int(max_replicas)
        self.S, self.H, self.bmax = self.lat.shape
        self.visits = [int(((self.mask >> np.uint32(s)) & 1).sum()) for s in range(self.S)]
        self.calls = 0
        self.log = []

    # ---- the Estimator, one candidate per call
    def p99(self, cfg):
        self.calls += 1
        hw = np.array([[c[0] for c in cfg]], np.uint8)
        bt = np.array([[c[1] for c in cfg]], np.uint8)
        rp = np.array([[c[2] for c in cfg]], np.uint16)
        r = oracle.run(self.parents, self.lat, self.price, self.arr, self.mask, hw, bt, rp, self.slo)
        return int(r["p99_us"][0])

    def feasible(self, cfg):
        return self.p99(cfg) <= self.slo

    def cost(self, cfg):
        return sum(int(c[2]) * int(self.price[s, c[0]]) for s, c in enumerate(cfg))

    # ---- Algorithm 1
    def best_hw(self, s):
        return int(np.argmin(self.lat[s, :, 0]))  # argmin returns the first minimum

    def service_time(self, cfg):
        longest = [0] * self.S
        for s in range(self.S):
            up = max([longest[p] for p in self.parents[s]], default=0)
            longest[s] = up + int(self.lat[s, cfg[s][0], 0])
        return max(longest)

    def find_min_thru(self, cfg):
        best = None
        for s in range(self.S):
            if self.visits[s] == 0:
                continue
            if best is None:
                best = s
                continue
            hs, bs, rs = cfg[s]
            hb, bb, rb = cfg[best]
            ls, lb = int(self.lat[s, hs, bs - 1]), int(self.lat[best, hb, bb - 1])
            # thru(s) < thru(best)  <=>  rs*bs/(ls*vs) < rb*bb/(lb*vb)
            if rs * bs * lb * self.visits[best] < rb * bb * ls * self.visits[s]:
                best = s
        return best

    def initialize(self):
        cfg = [(self.best_hw(s), 1, 1) for s in range(self.S)]
        if self.service_time(cfg) > self.slo:
            return None
        while not self.feasible(cfg):
            s = self.find_min_thru(cfg)
            if s is None or cfg[s][2] >= self.rmax:
                return None
            cfg[s] = (cfg[s][0], cfg[s][1], cfg[s][2] + 1)
        return cfg

    # ---- the three actions of Algorithm 2
    def increase_batch(self, cfg, s):
        h, b, r = cfg[s]
        if 2 * b > self.bmax:
            return None
        new = list(cfg)
        new[s] = (h, 2 * b, r)
        return new

    def remove_replica(self, cfg, s):
        h, b, r = cfg[s]
        if r <= 1:
            return None
        new = list(cfg)
        new[s] = (h, b, r - 1)
        return new

    def downgrade_hw(self, cfg, s):
        h = cfg[s][0]
        cheaper = [k for k in range(self.H) if int(self.price[s, k]) < int(self.price[s, h])]
        if not cheaper:
            return None
        top = max(int(self.price[s, k]) for k in cheaper)
        h2 = min(k for k in cheaper if int(self.price[s, k]) == top)
        new = list(cfg)
        new[s] = (h2, 1, 1)
        while not self.feasible(new):
            if new[s][2] >= self.rmax:
                return None
            new[s] = (h2, 1, new[s][2] + 1)
        while True:
            best = None
            for act in (self.increase_batch, self.remove_replica):
                cand = act(new, s)
                if cand is not None and self.feasible(cand) and (best is None or self.cost(cand) < self.cost(best)):
                    best = cand
            if best is None:
                break
            new = best
        return new if self.cost(new) < self.cost(cfg) else None

    # ---- Algorithm 2
    def minimize_cost(self):
        cfg = self.initialize()
        if cfg is None:
            return None
        self.log.append(("init", -1, self.cost(cfg), [tuple(c) for c in cfg]))
        while True:
            best, tag = None, None
            for s in range(self.S):
                for name, act in (("batch", self.increase_batch), ("replica", self.remove_replica), ("hw", self.downgrade_hw)):
                    cand = act(cfg, s)
                    if cand is None:
                        continue
                    if name != "hw" and not self.feasible(cand):
                        continue
                    if best is None or self.cost(cand) < self.cost(best):
                        best, tag = cand, (name, s)
            if best is None:
                return cfg
            cfg = best
            self.log.append((tag[0], tag[1], self.cost(cfg), [tuple(c) for c in cfg]))
