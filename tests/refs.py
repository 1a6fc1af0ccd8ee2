"""Independent, deliberately naive re-statements of the Estimator's semantics
(arXiv 1812.01776, Section 4.2) used only to pin the C oracle.  None of them shares code
with the oracle or with the GPU path.

  lindley            textbook single-server recursion (R=1, B=1, one stage)
  tick_sim           1-us time-stepped simulator, polling instead of events (tiny inputs)
  stage_scan_sim     per-stage formulation: each stage only needs its own sorted ready stream
"""
import numpy as np


def lindley(arrival, D):
    done = []
    prev = 0
    for t in arrival:
        prev = max(prev, int(t)) + D
        done.append(prev)
    return np.array(done, dtype=np.int64)


def _children(parents):
    ch = [[] for _ in parents]
    for c, ps in enumerate(parents):
        for p in ps:
            ch[p].append(c)
    return ch


def tick_sim(parents, lat_us, arrival, mask, hw, batch, replicas, horizon=None):
    """Advance a clock 1 us at a time.  At each tick: finish batches that end now, admit
    arrivals, poll every (stage, query) pair for 'all parents finished', then dispatch."""
    S = len(parents)
    n = len(arrival)
    ch = _children(parents)
    done = [[None] * n for _ in range(S)]
    ready = [[None] * n for _ in range(S)]
    waiting = [[] for _ in range(S)]       # (ready, q)
    running = [[] for _ in range(S)]       # (end, [members])
    idle = [int(r) for r in replicas]
    arrived = [False] * n
    n_final = 0
    t = 0
    sinks = [s for s in range(S) if not ch[s]]
    while n_final < n:
        if horizon is not None and t > horizon:
            raise AssertionError("tick_sim ran past the horizon")
        for s in range(S):
            still = []
            for end, members in running[s]:
                if end == t:
                    idle[s] += 1
                    for q in members:
                        done[s][q] = t
                else:
                    still.append((end, members))
            running[s] = still
        for q in range(n):
            if not arrived[q] and int(arrival[q]) == t:
                arrived[q] = True
        changed = True
        while changed:
            changed = False
            for c in range(S):
                for q in range(n):
                    if ready[c][q] is not None or not arrived[q]:
                        continue
                    if parents[c]:
                        if any(done[p][q] is None for p in parents[c]):
                            continue
                        r = max(done[p][q] for p in parents[c])
                    else:
                        r = int(arrival[q])
                    ready[c][q] = r
                    changed = True
                    if (int(mask[q]) >> c) & 1:
                        waiting[c].append((r, q))
                    else:
                        done[c][q] = r
        for s in range(S):
            waiting[s].sort()
            while idle[s] > 0 and waiting[s]:
                b = min(int(batch[s]), len(waiting[s]))
                members = [q for _, q in waiting[s][:b]]
                waiting[s] = waiting[s][b:]
                end = t + int(lat_us[s][int(hw[s])][b - 1])
                if horizon is not None:
                    end = min(end, horizon)
                running[s].append((end, members))
                idle[s] -= 1
        n_final = sum(1 for q in range(n) if all(done[s][q] is not None for s in sinks))
        # a batch clamped to the current tick must be finished before the clock moves on
        if not any(end == t for s in range(S) for end, _ in running[s]):
            t += 1
    lat = np.array([max(done[s][q] for s in sinks) - int(arrival[q]) for q in range(n)], dtype=np.int64)
    return lat, np.array(done, dtype=np.int64)


def stage_scan_sim(parents, lat_us, arrival, mask, hw, batch, replicas, horizon=2**32 - 1):
    """Feed-forward DAG with unbounded queues: stage s depends only on its own ready stream.
    Sort the visiting queries by (ready, qid) and form batches greedily against the multiset
    of replica free times."""
    S = len(parents)
    n = len(arrival)
    ch = _children(parents)
    arrival = [int(a) for a in arrival]
    done = [[0] * n for _ in range(S)]
    for s in range(S):
        if parents[s]:
            ready = [max(done[p][q] for p in parents[s]) for q in range(n)]
        else:
            ready = list(arrival)
        order = sorted((ready[q], q) for q in range(n) if (int(mask[q]) >> s) & 1)
        for q in range(n):
            if not (int(mask[q]) >> s) & 1:
                done[s][q] = ready[q]
        free = [0] * int(replicas[s])
        B = int(batch[s])
        L = lat_us[s][int(hw[s])]
        i = 0
        m = len(order)
        while i < m:
            j = min(range(len(free)), key=lambda r: free[r])
            T = max(free[j], order[i][0])
            b = 1
            while b < B and i + b < m and order[i + b][0] <= T:
                b += 1
            end = min(T + int(L[b - 1]), horizon)
            free[j] = end
            for k in range(i, i + b):
                done[s][order[k][1]] = end
            i += b
    sinks = [s for s in range(S) if not ch[s]]
    lat = np.array([max(done[s][q] for s in sinks) - arrival[q] for q in range(n)], dtype=np.int64)
    return lat, np.array(done, dtype=np.int64)
