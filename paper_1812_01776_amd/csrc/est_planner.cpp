// Greedy low-frequency planner (arXiv 1812.01776, Section 4.3, Algorithms 1 and 2) on top of the
// batched Estimator: the search itself is host code, every Feasible() test is answered by the GPU
// simulation, and the candidates of one step are evaluated together in one estimator_run_dev call
// instead of one at a time.  The decisions are those of the sequential algorithm:
//   * Initialize adds a replica to the throughput bottleneck until the pipeline is feasible; the
//     bottleneck sequence does not depend on the feasibility answers, so the next 32 configurations of
//     that sequence are evaluated at once and the first feasible one is taken;
//   * DowngradeHW re-initialises one model on the next cheaper hardware by adding replicas until
//     feasible, then walks IncreaseBatch / RemoveReplica on that model alone: every configuration that
//     search can reach differs from the current one only in that model's (batch, replicas) on the
//     cheaper hardware, so that whole grid (batch 1, 2, 4, ... x replicas 1..max) is evaluated and the
//     search becomes table look-ups;
//   * one iteration of MinimizeCost evaluates IncreaseBatch and RemoveReplica of every model together
//     with the grids above in ONE call, then picks the cheapest feasible result (first in
//     (model, action) order on ties).
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/estimator.h"
#include "est_backend.h"
#include "est_handle.h"

namespace {

typedef std::vector<est_stage_cfg_t> Cfg;  // one entry per stage

struct DevMem {  // device memory freed on every path out
    void *p;
    explicit DevMem(size_t bytes) : p(bytes ? estbe::dmalloc(bytes) : nullptr) {}
    ~DevMem() {
        if (p) estbe::dfree(p);
    }
    DevMem(const DevMem &) = delete;
    DevMem &operator=(const DevMem &) = delete;
};

struct Planner {
    estimator *h;
    uint32_t S, H, Bmax, rmax, slo;
    uint64_t n;
    const uint32_t *d_arr = nullptr, *d_mask = nullptr;
    std::vector<uint64_t> visits;
    uint32_t calls = 0;
    uint64_t candidates = 0;
    int err = EST_OK;

    uint32_t lat(uint32_t s, uint32_t hw, uint32_t b) const { return h->lat[((size_t)s * H + hw) * Bmax + (b - 1)]; }
    uint64_t price(uint32_t s, uint32_t hw) const { return h->cost[(size_t)s * H + hw]; }
    uint64_t cost(const Cfg &c) const {
        uint64_t t = 0;
        for (uint32_t s = 0; s < S; ++s) t += (uint64_t)c[s].replicas * price(s, c[s].hw);
        return t;
    }

    // One Estimator call: P99 of every candidate.  Returns false (err set) on failure.
    bool evaluate(const std::vector<Cfg> &cands, std::vector<uint32_t> &p99) {
        p99.assign(cands.size(), 0);
        if (cands.empty()) return true;
        const uint64_t C = cands.size();
        std::vector<est_stage_cfg_t> flat(C * S);
        for (uint64_t i = 0; i < C; ++i) memcpy(&flat[i * S], cands[i].data(), S * sizeof(est_stage_cfg_t));
        DevMem m_cfg(C * S * sizeof(est_stage_cfg_t)), m_p99(C * 4), m_miss(C * 4), m_cost(C * 8);
        void *d_cfg = m_cfg.p, *d_p99 = m_p99.p, *d_miss = m_miss.p, *d_cost = m_cost.p;
        bool ok = d_cfg && d_p99 && d_miss && d_cost;
        if (!ok) {
            err = EST_ENOMEM;
            h->err = "planner: device allocation failed";
        }
        if (ok && (estbe::h2d(d_cfg, flat.data(), C * S * sizeof(est_stage_cfg_t), nullptr) || estbe::sync(nullptr))) {
            ok = false;
            err = EST_EDEVICE;
            h->err = std::string("planner: upload configurations: ") + estbe::last_error();
        }
        if (ok) {
            est_trace_t tr;
            tr.n = n;
            tr.arrival_us = d_arr;
            tr.visit_mask = d_mask;
            est_result_t out;
            out.p99_us = (uint32_t *)d_p99;
            out.miss_count = (uint32_t *)d_miss;
            out.cost_uusd_hr = (uint64_t *)d_cost;
            const int rc = estimator_run_dev(h, &tr, (const est_stage_cfg_t *)d_cfg, C, slo, &out, nullptr, 0, nullptr);
            if (rc != EST_OK) {
                ok = false;
                err = rc;
            } else if (estbe::d2h(p99.data(), d_p99, C * 4, nullptr) || estbe::sync(nullptr)) {
                ok = false;
                err = EST_EDEVICE;
                h->err = std::string("planner: download results: ") + estbe::last_error();
            }
        }
        ++calls;
        candidates += C;
        return ok;
    }

    // ---- Algorithm 1
    uint32_t best_hw(uint32_t s) const {
        uint32_t b = 0;
        for (uint32_t k = 1; k < H; ++k)
            if (lat(s, k, 1) < lat(s, b, 1)) b = k;
        return b;
    }
    uint64_t service_time(const Cfg &c) const {  // longest path of batch-1 latencies
        std::vector<uint64_t> longest(S, 0);
        uint64_t best = 0;
        for (uint32_t s = 0; s < S; ++s) {
            uint64_t up = 0;
            for (uint32_t e = h->dag.parent_off[s]; e < h->dag.parent_off[s + 1]; ++e) up = std::max(up, longest[h->dag.parent_idx[e]]);
            longest[s] = up + lat(s, c[s].hw, 1);
            best = std::max(best, longest[s]);
        }
        return best;
    }
    // the stage with the smallest replicas * batch / (latency * visits); -1 if nobody visits anything
    int find_min_thru(const Cfg &c) const {
        int best = -1;
        for (uint32_t s = 0; s < S; ++s) {
            if (visits[s] == 0) continue;
            if (best < 0) {
                best = (int)s;
                continue;
            }
            const unsigned __int128 lhs = (unsigned __int128)((uint64_t)c[s].replicas * c[s].batch) * lat(best, c[best].hw, c[best].batch) * visits[best];
            const unsigned __int128 rhs = (unsigned __int128)((uint64_t)c[best].replicas * c[best].batch) * lat(s, c[s].hw, c[s].batch) * visits[s];
            if (lhs < rhs) best = (int)s;
        }
        return best;
    }
    // 1 = found (cfg updated), 0 = no feasible configuration, -1 = error
    int initialize(Cfg &cfg) {
        cfg.resize(S);
        for (uint32_t s = 0; s < S; ++s) {
            cfg[s].hw = (uint8_t)best_hw(s);
            cfg[s].batch = 1;
            cfg[s].replicas = 1;
        }
        if (service_time(cfg) > slo) return 0;
        for (;;) {
            // the next configurations on the bottleneck path
            std::vector<Cfg> path;
            path.push_back(cfg);
            bool dead = false;
            while (path.size() < 32) {
                Cfg nx = path.back();
                const int s = find_min_thru(nx);
                if (s < 0 || nx[s].replicas >= rmax) {
                    dead = true;
                    break;
                }
                nx[s].replicas++;
                path.push_back(nx);
            }
            std::vector<uint32_t> p99;
            if (!evaluate(path, p99)) return -1;
            for (size_t i = 0; i < path.size(); ++i)
                if (p99[i] <= slo) {
                    cfg = path[i];
                    return 1;
                }
            if (dead) return 0;
            // continue one step beyond the last configuration evaluated
            cfg = path.back();
            const int s = find_min_thru(cfg);
            if (s < 0 || cfg[s].replicas >= rmax) return 0;
            cfg[s].replicas++;
        }
    }

    // ---- the actions of Algorithm 2
    bool increase_batch(const Cfg &c, uint32_t s, Cfg &out) const {
        if (2u * c[s].batch > Bmax) return false;
        out = c;
        out[s].batch = (uint8_t)(2u * c[s].batch);
        return true;
    }
    bool remove_replica(const Cfg &c, uint32_t s, Cfg &out) const {
        if (c[s].replicas <= 1) return false;
        out = c;
        out[s].replicas--;
        return true;
    }
    int cheaper_hw(const Cfg &c, uint32_t s) const {  // the most expensive strictly cheaper type, -1 if none
        int pick = -1;
        for (uint32_t k = 0; k < H; ++k) {
            if (price(s, k) >= price(s, c[s].hw)) continue;
            if (pick < 0 || price(s, k) > price(s, (uint32_t)pick)) pick = (int)k;
        }
        return pick;
    }
};

}  // namespace

extern "C" int estimator_plan(estimator_t *h, const est_trace_t *trace, uint32_t slo_us, uint32_t max_replicas,
                              est_stage_cfg_t *config_out, est_plan_result_t *result, est_plan_step_t *steps_out,
                              uint32_t steps_cap) {
    if (!h) return EST_EINVAL;
    auto bad = [&](const char *msg) {
        h->err = msg;
        return EST_EINVAL;
    };
    if (!trace || !config_out || !result) return bad("planner: NULL argument");
    if (trace->n > 0 && (!trace->arrival_us || !trace->visit_mask)) return bad("planner: trace arrays are NULL");
    if (max_replicas < 1 || max_replicas > EST_MAX_REPLICAS) return bad("planner: max_replicas out of range");
    if (steps_cap > 0 && !steps_out) return bad("planner: steps_out is NULL");
    if (trace->n >= (1ull << 31)) return bad("planner: trace too large");
    for (uint64_t q = 1; q < trace->n; ++q)
        if (trace->arrival_us[q] < trace->arrival_us[q - 1]) return bad("planner: arrival times decrease");
    try {
        Planner P;
        P.h = h;
        P.S = h->dag.S;
        P.H = h->dag.H;
        P.Bmax = h->dag.Bmax;
        P.rmax = max_replicas;
        P.slo = slo_us;
        P.n = trace->n;
        P.visits.assign(P.S, 0);
        for (uint64_t q = 0; q < trace->n; ++q)
            for (uint32_t s = 0; s < P.S; ++s) P.visits[s] += (trace->visit_mask[q] >> s) & 1u;
        DevMem m_arr(trace->n * 4), m_mask(trace->n * 4);
        if (trace->n > 0) {
            if (!m_arr.p || !m_mask.p || estbe::h2d(m_arr.p, trace->arrival_us, trace->n * 4, nullptr) ||
                estbe::h2d(m_mask.p, trace->visit_mask, trace->n * 4, nullptr) || estbe::sync(nullptr)) {
                h->err = "planner: cannot place the trace on the device";
                return EST_ENOMEM;
            }
        }
        P.d_arr = (const uint32_t *)m_arr.p;
        P.d_mask = (const uint32_t *)m_mask.p;

        uint32_t n_steps = 0;
        auto log_step = [&](uint32_t action, int32_t stage, uint64_t cost) {
            if (n_steps < steps_cap) {
                steps_out[n_steps].action = action;
                steps_out[n_steps].stage = stage;
                steps_out[n_steps].cost_uusd_hr = cost;
            }
            ++n_steps;
        };

        Cfg cfg;
        const int init = P.initialize(cfg);
        if (init < 0) return P.err;
        memset(result, 0, sizeof *result);
        if (init == 0) {
            result->estimator_calls = P.calls;
            result->candidates = P.candidates;
            return EST_OK;  // feasible stays 0
        }
        log_step(EST_PLAN_INIT, -1, P.cost(cfg));

        for (;;) {
            // -- candidates of this iteration: per model IncreaseBatch and RemoveReplica, and for DowngradeHW the
            //    whole (batch, replicas) grid of that model on the cheaper hardware.  The action's replica search
            //    and its local search only ever visit grid points, so one batched Estimator call answers every
            //    question the iteration can ask and the walk itself runs on the host from the table.
            std::vector<Cfg> cands;
            std::vector<int> idx_inc(P.S, -1), idx_rem(P.S, -1), idx_down(P.S, -1), hw2(P.S, -1);
            uint32_t nb = 0;  // batch sizes 1, 2, 4, ... that fit the profile
            while ((2u << nb) <= P.Bmax) ++nb;
            ++nb;
            for (uint32_t s = 0; s < P.S; ++s) {
                Cfg c;
                if (P.increase_batch(cfg, s, c)) {
                    idx_inc[s] = (int)cands.size();
                    cands.push_back(c);
                }
                if (P.remove_replica(cfg, s, c)) {
                    idx_rem[s] = (int)cands.size();
                    cands.push_back(c);
                }
                hw2[s] = P.cheaper_hw(cfg, s);
                if (hw2[s] >= 0) {
                    idx_down[s] = (int)cands.size();
                    for (uint32_t k = 0; k < nb; ++k)
                        for (uint32_t r = 1; r <= P.rmax; ++r) {
                            c = cfg;
                            c[s].hw = (uint8_t)hw2[s];
                            c[s].batch = (uint8_t)(1u << k);
                            c[s].replicas = (uint16_t)r;
                            cands.push_back(c);
                        }
                }
            }
            std::vector<uint32_t> p99;
            if (!P.evaluate(cands, p99)) return P.err;
            // -- DowngradeHW: smallest feasible replica count at batch 1, then IncreaseBatch / RemoveReplica on
            //    that model alone while one of them stays feasible (the cheaper of the two, the larger batch when
            //    they cost the same)
            std::vector<Cfg> local(P.S);
            std::vector<char> alive(P.S, 0);
            for (uint32_t s = 0; s < P.S; ++s) {
                if (idx_down[s] < 0) continue;
                auto at = [&](uint32_t k, uint32_t r) { return (size_t)idx_down[s] + (size_t)k * P.rmax + (r - 1); };
                uint32_t k = 0, r = 1;
                while (r <= P.rmax && p99[at(0, r)] > P.slo) ++r;
                if (r > P.rmax) continue;
                const bool removal_is_cheaper = P.price(s, (uint32_t)hw2[s]) > 0;
                for (;;) {
                    const bool inc_ok = k + 1 < nb && p99[at(k + 1, r)] <= P.slo;
                    const bool rem_ok = r > 1 && p99[at(k, r - 1)] <= P.slo;
                    if (rem_ok && (!inc_ok || removal_is_cheaper))
                        --r;
                    else if (inc_ok)
                        ++k;
                    else
                        break;
                }
                local[s] = cands[at(k, r)];
                alive[s] = 1;
            }
            // -- the cheapest feasible result, first in (model, action) order on ties
            const uint64_t cur = P.cost(cfg);
            bool have = false;
            Cfg best;
            uint64_t best_cost = 0;
            uint32_t best_action = 0;
            int32_t best_stage = -1;
            auto consider = [&](const Cfg &c, uint32_t action, uint32_t s) {
                const uint64_t k = P.cost(c);
                if (!have || k < best_cost) {
                    have = true;
                    best = c;
                    best_cost = k;
                    best_action = action;
                    best_stage = (int32_t)s;
                }
            };
            for (uint32_t s = 0; s < P.S; ++s) {
                if (idx_inc[s] >= 0 && p99[idx_inc[s]] <= P.slo) consider(cands[idx_inc[s]], EST_PLAN_INCREASE_BATCH, s);
                if (idx_rem[s] >= 0 && p99[idx_rem[s]] <= P.slo) consider(cands[idx_rem[s]], EST_PLAN_REMOVE_REPLICA, s);
                if (alive[s] && P.cost(local[s]) < cur) consider(local[s], EST_PLAN_DOWNGRADE_HW, s);
            }
            if (!have) break;
            cfg = best;
            log_step(best_action, best_stage, best_cost);
        }
        // the answer, with its P99
        std::vector<Cfg> fin(1, cfg);
        std::vector<uint32_t> fp;
        if (!P.evaluate(fin, fp)) return P.err;
        memcpy(config_out, cfg.data(), P.S * sizeof(est_stage_cfg_t));
        result->feasible = 1;
        result->n_steps = n_steps;
        result->estimator_calls = P.calls;
        result->candidates = P.candidates;
        result->cost_uusd_hr = P.cost(cfg);
        result->p99_us = fp[0];
        return EST_OK;
    } catch (const std::bad_alloc &) {
        h->err = "planner: host allocation failed";
        return EST_ENOMEM;
    } catch (...) {
        h->err = "planner: unexpected exception";
        return EST_EINTERNAL;
    }
}

// ---- hand-off to the tuner: traffic envelope (one kernel over the trace) and per-model ratios
extern "C" int estimator_tuner_handoff(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *config,
                                       uint32_t service_time_us, est_handoff_t *out) {
    if (!h) return EST_EINVAL;
    auto bad = [&](const char *msg) {
        h->err = msg;
        return EST_EINVAL;
    };
    if (!trace || !config || !out) return bad("handoff: NULL argument");
    if (trace->n > 0 && (!trace->arrival_us || !trace->visit_mask)) return bad("handoff: trace arrays are NULL");
    if (service_time_us == 0) return bad("handoff: service time must be positive");
    if (trace->n >= (1ull << 31)) return bad("handoff: trace too large");
    const uint32_t S = h->dag.S, H = h->dag.H, Bmax = h->dag.Bmax;
    for (uint32_t s = 0; s < S; ++s)
        if (config[s].hw >= H || config[s].batch < 1 || config[s].batch > Bmax || config[s].replicas < 1 || config[s].replicas > EST_MAX_REPLICAS)
            return bad("handoff: configuration entry out of range");
    for (uint64_t q = 1; q < trace->n; ++q)
        if (trace->arrival_us[q] < trace->arrival_us[q - 1]) return bad("handoff: arrival times decrease");
    est_handoff_t r;
    memset(&r, 0, sizeof r);
    for (uint64_t w = service_time_us; r.n_windows < EST_MAX_WINDOWS && (r.n_windows == 0 || w <= 60000000ull); w *= 2)
        r.window_us[r.n_windows++] = w;
    if (trace->n > 0) {
        EstEnvArgs a;
        memset(&a, 0, sizeof a);
        DevMem m_arr(trace->n * 4), m_q(EST_MAX_WINDOWS * 4);
        void *d_arr = m_arr.p, *d_q = m_q.p;
        int rc = EST_OK;
        if (!d_arr || !d_q) {
            h->err = "handoff: device allocation failed";
            rc = EST_ENOMEM;
        } else if (estbe::h2d(d_arr, trace->arrival_us, trace->n * 4, nullptr) || estbe::zero(d_q, EST_MAX_WINDOWS * 4, nullptr)) {
            h->err = std::string("handoff: upload: ") + estbe::last_error();
            rc = EST_EDEVICE;
        } else {
            a.arrival = (const uint32_t *)d_arr;
            a.n = trace->n;
            a.n_win = r.n_windows;
            for (uint32_t i = 0; i < r.n_windows; ++i) a.win_us[i] = r.window_us[i];
            a.max_queries = (uint32_t *)d_q;
            if (estbe::launch_envelope(a, nullptr) || estbe::d2h(r.max_queries, d_q, r.n_windows * 4, nullptr) || estbe::sync(nullptr)) {
                h->err = std::string("handoff: envelope kernel: ") + estbe::last_error();
                rc = EST_EDEVICE;
            }
        }
        if (rc != EST_OK) return rc;
    }
    const uint64_t span = trace->n > 0 ? (uint64_t)trace->arrival_us[trace->n - 1] - trace->arrival_us[0] : 0;
    for (uint32_t s = 0; s < S; ++s) {
        uint64_t visits = 0;
        for (uint64_t q = 0; q < trace->n; ++q) visits += (trace->visit_mask[q] >> s) & 1u;
        const uint64_t L = h->lat[((size_t)s * H + config[s].hw) * Bmax + (config[s].batch - 1)];
        r.mu_num[s] = (uint64_t)config[s].batch * 1000000ull;
        r.mu_den[s] = L;
        // lambda s_m / (R mu_m) = (n / span) (visits / n) / (R batch / L) = visits L / (span R batch)   (times in us cancel)
        // (a trace that spans no time has no rate: 0 / 0, which the caller must test for before dividing)
        r.rho_num[s] = span ? visits * L : 0;
        r.rho_den[s] = span * config[s].replicas * config[s].batch;
    }
    *out = r;
    return EST_OK;
}


// ---- latency tables for models whose latency depends on the input (Section 8, second limitation): the profile
//      entry is the tail of the latencies measured over the sample queries.  Host code, exact integer arithmetic.
extern "C" int estimator_profile_tail(const uint32_t *samples_us, uint64_t n_entries, uint32_t n_samples, uint32_t mode,
                                      uint32_t param, uint32_t *lat_us_out) {
    if (n_entries == 0) return EST_OK;
    if (!samples_us || !lat_us_out) return EST_EINVAL;
    if (n_samples < 1 || n_samples > EST_MAX_PROFILE_SAMPLES) return EST_EINVAL;
    if (mode != EST_TAIL_PERCENTILE && mode != EST_TAIL_SIGMA) return EST_EINVAL;
    if (mode == EST_TAIL_PERCENTILE && (param < 1 || param > 10000)) return EST_EINVAL;
    if (mode == EST_TAIL_SIGMA && param > 10000) return EST_EINVAL;
    typedef unsigned __int128 u128;
    std::vector<uint32_t> res, v;
    try {
        res.resize(n_entries);
        v.resize(n_samples);
    } catch (const std::bad_alloc &) {
        return EST_ENOMEM;
    }
    const uint64_t n = n_samples;
    for (uint64_t e = 0; e < n_entries; ++e) {
        const uint32_t *x = samples_us + e * n;
        if (mode == EST_TAIL_PERCENTILE) {
            // nearest rank: the k-th smallest, k = ceil(param x n / 10000)
            const uint64_t k = ((uint64_t)param * n + 9999) / 10000;
            std::copy(x, x + n, v.begin());
            std::nth_element(v.begin(), v.begin() + (k - 1), v.end());
            res[e] = v[k - 1];
        } else {
            // the smallest integer t with t >= mean + (param / 1000) sigma, sigma^2 = (n S2 - S1^2) / n^2:
            //   n t - S1 >= (param / 1000) sqrt(D), D = n S2 - S1^2   <=>   (1000 (n t - S1))^2 >= param^2 D  (left side >= 0)
            u128 s1 = 0, s2 = 0;
            for (uint64_t i = 0; i < n; ++i) {
                s1 += x[i];
                s2 += (u128)x[i] * x[i];
            }
            const u128 D = (u128)n * s2 - s1 * s1, rhs = (u128)param * param * D;
            uint64_t lo = (uint64_t)((s1 + n - 1) / n), hi = 1ull << 36;  // t >= ceil(mean); sigma <= half the range, so mean + 10 sigma < 2^36
            while (lo < hi) {  // (the left side grows with t)
                const uint64_t t = lo + (hi - lo) / 2;
                const u128 a = ((u128)n * t - s1) * 1000u;
                if (a * a >= rhs) hi = t; else lo = t + 1;
            }
            if (lo > 0xFFFFFFFFull) return EST_EINVAL;  // does not fit a latency
            res[e] = (uint32_t)lo;
        }
        if (res[e] == 0) return EST_EINVAL;  // a latency table has no zero entries
    }
    std::copy(res.begin(), res.end(), lat_us_out);
    return EST_OK;
}
