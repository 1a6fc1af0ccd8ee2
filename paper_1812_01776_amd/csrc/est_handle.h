// The handle behind estimator_t, shared by the host planner of the simulation (est_host.cpp) and
// the greedy configuration planner (est_planner.cpp).
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/estimator.h"
#include "est_types.h"

struct estimator {
    EstDag dag;
    std::vector<uint32_t> lat;
    std::vector<uint64_t> cost;
    uint64_t sum_max_lat = 0;  // sum over stages of the largest profiled latency
    EstDag *d_dag = nullptr;
    uint32_t *d_lat = nullptr;
    uint64_t *d_cost = nullptr;
    EstPlan *d_plan = nullptr;
    EstStatus *d_status = nullptr;
    // made once, so that a run that must not allocate has them: events, page-locked staging for the plan
    // going up and the status words coming back
    void *ev[8] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    struct Staging { EstStatus st[2]; EstPlan plan; } *pin = nullptr;
    void *ws = nullptr;  // scratch allocated by the library when the caller passes none
    size_t ws_bytes = 0;
    std::string err;
    est_stats_t stats;
    bool have_stats = false;
};
