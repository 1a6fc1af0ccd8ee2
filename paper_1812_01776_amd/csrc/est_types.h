// Internal data structures shared by the host planner and the device code.
#pragma once
#include <stdint.h>

#include "../../include/estimator.h"  // EST_MAX_STAGES and the other public limits

#define EST_WAVE 64
#define EST_DBG_WORDS 16          // diagnostics: words per candidate and stage
#define EST_MW_WAVES 4            // wavefronts that share one candidate in calls that leave the device mostly empty
#define EST_KMAX EST_MAX_MERGE_SOURCES   // sources of one merge operation (accept masks are 8 bits)
#define EST_MAX_OPS 72          // <= 2 per stage + the latency sink
#define EST_MAX_RINGS 66
#define EST_MAX_EDGES (EST_MAX_OPS * EST_KMAX)
#define EST_MAX_CONS 36         // consumers of one ring
#define EST_TRACE_BIT 32        // bit of the "arrival trace" pseudo-source in a source set
#define EST_SRC_TRACE (-1)
#define EST_LDS_MERGE_BYTES(k) ((k) * 1664u)   // LDS of one wavefront for a k-source merge: staged keys 128 x 8, passed-on keys 64 x 8, accept masks 128 per source
#define EST_LDS_SCAN_BYTES(rb, ring) (1440u + 8u * (ring) + 4u * (rb))   // ... for a scan whose replica slots hold rb members and whose in-ring holds ring keys (128 or 256)

enum { EST_OP_SCAN = 0, EST_OP_MERGE = 1, EST_OP_LAT = 2 };

// One stream between operations: a power-of-two ring of (time << 32 | query) keys per candidate.
struct EstRing {
    uint64_t off;       // element offset inside one candidate's ring area
    uint32_t cap_mask;  // capacity - 1
    uint32_t n_cons;
    uint16_t cons_edge[EST_MAX_CONS];  // read cursors of the ring's consumers
};

struct EstOp {
    uint32_t type;      // EST_OP_*
    uint32_t stage;     // SCAN: the stage simulated; MERGE: the stage fed; LAT: unused
    uint32_t n_src;
    int32_t src_ring[EST_KMAX];   // ring index or EST_SRC_TRACE
    uint32_t src_edge[EST_KMAX];  // index of this consumer's read cursor
    int32_t out_ring;             // -1 for LAT
    uint32_t acc_idx;             // MERGE/LAT: which accept-mask array [n] to use
    uint32_t has_cnt;             // MERGE/LAT: some query draws from more than one source
    uint64_t tab_off;             // MERGE/LAT: byte offset of this op's time tables inside one candidate's table area
    uint32_t tab_mask;            // MERGE/LAT: bit j = source j feeds some query together with another source and has a
                                  // table (uint32 [tab_len], indexed by query: the time of the query's element in source j)
    uint32_t tab_len;             // MERGE/LAT: entries of one table (queries, rounded up)
    uint32_t rep_off;             // SCAN: word offset of the replica table inside one candidate's area
    uint32_t r_max;               // SCAN: replica table width (largest replica count of the stage in this run)
    uint64_t slot_off;            // SCAN: word offset of the member slots inside one candidate's slot area
    uint32_t b_max;               // SCAN: slot width (largest max-batch of the stage in this run)
    uint32_t filtered;            // SCAN: only the source elements whose accept mask has bit 0 set visit the stage
    uint32_t owner;               // which wavefront of the workgroup runs the operation when a candidate has several (0 .. EST_MW_WAVES-1)
    uint32_t pad;
};

struct EstPlan {
    uint32_t n_ops, n_rings, n_edges, state_words;
    // state words of one candidate: wr[n_rings] | fin[n_rings] | rd[n_edges] | opdone[n_ops] | miss, latency count | pub[n_rings]
    uint32_t wr_off, fin_off, rd_off, done_off, miss_off, max_src, pub_off, scan_ring;  // max_src: widest merge; pub: published prefix of each ring; scan_ring: keys in a scan's LDS in-ring
    EstOp ops[EST_MAX_OPS];
    EstRing rings[EST_MAX_RINGS];
};

// Output of the trace / configuration scan that the host needs to build a plan.
struct EstStatus {
    uint64_t src_union[EST_MAX_STAGES + 1];  // per stage (and the sink): union of nearest-visited-ancestor sets
    uint32_t multi[EST_MAX_STAGES + 1];      // some visiting query has more than one such ancestor
    uint64_t multi_union[EST_MAX_STAGES + 1];  // union of those queries' nearest-visited-ancestor sets
    uint32_t n_visit[EST_MAX_STAGES + 1];    // queries visiting the stage ([S] = n)
    uint32_t r_max[EST_MAX_STAGES];          // largest replica count per stage over all candidates
    uint32_t b_max[EST_MAX_STAGES];          // largest max-batch per stage over all candidates
    uint32_t bad_trace;                      // arrivals decrease somewhere
    uint32_t bad_cfg;                        // a configuration entry is out of range
    uint32_t last_arrival;
    uint32_t sim_error;                      // set by the simulation kernel on an inconsistency
    uint32_t next_cfg;                       // work counter: next candidate to hand to a free wavefront
    uint32_t pad;
};

struct EstStageCfg {  // same layout as est_stage_cfg_t
    uint8_t hw, batch;
    uint16_t replicas;
};

struct EstDag {
    uint32_t S, H, Bmax, pad;
    uint32_t parent_off[EST_MAX_STAGES + 2];   // [S+1]; entry S+1 closes the virtual sink's list
    uint32_t parent_idx[EST_MAX_STAGES * EST_MAX_STAGES / 2 + EST_MAX_STAGES];  // real parents, then the sinks
};

// Arguments of the simulation kernel.
struct EstSimArgs {
    const EstPlan *plan;
    const EstDag *dag;
    const uint32_t *lat_us;        // [S][H][Bmax]
    const uint64_t *cost_uusd_hr;  // [S][H]
    const uint32_t *arrival;       // [n]
    const uint64_t *trace_keys;    // [n] arrival << 32 | q
    const uint8_t *acc;            // [n_acc][n_pad] accept masks
    uint64_t acc_stride;           // n_pad
    const EstStageCfg *cfg;        // [n_cfg][S], already offset to the tile
    uint32_t n;                    // queries
    uint32_t n_cfg;                // candidates in this launch
    uint32_t slo_us;
    uint32_t lat_by_qid;           // 1: latencies indexed by query (checking mode)
    uint32_t max_src;              // widest merge of the plan (sizes the LDS)
    uint32_t lds_bytes;            // LDS per wavefront
    uint32_t n_slots;              // wavefronts that share the candidates of this launch, each with its own scratch
    uint32_t have_lat;             // 1: select P99 from the slot's latency array after each candidate
    // per-slot scratch, slot k at base + k * stride
    uint32_t *state;    uint64_t state_stride;   // words
    uint64_t *rings;    uint64_t ring_stride;    // elements
    uint32_t *rep;      uint64_t rep_stride;     // words
    uint32_t *slots;    uint64_t slot_stride;    // words
    uint8_t *tabs;      uint64_t tab_stride;     // bytes: the time tables of the merges that join several streams
    uint32_t *lat;      uint64_t lat_stride;     // words
    EstStatus *status;
    uint64_t *dbg_ticks;           // optional: [n_cfg] 100 MHz ticks each candidate took, then [n_cfg][EST_MAX_STAGES][8] counters (diagnostics)
    uint32_t *p99; uint32_t *miss; uint64_t *cost;   // [n_cfg] results
    // Shared upstream stages (Section 4.3: the candidates of one planner step differ from a common base
    // in one model, so everything upstream of the change is simulated once).  Only read by the kernel
    // variant launched when skip_ops is set.
    const uint64_t *skip_ops;      // [n_cfg]: bit i = operation i is not run for this candidate
    const uint32_t *base_of;       // [n_cfg]: whose captured streams stand in for the skipped producers (replay only)
    const EstPlan *cap_plan;       // layout of one captured candidate's streams
    const uint64_t *cap_rings;  uint64_t cap_ring_stride;    // elements; null = nothing is replayed (a capture launch)
    const uint32_t *cap_state;  uint64_t cap_state_stride;   // words
    uint32_t slot_by_cfg;          // 1: candidate t works in scratch slot t and its streams stay there (capture)
    uint32_t pad3;
    const uint32_t *order;         // optional [n_cfg]: the k-th candidate handed out is order[k] (longest first)
};

struct EstPrepArgs {
    const EstDag *dag;
    const uint32_t *arrival;
    const uint32_t *mask;
    uint32_t n;
    // pass 2
    uint64_t *trace_keys;
    uint8_t *acc; uint64_t acc_stride;
    uint32_t n_acc;
    uint32_t acc_stage[EST_MAX_STAGES + 1];               // stage (or S = sink) each accept array belongs to
    uint8_t acc_slot_of_src[EST_MAX_STAGES + 1][EST_TRACE_BIT + 1];  // source id -> slot bit, 0xFF = not a source
    EstStatus *status;
};

// Traffic envelope (Section 5): the largest number of arrivals inside any window of each width.
struct EstEnvArgs {
    const uint32_t *arrival;         // [n], non-decreasing
    uint64_t n;
    uint32_t n_win;
    uint64_t win_us[EST_MAX_WINDOWS];
    uint32_t *max_queries;           // [n_win], zero on entry
};

struct EstCfgArgs {
    const EstDag *dag;
    const EstStageCfg *cfg;
    uint64_t n_cfg;
    EstStatus *status;
};
